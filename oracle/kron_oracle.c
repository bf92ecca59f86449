/*
 * CPU oracle for Kron-Matmul:  Y = X * (F_1 (x) F_2 (x) ... (x) F_N).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is judged against.  It shares no code, table or constant with
 * the HIP path and must never be called from it.
 *
 * Two independent computations live here:
 *
 *   kron_oracle_*      The sliced-multiply iteration of the paper's
 *                      Algorithm 1 (section "The FastKron Algorithm"), taken
 *                      step by step: for f = N..1, every length-P_f slice of a
 *                      row is contracted with every column of F_f and the
 *                      result for (slice s, column q) lands at output column
 *                      q*(K/P_f)+s.  Loops are 0-based; per-factor shapes
 *                      P_f x Q_f generalise the equal-shape listing.
 *
 *   kron_bruteforce_*  The definition (section 2, block form of the Kronecker
 *                      product): G is built by repeated two-factor products
 *                      G = A (x) B with G[(ia*Pb+ib)][(ja*Qb+jb)] = A[ia][ja]*B[ib][jb]
 *                      and Y = X*G by a triple loop.  Tiny sizes only.
 *
 * All matrices are row-major.  X is M x prod(P), F_f is P_f x Q_f, Y is
 * M x prod(Q).  F[0] is the leftmost factor (slowest index digit).
 *
 * Precision: fp32 problems accumulate and carry intermediates in double;
 * fp64 problems in long double (x87 80-bit here).  The result is rounded to
 * the I/O type once, at the end.
 *
 * Rows are independent; OpenMP threads split the rows.  Return value is 0 on
 * success, non-zero on invalid arguments or allocation failure.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int kron_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* widest row any iteration produces or consumes */
static int64_t max_width(int N, const int *P, const int *Q, int64_t *k_in, int64_t *k_out)
{
    int64_t K = 1, L = 1, w, cur;
    for (int f = 0; f < N; ++f) { K *= P[f]; L *= Q[f]; }
    *k_in = K; *k_out = L;
    w = K; cur = K;
    for (int f = N - 1; f >= 0; --f) {
        cur = cur / P[f] * Q[f];
        if (cur > w) w = cur;
    }
    return w;
}

static int check_shapes(int64_t M, int N, const int *P, const int *Q)
{
    if (M < 0 || N < 1 || !P || !Q) return 1;
    for (int f = 0; f < N; ++f) if (P[f] < 1 || Q[f] < 1) return 1;
    return 0;
}

#define DEFINE_ORACLE(NAME, IO_T, ACC_T)                                            \
int NAME(int64_t M, int N, const int *P, const int *Q,                              \
         const IO_T *X, const IO_T *const *F, IO_T *Y)                              \
{                                                                                   \
    int64_t K0, L0, W;                                                              \
    int fail = 0;                                                                   \
    if (check_shapes(M, N, P, Q) || !F) return 1;                                   \
    W = max_width(N, P, Q, &K0, &L0);                                               \
    if (M == 0) return 0;                                                           \
    if (!X || !Y) return 1;                                                         \
    _Pragma("omp parallel")                                                         \
    {                                                                               \
        ACC_T *cur = (ACC_T *)malloc((size_t)W * sizeof(ACC_T));                    \
        ACC_T *nxt = (ACC_T *)malloc((size_t)W * sizeof(ACC_T));                    \
        if (!cur || !nxt) {                                                         \
            _Pragma("omp atomic write")                                             \
            fail = 1;                                                               \
        }                                                                           \
        _Pragma("omp barrier")                                                      \
        if (!fail) {                                                                \
            _Pragma("omp for schedule(dynamic, 1)")                                 \
            for (int64_t i = 0; i < M; ++i) {                                       \
                int64_t K = K0;                                                     \
                for (int64_t c = 0; c < K0; ++c) cur[c] = (ACC_T)X[i * K0 + c];     \
                for (int f = N - 1; f >= 0; --f) {      /* last factor first */     \
                    const IO_T *Ff = F[f];                                          \
                    const int64_t Pf = P[f], Qf = Q[f];                             \
                    const int64_t S = K / Pf;           /* slices in the row  */    \
                    const int64_t L = S * Qf;           /* output width       */    \
                    for (int64_t j = 0; j < L; ++j) {                               \
                        const int64_t s = j % S;        /* which slice        */    \
                        const int64_t q = j / S;        /* which F column     */    \
                        ACC_T acc = 0;                                              \
                        for (int64_t p = 0; p < Pf; ++p)                            \
                            acc += cur[s * Pf + p] * (ACC_T)Ff[p * Qf + q];         \
                        nxt[j] = acc;                                               \
                    }                                                               \
                    { ACC_T *t = cur; cur = nxt; nxt = t; }                         \
                    K = L;                                                          \
                }                                                                   \
                for (int64_t c = 0; c < L0; ++c) Y[i * L0 + c] = (IO_T)cur[c];      \
            }                                                                       \
        }                                                                           \
        free(cur); free(nxt);                                                       \
    }                                                                               \
    return fail ? 2 : 0;                                                            \
}

DEFINE_ORACLE(kron_oracle_f32, float, double)
DEFINE_ORACLE(kron_oracle_f64, double, long double)

/* One sliced-multiply iteration on its own (Algorithm 1, body of the loop over
 * f): Yout (M x (K/P)*Q) from Yin (M x K) and one factor.  Rounded to the I/O
 * type, so chaining these rounds every intermediate, unlike kron_oracle_*. */
#define DEFINE_STEP(NAME, IO_T, ACC_T)                                              \
int NAME(int64_t M, int64_t K, int P, int Q,                                        \
         const IO_T *Yin, const IO_T *Ff, IO_T *Yout)                               \
{                                                                                   \
    if (M < 0 || K < 0 || P < 1 || Q < 1 || K % P) return 1;                        \
    const int64_t S = K / P, L = S * Q;                                             \
    _Pragma("omp parallel for schedule(static)")                                    \
    for (int64_t i = 0; i < M; ++i)                                                 \
        for (int64_t j = 0; j < L; ++j) {                                           \
            const int64_t s = j % S, q = j / S;                                     \
            ACC_T acc = 0;                                                          \
            for (int64_t p = 0; p < P; ++p)                                         \
                acc += (ACC_T)Yin[i * K + s * P + p] * (ACC_T)Ff[p * (int64_t)Q + q]; \
            Yout[i * L + j] = (IO_T)acc;                                            \
        }                                                                           \
    return 0;                                                                       \
}

DEFINE_STEP(kron_sliced_multiply_f32, float, double)
DEFINE_STEP(kron_sliced_multiply_f64, double, long double)

/* Definition-level brute force.  G is materialised (prod(P) x prod(Q) long
 * doubles), so the caller keeps prod(P)*prod(Q) small. */
#define DEFINE_BRUTE(NAME, IO_T)                                                    \
int NAME(int64_t M, int N, const int *P, const int *Q,                              \
         const IO_T *X, const IO_T *const *F, IO_T *Y)                              \
{                                                                                   \
    int64_t K0, L0;                                                                 \
    if (check_shapes(M, N, P, Q) || !F) return 1;                                   \
    (void)max_width(N, P, Q, &K0, &L0);                                             \
    if (K0 * L0 > ((int64_t)1 << 26)) return 3;                                     \
    if (M == 0) return 0;                                                           \
    if (!X || !Y) return 1;                                                         \
    /* G starts as F_1 and absorbs one factor at a time on its right */            \
    int64_t gr = P[0], gc = Q[0];                                                   \
    long double *G = (long double *)malloc((size_t)(gr * gc) * sizeof(long double));\
    if (!G) return 2;                                                               \
    for (int64_t e = 0; e < gr * gc; ++e) G[e] = (long double)F[0][e];              \
    for (int f = 1; f < N; ++f) {                                                   \
        const int64_t pb = P[f], qb = Q[f];                                         \
        const int64_t nr = gr * pb, nc = gc * qb;                                   \
        long double *H = (long double *)malloc((size_t)(nr * nc) * sizeof(long double)); \
        if (!H) { free(G); return 2; }                                              \
        for (int64_t ia = 0; ia < gr; ++ia)                                         \
            for (int64_t ja = 0; ja < gc; ++ja)                                     \
                for (int64_t ib = 0; ib < pb; ++ib)                                 \
                    for (int64_t jb = 0; jb < qb; ++jb)                             \
                        H[(ia * pb + ib) * nc + (ja * qb + jb)] =                   \
                            G[ia * gc + ja] * (long double)F[f][ib * qb + jb];      \
        free(G); G = H; gr = nr; gc = nc;                                           \
    }                                                                               \
    for (int64_t i = 0; i < M; ++i)                                                 \
        for (int64_t j = 0; j < L0; ++j) {                                          \
            long double acc = 0;                                                    \
            for (int64_t k = 0; k < K0; ++k)                                        \
                acc += (long double)X[i * K0 + k] * G[k * L0 + j];                  \
            Y[i * L0 + j] = (IO_T)acc;                                              \
        }                                                                           \
    free(G);                                                                        \
    return 0;                                                                       \
}

DEFINE_BRUTE(kron_bruteforce_f32, float)
DEFINE_BRUTE(kron_bruteforce_f64, double)
