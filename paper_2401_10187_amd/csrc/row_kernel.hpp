// Every factor of a Kron-Matmul applied to a short row inside one launch, for any factor shapes.
//
// The fusion of section 4.2 needs equal-shaped factors because its tile is cut to P^N_fused
// elements.  When a whole row and every intermediate of it (Algorithm 1's Y^1, Y^2) fit LDS, the
// row itself is the tile and nothing has to be cut: a workgroup loads one row of X, applies factor
// N, N-1, ..., 1 by the rule of Algorithm 1 (slice s times column q goes to q*(K/P) + s) between two
// LDS buffers, and the last factor writes the row of Y.  Factor shapes are run-time values, so
// distinct and rectangular factors (the real-world sizes of Table 4: 52x50 with 65x20, 5x5 with
// 2x2 and 25x25) cost one launch instead of one per factor.  All factors are copied to LDS when
// the workgroup starts (one exposed memory latency for them and the first row together): their
// elements are read by every thread, and as LDS broadcasts they cost a fraction of what the same
// reads cost through the vector memory path.  Plain FMA code with a 2 x 4 register tile: this
// kernel is for launch-bound problems, and the planner prices it so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace km {

constexpr int ROW_MAXF = 8;                // factors per launch
constexpr int ROW_THREADS_MANY = 256;      // threads per row when there are many rows (eight rows per compute unit)
constexpr int ROW_THREADS_FEW = 1024;      // ... when there are few: sixteen wavefronts hide each other's latencies
constexpr int ROW_FEW_ROWS = 512;          // "few": at most two rows per compute unit
constexpr int ROW_SB = 2;                  // slices per thread
constexpr int ROW_QB = 4;                  // factor columns per thread
constexpr int ROW_LDS_LIMIT = 96 * 1024;   // row buffers and factors

// Row buffers skip one word in 33, so that reads P words apart (one slice per lane) spread over the
// banks also when P is a multiple of 32.
__host__ __device__ constexpr int row_pad(int e) { return e + (e >> 5); }

// LDS bytes for rows of at most max_width elements and factors of factor_elems elements together
__host__ __device__ constexpr int64_t row_lds_bytes(int64_t max_width, int64_t factor_elems, int esize)
{
    return (2 * (max_width + (max_width >> 5) + 1) + factor_elems) * esize;
}

struct RowFactors {
    const void* f[ROW_MAXF];               // in order of application (last factor of the product first)
    int P[ROW_MAXF], Q[ROW_MAXF];
    unsigned long long magic[ROW_MAXF];    // ceil(2^40 / slice blocks of the factor's step): u / blocks = (u * magic) >> 40
    int n;
};

template <typename T, int ROW_THREADS>
__global__ __launch_bounds__(ROW_THREADS)
void row_sliced_multiply(const T* __restrict__ Xg, T* __restrict__ Yg, const RowFactors fa,
                         int k_in, int k_out, int max_width, int64_t M)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char row_lds[];
    const int buf_elems = row_pad(max_width) + 1;
    T* buf0 = reinterpret_cast<T*>(row_lds);
    T* buf1 = buf0 + buf_elems;
    T* fbuf = buf1 + buf_elems;
    const int tid = threadIdx.x;

    // All factors (one after the other, in order of application) and the workgroup's first row are
    // fetched as one list of elements, so that their loads are in flight together: one memory
    // latency instead of one per factor.  The code is kept short on purpose (run-time loops, one
    // path for full and partial column blocks): for the small problems this kernel serves, fetching
    // instructions costs as much as executing them.
    // (Only the first ROW_HEAD_TRIPS trips of a long row are part of that list; the rest, and every
    // further row of the workgroup, is loaded four trips at a time, loads ahead of the LDS writes.)
    // Rows that are whole 16-byte vectors (they then start on 16-byte boundaries as X does) are loaded as such.
    typedef T RowVec __attribute__((ext_vector_type(16 / sizeof(T))));
    constexpr int VN = 16 / (int)sizeof(T);
    const bool vec_rows = k_in % VN == 0;
    auto load_row = [&](const T* src, int from) {
        if (vec_rows) {
            const int nv = k_in / VN;
            for (int v0 = from / VN + tid; v0 < nv; v0 += 4 * ROW_THREADS) {
                RowVec v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int vi = v0 + j * ROW_THREADS;
                    if (vi < nv) v[j] = reinterpret_cast<const RowVec*>(src)[vi];
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int vi = v0 + j * ROW_THREADS;
                    if (vi < nv)
#pragma unroll
                        for (int k = 0; k < VN; ++k) buf0[row_pad(vi * VN + k)] = v[j][k];
                }
            }
            return;
        }
        for (int e0 = from + tid; e0 < k_in; e0 += 4 * ROW_THREADS) {
            T v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int e = e0 + j * ROW_THREADS;
                v[j] = e < k_in ? src[e] : T(0);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int e = e0 + j * ROW_THREADS;
                if (e < k_in) buf0[row_pad(e)] = v[j];
            }
        }
    };
    constexpr int ROW_HEAD_TRIPS = 4;
    const int head = k_in < ROW_HEAD_TRIPS * ROW_THREADS ? k_in : ROW_HEAD_TRIPS * ROW_THREADS;
    int nf = 0;
    for (int i = 0; i < fa.n; ++i) nf += fa.P[i] * fa.Q[i];
    {
        const int total = nf + (blockIdx.x < M ? head : 0);
        const T* src = Xg + (int64_t)blockIdx.x * k_in;
        for (int idx = tid; idx < total; idx += ROW_THREADS) {
            const T* from = src;
            int off = idx - nf, first = 0;
            for (int i = 0; i < fa.n; ++i) {
                const int n = fa.P[i] * fa.Q[i];
                if (idx >= first && idx < first + n) { from = static_cast<const T*>(fa.f[i]); off = idx - first; }
                first += n;
            }
            const T v = from[off];
            if (idx < nf) fbuf[idx] = v;
            else buf0[row_pad(idx - nf)] = v;
        }
        if (blockIdx.x < M && head < k_in) load_row(src, head);
    }
    for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
        T* Yrow = Yg + row * k_out;
        if (row != blockIdx.x) {
            load_row(Xg + row * k_in, 0);
        }
        __syncthreads();                                 // the row (and, the first time, the factors) are in LDS
        T* cur = buf0;
        T* nxt = buf1;
        const T* fcur = fbuf;
        int K = k_in;
        for (int i = 0; i < fa.n; ++i) {
            const int P = fa.P[i], Q = fa.Q[i];
            const int S = K / P, L = S * Q;
            const bool last = i == fa.n - 1;
            // A thread takes ROW_SB slices (s_blocks apart, so that consecutive threads still take
            // consecutive slices) and ROW_QB consecutive columns; columns past Q are computed on
            // the last column's elements and dropped.
            const int s_blocks = (S + ROW_SB - 1) / ROW_SB;
            const int q_blocks = (Q + ROW_QB - 1) / ROW_QB;
            const int units = s_blocks * q_blocks;
            const unsigned long long magic = fa.magic[i];
            for (int u = tid; u < units; u += ROW_THREADS) {
                const int qb = (int)(((unsigned long long)u * magic) >> 40);     // u / s_blocks
                const int s0 = u - qb * s_blocks, q0 = qb * ROW_QB;
                int xs[ROW_SB], col[ROW_QB];
#pragma unroll
                for (int b = 0; b < ROW_SB; ++b) {
                    const int s = s0 + b * s_blocks;
                    xs[b] = (s < S ? s : 0) * P;
                }
#pragma unroll
                for (int k = 0; k < ROW_QB; ++k) col[k] = q0 + k < Q ? q0 + k : Q - 1;
                T acc[ROW_SB][ROW_QB];
#pragma unroll
                for (int b = 0; b < ROW_SB; ++b)
#pragma unroll
                    for (int k = 0; k < ROW_QB; ++k) acc[b][k] = T(0);
#pragma unroll 2
                for (int p = 0; p < P; ++p) {
                    T fv[ROW_QB];
#pragma unroll
                    for (int k = 0; k < ROW_QB; ++k) fv[k] = fcur[p * Q + col[k]];
#pragma unroll
                    for (int b = 0; b < ROW_SB; ++b) {
                        const T xv = cur[row_pad(xs[b] + p)];
#pragma unroll
                        for (int k = 0; k < ROW_QB; ++k) acc[b][k] += xv * fv[k];
                    }
                }
#pragma unroll
                for (int b = 0; b < ROW_SB; ++b)
#pragma unroll
                    for (int k = 0; k < ROW_QB; ++k)
                        if (s0 + b * s_blocks < S && q0 + k < Q) {
                            const int j = (q0 + k) * S + s0 + b * s_blocks;
                            if (last) Yrow[j] = acc[b][k];
                            else nxt[row_pad(j)] = acc[b][k];
                        }
            }
            __syncthreads();                             // `cur` is free again, `nxt` complete
            T* t = cur; cur = nxt; nxt = t;
            fcur += P * Q;
            K = L;
        }
    }
}

}  // namespace km
