// Fused sliced multiplies for small factors (P, Q <= 12): several factors per LDS pass.
//
// Same tile and same final scatter as fused_kernel.hpp (section 4.2 of the paper), but a thread
// now owns a group of P^G contiguous elements and applies G factors to it entirely in registers
// before anything goes back to LDS.  Applying the sliced-multiply rule of Algorithm 1 G times to the
// P^G elements seen as a tiny row gives them the order (q_1, ..., q_G), i.e. exactly the column
// index qq of the G-factor group, so the LDS write of a "super-stage" is the ordinary rule with
// Q^G columns: (group s, column qq) -> qq*S + s.  With P = 2 three factors cost one LDS round trip
// instead of three; with P = 4 two factors do.
//
// Up to three super-stages (G0, G1, G2 factors; 0 = unused) per launch.  Nothing in the rule needs
// the stages to share a factor shape: stage j has its own (Pj, Qj), so neighbouring runs of different
// small shapes (2x2 beside 4x4, 5x5 beside 2x2) are one launch too; within a stage the factors are
// equal-shaped.  Factor elements are read
// with scalar loads, as in fused_kernel.hpp.  LDS rows (one group each) are padded when their
// length is an even number of 16-byte units above two, which would otherwise put the 16-byte reads
// of eight consecutive lanes into the same banks.
//
// A tile is a stretch of one row, or, for problems with many short rows, several whole rows (the
// T_M of section 4): rows are contiguous in memory and pass through the stages as one long tile.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "fused_kernel.hpp"   // ipow, Vec16, as_constant, stream_load/stream_store
#include "plan.hpp"           // unaligned_vectors

namespace km {

template <int N> struct FactorPtrs { const void* f[N]; };

// STMAX bounds the tile (LDS, registers, unrolled trip counts); the number of slices actually in a
// tile, st <= STMAX, is a launch parameter so that one instance serves every row length whose
// K/P^NF has a divisor in range (rows of 3^7 or 6^7 elements, M = 1 problems, ...).
// (A fourth super-stage, G3 factors of the third stage's shape, serves rows of P^4 elements that fit
// LDS whole: one launch instead of two.)
template <typename T_, int P0, int Q0, int G0, int P1, int Q1, int G1, int P2, int Q2, int G2, int STMAX_, int NT_, int G3 = 0>
struct MixedShape {
    typedef T_ T;
    static constexpr int STMAX = STMAX_, NT = NT_;
    static constexpr int NS = (G0 > 0) + (G1 > 0) + (G2 > 0) + (G3 > 0);
    static constexpr int NF = G0 + G1 + G2 + G3;
    static constexpr int VN = Vec16<T>::N;
    static constexpr int g(int j) { return j == 0 ? G0 : (j == 1 ? G1 : (j == 2 ? G2 : G3)); }
    static constexpr int p(int j) { return j == 0 ? P0 : (j == 1 ? P1 : P2); }      // factor shape of stage j
    static constexpr int q(int j) { return j == 0 ? Q0 : (j == 1 ? Q1 : Q2); }
    static constexpr int done(int j) { return (j > 0 ? G0 : 0) + (j > 1 ? G1 : 0) + (j > 2 ? G2 : 0); }
    static constexpr int pg(int j) { return (int)ipow(p(j), g(j)); }      // elements a thread reads per group
    static constexpr int qg(int j) { return (int)ipow(q(j), g(j)); }      // elements it produces
    static constexpr int qdone(int j) { return (j > 0 ? qg(0) : 1) * (j > 1 ? qg(1) : 1) * (j > 2 ? qg(2) : 1); }   // columns of the stages before j
    static constexpr int ptodo(int j) { return (j <= 0 ? pg(0) : 1) * (j <= 1 ? pg(1) : 1) * (j <= 2 ? pg(2) : 1) * (j <= 3 ? pg(3) : 1); } // elements per slice still to contract
    static constexpr int per_slice(int j) { return ptodo(j) * qdone(j); }   // tile elements per unit of st
    static constexpr int wmax(int j) { return (int)ipow(p(j) > q(j) ? p(j) : q(j), g(j)); }
    static constexpr int qchunk(int j)  // columns of one factor whose elements fit 64 scalar registers
    {
        int c = q(j);
        while (c > 1 && (p(j) * c * (int)sizeof(T)) / 4 > 64) {
            --c;
            while (c > 1 && q(j) % c) --c;
        }
        return c;
    }
    static constexpr int pad(int j)
    {
        const int bytes = pg(j) * (int)sizeof(T);
        if (bytes % 16) return 0;
        const int units = bytes / 16;
        return (units % 2 == 0 && units > 2) ? VN : 0;
    }
    static constexpr int rows_per_slice(int j) { return per_slice(j) / pg(j); }     // groups per unit of st
    static constexpr int max_rows(int j) { return STMAX * rows_per_slice(j); }
    static constexpr int lds_elems()
    {
        int m = 0;
        for (int j = 0; j < NS; ++j) {
            const int e = max_rows(j) * (pg(j) + pad(j));
            m = e > m ? e : m;
        }
        return m;
    }
    // every stage's groups have odd length: nothing reads LDS in 16-byte vectors
    static constexpr bool ALL_ODD = P0 % 2 == 1 && (G1 == 0 || P1 % 2 == 1) && (G2 == 0 || P2 % 2 == 1);
    // 32 bytes of slack where a tile that starts off a 16-byte boundary is held shifted by up to VN - 1
    // elements (odd P only; tiles of exactly 64 KB must not grow: two of them no longer share a compute unit)
    static constexpr int LDS_SLACK = ALL_ODD ? 32 : 0;
    static constexpr int LDS_BYTES = (lds_elems() * (int)sizeof(T) + 15) / 16 * 16 + LDS_SLACK;
    // the tile only occupies what its st slices need, so short tiles leave LDS to more workgroups
    static constexpr int LDS_PER_SLICE = lds_elems() / STMAX * (int)sizeof(T);
    static constexpr bool VEC_ROWS = pg(0) % VN == 0;
    static_assert(G0 > 0 && (G1 > 0 || G2 == 0) && (G2 > 0 || G3 == 0), "super-stages are filled from the first");
};

// every stage with the same factor shape
template <typename T, int P, int Q, int G0, int G1, int G2, int STMAX, int NT, int G3 = 0>
using MultiShape = MixedShape<T, P, Q, G0, P, Q, G1, P, Q, G2, STMAX, NT, G3>;

// (KEEP: ordinary instead of non-temporal stores, for output the next launch reads back out of the
// last-level cache; see out_store.)
// Tiles of whole rows: the final stage leaves the tile's output rows in LDS, unpadded and in
// memory order (they are contiguous in Y), and this writes them out with contiguous stores.
template <typename T, int NT, bool KEEP>
__device__ __forceinline__ void multi_store_rows(const T* __restrict__ tile, T* __restrict__ dst, int n, bool vec_ok)
{
    typedef typename Vec16<T>::type V;
    constexpr int VN = Vec16<T>::N, UN = 4;
    const int tid = threadIdx.x;
    if (vec_ok) {
        const int nv = n / VN;
        for (int base = 0; base < nv; base += UN * NT) {
            V tmp[UN];
#pragma unroll
            for (int i = 0; i < UN; ++i) {
                const int v = base + tid + i * NT;
                if (v < nv) tmp[i] = reinterpret_cast<const V*>(tile)[v];
            }
#pragma unroll
            for (int i = 0; i < UN; ++i) {
                const int v = base + tid + i * NT;
                if (v < nv) out_store<KEEP>(tmp[i], &reinterpret_cast<V*>(dst)[v]);
            }
        }
    } else {
        for (int base = 0; base < n; base += UN * NT) {
#pragma unroll
            for (int i = 0; i < UN; ++i) {
                const int e = base + tid + i * NT;
                if (e < n) out_store<KEEP>(tile[e], &dst[e]);
            }
        }
    }
}

// position in LDS of flat tile index c when rows of `PGN` elements are padded by `PADN`
template <int PGN, int PADN>
__device__ __forceinline__ int multi_lds_index(int c) { return PADN == 0 ? c : c + (c / PGN) * PADN; }

template <class Sh, int J, bool KEEP>
__device__ __forceinline__ void multi_stage(typename Sh::T* __restrict__ tile, const FactorPtrs<Sh::NF>& fp,
                                            typename Sh::T* __restrict__ Yrow, int64_t s_row, int64_t h, int st,
                                            int sr_tile, int64_t k_out, int rows_here, int tile_rows)
{
    typedef typename Sh::T T;
    typedef typename Vec16<T>::type V;
    constexpr int VN = Sh::VN, NT = Sh::NT, P = Sh::p(J), Q = Sh::q(J);
    constexpr int GJ = Sh::g(J), PGJ = Sh::pg(J), QGJ = Sh::qg(J), PADJ = Sh::pad(J), WMAX = Sh::wmax(J);
    constexpr int R = (Sh::max_rows(J) + NT - 1) / NT;
    constexpr bool LAST = J == Sh::NS - 1;
    const int SJ = st * Sh::rows_per_slice(J);           // groups in the tile at this super-stage
    const int tid = threadIdx.x;

    T out[R][QGJ];
    if constexpr (GJ == 1 && (P * Q * (int)sizeof(T)) / 4 > 64) {
        // One factor whose elements do not fit the scalar registers at once (8x8 doubles): take its
        // columns in chunks that do, and run every slice of the thread against one chunk before the
        // next chunk is fetched.
        constexpr int QCH = Sh::qchunk(J);
        T xs[R][P];
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int s = tid + i * NT;
            if (s < SJ) {
                const T* src = tile + s * (PGJ + PADJ);
                if constexpr ((PGJ * sizeof(T)) % 16 == 0) {
#pragma unroll
                    for (int c = 0; c < PGJ / VN; ++c) {
                        const V v = reinterpret_cast<const V*>(src)[c];
#pragma unroll
                        for (int e = 0; e < VN; ++e) xs[i][VN * c + e] = v[e];
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < PGJ; ++e) xs[i][e] = src[e];
                }
            } else {
#pragma unroll
                for (int e = 0; e < PGJ; ++e) xs[i][e] = T(0);
            }
        }
        // Results go straight to their destination, one chunk of columns per trip of a loop that is
        // deliberately not unrolled (unrolled, all of the factor would be fetched up front again).
        const auto Fc = as_constant(static_cast<const T*>(fp.f[Sh::done(J)]));
        if (!LAST || tile_rows > 1) __syncthreads();     // every slice has been read
        constexpr int QREST1 = Sh::qdone(J);
#pragma unroll 1
        for (int q0 = 0; q0 < Q; q0 += QCH) {
#pragma unroll
            for (int i = 0; i < R; ++i) {
                const int s = tid + i * NT;
#pragma unroll
                for (int qq = 0; qq < QCH; ++qq) {
                    const int q = q0 + qq;
                    T acc = xs[i][0] * Fc[q];
#pragma unroll
                    for (int p = 1; p < P; ++p) acc += xs[i][p] * Fc[p * Q + q];
                    if (s < SJ) {
                        if constexpr (!LAST) {
                            constexpr int PGN1 = Sh::pg(J + 1 < Sh::NS ? J + 1 : J), PADN1 = Sh::pad(J + 1 < Sh::NS ? J + 1 : J);
                            tile[multi_lds_index<PGN1, PADN1>(q * SJ + s)] = acc;
                        } else {
                            const int m = (s % st) / sr_tile;        // row of the tile (0 unless it holds whole rows)
                            const int64_t at = m * k_out + (int64_t)(s / st + q * QREST1) * s_row + h * sr_tile + (s % st) % sr_tile;
                            if (tile_rows > 1) tile[at] = acc;       // whole rows: collected in LDS, stored below
                            else out_store<KEEP>(acc, &Yrow[at]);
                        }
                    }
                }
            }
        }
        if (!LAST || tile_rows > 1) __syncthreads();
        if constexpr (LAST) {
            if (tile_rows > 1) multi_store_rows<T, NT, KEEP>(tile, Yrow, (int)(rows_here * k_out), k_out % VN == 0);
        }
        return;
    } else {
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int s = tid + i * NT;
        T x[WMAX], y[WMAX];
        if (s < SJ) {
            const T* src = tile + s * (PGJ + PADJ);
            if constexpr ((PGJ * sizeof(T)) % 16 == 0) {
#pragma unroll
                for (int c = 0; c < PGJ / VN; ++c) {
                    const V v = reinterpret_cast<const V*>(src)[c];
#pragma unroll
                    for (int e = 0; e < VN; ++e) x[VN * c + e] = v[e];
                }
            } else {
#pragma unroll
                for (int e = 0; e < PGJ; ++e) x[e] = src[e];
            }
        } else {
#pragma unroll
            for (int e = 0; e < PGJ; ++e) x[e] = T(0);
        }
        // G factors in registers: the rule of Algorithm 1 on a row of W = P^(G-gi) * Q^gi elements
#pragma unroll
        for (int gi = 0; gi < GJ; ++gi) {
            const auto Fc = as_constant(static_cast<const T*>(fp.f[Sh::done(J) + gi]));
            const int W = (int)(ipow(P, GJ - gi) * ipow(Q, gi));
            const int S = W / P;
#pragma unroll
            for (int sp = 0; sp < S; ++sp)
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    T acc = x[sp * P] * Fc[q];
#pragma unroll
                    for (int p = 1; p < P; ++p) acc += x[sp * P + p] * Fc[p * Q + q];
                    y[q * S + sp] = acc;
                }
#pragma unroll
            for (int e = 0; e < S * Q; ++e) x[e] = y[e];
        }
#pragma unroll
        for (int qq = 0; qq < QGJ; ++qq) out[i][qq] = x[qq];
    }
    }
    if constexpr (!LAST) {
        constexpr int PGN = Sh::pg(J + 1), PADN = Sh::pad(J + 1);
        __syncthreads();                                 // every group has been read
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int s = tid + i * NT;
            if (s < SJ) {
#pragma unroll
                for (int qq = 0; qq < QGJ; ++qq) tile[multi_lds_index<PGN, PADN>(qq * SJ + s)] = out[i][qq];
            }
        }
        __syncthreads();
    } else {
        if (tile_rows > 1) __syncthreads();              // every group has been read; LDS is reused for the rows
        // local (qq, s) with s = qrest*st + r  ->  column (qq*QREST + qrest)*s_row + h*st + r, QREST the
        // columns of the earlier stages; when the
        // tile holds several whole rows, r = m*s_row + r' and the element belongs to row m of the tile
        constexpr int QREST = Sh::qdone(J);
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int s = tid + i * NT;
            if (s < SJ) {
                const int m = (s % st) / sr_tile;            // row of the tile (0 unless it holds whole rows)
                const int64_t at = m * k_out + (int64_t)(s / st) * s_row + h * sr_tile + (s % st) % sr_tile;
                if (tile_rows > 1) {                         // whole rows: collected in LDS, stored below
#pragma unroll
                    for (int qq = 0; qq < QGJ; ++qq) tile[at + (int64_t)(qq * QREST) * s_row] = out[i][qq];
                } else {
#pragma unroll
                    for (int qq = 0; qq < QGJ; ++qq) out_store<KEEP>(out[i][qq], &Yrow[at + (int64_t)(qq * QREST) * s_row]);
                }
            }
        }
        if (tile_rows > 1) {
            __syncthreads();
            multi_store_rows<T, NT, KEEP>(tile, Yrow, (int)(rows_here * k_out), k_out % VN == 0);
        }
    }
}

template <class Sh, bool KEEP>
__global__ __launch_bounds__(Sh::NT)
void fused_multi_sliced_multiply(const typename Sh::T* __restrict__ Xg, typename Sh::T* __restrict__ Yg,
                                 const FactorPtrs<Sh::NF> fp,           // in order of application
                                 int64_t k_in, int64_t k_out, int64_t tiles_per_row, int64_t num_tiles, int st,
                                 int tile_rows, int64_t M)
{
    typedef typename Sh::T T;
    typedef typename Vec16<T>::type V;
    constexpr int VN = Sh::VN, NT = Sh::NT, STMAX = Sh::STMAX;
    extern __shared__ __attribute__((aligned(16))) unsigned char multi_lds[];
    T* tile = reinterpret_cast<T*>(multi_lds);           // (moved up by a few elements below for unaligned tiles)

    const int64_t t = xcd_contiguous_tile(blockIdx.x, num_tiles);
    // A tile is `st` slices: a stretch of one row (tile_rows == 1), or tile_rows whole rows, which are
    // contiguous in memory and go through the stages as one long tile; only the final store tells
    // the rows apart.
    const int64_t row = (t / tiles_per_row) * tile_rows;
    const int64_t h = t % tiles_per_row;
    const int sr_tile = st / tile_rows;                  // slices of one row inside the tile
    const int rows_here = (int)(M - row < tile_rows ? M - row : tile_rows);
    const int tk = st * Sh::per_slice(0);                // elements in a full tile
    const int valid = tile_rows > 1 ? (int)(rows_here * k_in) : tk;     // ... that exist (last tile of whole rows)
    const T* src = Xg + row * k_in + h * tk;
    T* Yrow = Yg + row * k_out;
    const int64_t s_row = tiles_per_row * sr_tile;
    const int tid = threadIdx.x;
    constexpr int PG0 = Sh::pg(0), PAD0 = Sh::pad(0);

    // 16-byte loads need every tile to start on a 16-byte boundary and rows of whole vectors
    if (Sh::VEC_ROWS && tk % VN == 0 && k_in % VN == 0) {
        const int nv = valid / VN;
        constexpr int RV = (STMAX * Sh::per_slice(0) / VN + NT - 1) / NT;
        V tmp[RV];
#pragma unroll
        for (int i = 0; i < RV; ++i) {
            const int v = tid + i * NT;
            if (v < nv) tmp[i] = stream_load(&reinterpret_cast<const V*>(src)[v]);
        }
#pragma unroll
        for (int i = 0; i < RV; ++i) {
            const int v = tid + i * NT;
            if (v < nv) *reinterpret_cast<V*>(tile + multi_lds_index<PG0, PAD0>(v * VN)) = tmp[i];
        }
    } else {
        // Tiles that do not start on a 16-byte boundary (rows of odd length): 16-byte loads from the
        // boundary below the tile, so the first vector may hold up to VN - 1 elements of the tile
        // before, which are dropped.  Below the tile there always is one when mis > 0 (X itself starts
        // on a 16-byte boundary); above it there need not be (the last tile of X), so a last vector
        // that is only partly the tile's is fetched element by element: nothing outside
        // [src - mis, src + valid) is read.
        const int mis = (int)((reinterpret_cast<uintptr_t>(src) / sizeof(T)) % VN);
        const V* vsrc = reinterpret_cast<const V*>(src - mis);
        const int nv = unaligned_vectors(valid, mis, VN), nfull = unaligned_whole_vectors(valid, mis, VN);
        constexpr int UN = 4;
        // With odd P nothing downstream reads LDS in vectors (every group length is odd) and no row is
        // padded, so the tile may sit in LDS shifted by `mis` elements: vector v of global memory then is
        // vector v of LDS and goes in with one 16-byte write, foreign elements at both ends included
        // (they fall outside the tile and are never read).  Otherwise the elements are placed one by one.
        constexpr bool SHIFT = Sh::ALL_ODD && PAD0 == 0;
        if constexpr (SHIFT) tile += mis;
        for (int base = 0; base < nfull; base += UN * NT) {
            V tmp[UN];
#pragma unroll
            for (int i = 0; i < UN; ++i) {
                const int v = base + tid + i * NT;
                if (v < nfull) tmp[i] = stream_load(&vsrc[v]);
            }
#pragma unroll
            for (int i = 0; i < UN; ++i) {
                const int v = base + tid + i * NT;
                if (v < nfull) {
                    if constexpr (SHIFT) {
                        reinterpret_cast<V*>(multi_lds)[v] = tmp[i];
                    } else {
#pragma unroll
                        for (int k = 0; k < VN; ++k) {
                            const int e = v * VN + k - mis;
                            if (e >= 0 && e < valid) tile[multi_lds_index<PG0, PAD0>(e)] = tmp[i][k];
                        }
                    }
                }
            }
        }
        if (nfull < nv && tid == NT - 1) {               // the tile's share of the last, partial vector
            for (int e = nfull * VN - mis < 0 ? 0 : nfull * VN - mis; e < valid; ++e) tile[multi_lds_index<PG0, PAD0>(e)] = src[e];
        }
    }
    __syncthreads();

    multi_stage<Sh, 0, KEEP>(tile, fp, Yrow, s_row, h, st, sr_tile, k_out, rows_here, tile_rows);
    if constexpr (Sh::NS > 1) multi_stage<Sh, 1, KEEP>(tile, fp, Yrow, s_row, h, st, sr_tile, k_out, rows_here, tile_rows);
    if constexpr (Sh::NS > 2) multi_stage<Sh, 2, KEEP>(tile, fp, Yrow, s_row, h, st, sr_tile, k_out, rows_here, tile_rows);
    if constexpr (Sh::NS > 3) multi_stage<Sh, 3, KEEP>(tile, fp, Yrow, s_row, h, st, sr_tile, k_out, rows_here, tile_rows);
}

}  // namespace km
