// Sliced multiplies on the matrix cores (MFMA), for factors whose P and Q are multiples of the MFMA
// block: the contraction of a slice with the factor (Algorithm 1's inner loop) is a dense product
//     D[q][s] = sum_p F[p][q] * X[s*P + p]            (Q x S) = F^T (Q x P) * Xslices^T (P x S)
// The factor is the A operand and stays in registers; slices are the B operand, so the lane
// dimension of the accumulator runs along the slice index and one accumulator register of a
// wavefront is a contiguous run of the output row (output column of (s, q) is q*(K/P)+s).
//
// The MFMA contraction index is split over lane groups (KG groups) and over issue steps.  Which
// element p a (group, step) pair stands for is free as long as A and B agree, so group g takes the
// contiguous range p in [g*P/KG, (g+1)*P/KG): every lane reads one contiguous piece of its slice
// from LDS with 16-byte reads.  LDS rows (one slice each) are padded so that eight consecutive
// lanes of such a read fall into different banks.
//
// A workgroup walks over `tiles_per_wg` consecutive tiles.  A tile is ST*P^NF contiguous elements of
// one row; NF = 1 or 2 factors are applied with the intermediate kept in LDS (section 4.2) and the
// result is scattered exactly as in the non-MFMA fused kernel.  The next tile is fetched from
// global memory into registers while the current one is being multiplied.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "fused_kernel.hpp"   // ipow, Vec16

namespace km {

typedef float mfma_f32x4 __attribute__((ext_vector_type(4)));
typedef float mfma_f32x16 __attribute__((ext_vector_type(16)));
typedef double mfma_f64x4 __attribute__((ext_vector_type(4)));

// v_mfma_f32_32x32x2_f32: A is 32x2, B is 2x32; lane l holds A[l%32][l/32], B[l/32][l%32];
// accumulator register v of lane l is D[8*(v/4) + 4*(l/32) + v%4][l%32]
// (row = row_lane(l) + row_reg(v)).
struct MfmaF32x32 {
    typedef float T;
    typedef mfma_f32x16 Acc;
    static constexpr int MB = 32, NB = 32, KG = 2, NACC = 16;
    static constexpr bool JOIN_BLOCKS = false;         // a register is already a 128-byte run of the output row
    static __device__ __forceinline__ int row_lane(int lane) { return 4 * (lane / 32); }
    static constexpr int row_reg(int v) { return 8 * (v / 4) + (v % 4); }
    static __device__ __forceinline__ Acc mma(float a, float b, Acc c) { return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0); }
};
// v_mfma_f32_16x16x4_f32: lane l holds A[l%16][l/16], B[l/16][l%16]; register v is D[4*(l/16) + v][l%16].
// A register holds four 64-byte runs of the output row.  Two neighbouring slice blocks are joined
// into 128-byte runs before the store (join_blocks below) where the tile allows it.
struct MfmaF32x16 {
    typedef float T;
    typedef mfma_f32x4 Acc;
    static constexpr int MB = 16, NB = 16, KG = 4, NACC = 4;
    static constexpr bool JOIN_BLOCKS = true;
    static __device__ __forceinline__ int row_lane(int lane) { return 4 * (lane / 16); }
    static constexpr int row_reg(int v) { return v; }
    static __device__ __forceinline__ Acc mma(float a, float b, Acc c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }
};
// v_mfma_f64_16x16x4_f64: same operand layout; register v is D[4*v + l/16][l%16].
struct MfmaF64x16 {
    typedef double T;
    typedef mfma_f64x4 Acc;
    static constexpr int MB = 16, NB = 16, KG = 4, NACC = 4;
    static constexpr bool JOIN_BLOCKS = false;         // 16 doubles are a 128-byte run
    static __device__ __forceinline__ int row_lane(int lane) { return lane / 16; }
    static constexpr int row_reg(int v) { return 4 * v; }
    static __device__ __forceinline__ Acc mma(double a, double b, Acc c) { return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0); }
};

// Registers x and y of the 16x16 fp32 accumulators of slice blocks 2k and 2k+1 (same register
// index v): afterwards lane l of x holds row 8*(l/32) + v, slice 32k + l%32, and lane l of y holds
// row 8*(l/32) + 4 + v of the same slice, so each half of a wavefront stores one 128-byte run.
// (v_permlane16_swap exchanges the odd 16-lane groups of x with the even ones of y.)
template <class Acc>
__device__ __forceinline__ void join_blocks(Acc& x, Acc& y, int v)
{
    const float xv = x[v], yv = y[v];
    const auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, xv), __builtin_bit_cast(unsigned, yv), false, false);
    x[v] = __builtin_bit_cast(float, (unsigned)r[0]);
    y[v] = __builtin_bit_cast(float, (unsigned)r[1]);
}

// NW wavefronts per workgroup; the factor's column blocks are dealt to QSPLIT wave groups and the
// slice blocks of a stage to the NW/QSPLIT wave groups along the other axis.
template <class OP, int P, int Q, int NF, int ST, int NW, int QSPLIT>
struct MfmaShape {
    typedef typename OP::T T;
    static constexpr int NT = NW * 64;
    static constexpr int PL = P / OP::KG;              // slice elements per lane
    static constexpr int QT = Q / OP::MB;              // column blocks of the factor
    static constexpr int QTW = QT / QSPLIT;            // ... per wavefront
    static constexpr int SG = NW / QSPLIT;             // wave groups along the slice axis
    static constexpr int VN = Vec16<T>::N;
    static constexpr int UNITS = P * (int)sizeof(T) / 16;                  // 16-byte units per slice
    static constexpr int PAD = (UNITS % 2 == 0 && UNITS != 2) ? VN : 0;    // make the row stride odd in units
    static constexpr int RS = P + PAD;                 // LDS row stride in elements
    static constexpr int size(int j) { return (int)(ST * ipow(P, NF - j) * ipow(Q, j)); }
    static constexpr int TK = size(0);
    static constexpr int lds_elems()
    {
        int m = 0;
        for (int j = 0; j < NF; ++j) m = size(j) / P * RS > m ? size(j) / P * RS : m;
        return m;
    }
    static constexpr int BUF_ELEMS = lds_elems();
    // Single factors stream through two tile buffers, except when the factor is split over the
    // wavefronts (large factors, MFMA-bound): there one buffer measured slightly faster.
    static constexpr int NBUF = (NF == 1 && QSPLIT == 1) ? 2 : 1;
    static constexpr int LDS_BYTES = NBUF * BUF_ELEMS * (int)sizeof(T);
    static constexpr int RV = TK / VN / NT;            // 16-byte vectors of a tile per thread
    // Slice block number `bi` of wave group `ws` out of `bpw` per group.  Joined stores need a
    // wavefront to own blocks 2k and 2k+1; otherwise the blocks are dealt round-robin.
    static constexpr bool joined(int bpw) { return OP::JOIN_BLOCKS && ST % (2 * OP::NB) == 0 && bpw % 2 == 0; }
    static __device__ __forceinline__ int block_of(int ws, int bi, int bpw)
    {
        return joined(bpw) ? 2 * (ws + (bi / 2) * SG) + bi % 2 : ws + bi * SG;
    }
    static_assert(P % OP::KG == 0 && Q % OP::MB == 0 && QT % QSPLIT == 0 && NW % QSPLIT == 0, "shape");
    static_assert((PL * sizeof(T)) % 16 == 0, "a lane's piece of a slice must be whole 16-byte vectors");
    static_assert(TK % (VN * NT) == 0, "tile must be a whole number of vectors per thread");
};

template <class OP, int P, int Q, int NF, int ST, int NW, int QSPLIT, int J, bool KEEP>
__device__ __forceinline__ void mfma_stage(typename OP::T* __restrict__ tile,
                                           const typename OP::T (&a)[MfmaShape<OP, P, Q, NF, ST, NW, QSPLIT>::QTW][MfmaShape<OP, P, Q, NF, ST, NW, QSPLIT>::PL],
                                           typename OP::T* __restrict__ Yrow, int64_t s_row, int64_t h)
{
    typedef MfmaShape<OP, P, Q, NF, ST, NW, QSPLIT> Sh;
    typedef typename OP::T T;
    typedef typename Vec16<T>::type V;
    constexpr int VN = Sh::VN, PL = Sh::PL, QTW = Sh::QTW, SG = Sh::SG, RS = Sh::RS;
    constexpr int SJ = Sh::size(J) / P;                // slices at this stage
    constexpr int NBLK = SJ / OP::NB;                  // slice blocks
    constexpr int BPW = NBLK / SG;                     // ... per wave group
    static_assert(SJ % OP::NB == 0 && NBLK % SG == 0, "slice blocks must divide among the wave groups");
    constexpr bool LAST = J == NF - 1;
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const int j = lane % OP::NB, g = lane / OP::NB;
    const int wq = wave % QSPLIT, ws = wave / QSPLIT;

    constexpr bool JOIN = LAST && Sh::joined(BPW);
    typename OP::Acc acc[LAST ? (JOIN ? 2 : 1) : BPW][QTW];
#pragma unroll
    for (int bi = 0; bi < BPW; ++bi) {
        const int s0 = (LAST ? Sh::block_of(ws, bi, BPW) : ws + bi * SG) * OP::NB;
        T b[PL];
        const V* src = reinterpret_cast<const V*>(tile + (s0 + j) * RS + g * PL);
#pragma unroll
        for (int c = 0; c < PL / VN; ++c) {
            const V v = src[c];
#pragma unroll
            for (int e = 0; e < VN; ++e) b[VN * c + e] = v[e];
        }
        const int ai = LAST ? (JOIN ? bi % 2 : 0) : bi;
#pragma unroll
        for (int qt = 0; qt < QTW; ++qt) {
#pragma unroll
            for (int v = 0; v < OP::NACC; ++v) acc[ai][qt][v] = T(0);
#pragma unroll
            for (int t = 0; t < PL; ++t) acc[ai][qt] = OP::mma(a[qt][t], b[t], acc[ai][qt]);
        }
        if constexpr (LAST) {
            // local (q, s), s = qrest*ST + r  ->  column (q*Q^(NF-1) + qrest)*s_row + h*ST + r
            constexpr int QREST = (int)ipow(Q, NF - 1);
            // (in-row offsets fit 32 bits: the planner only picks this kernel for rows below 2^31 bytes)
            const int sr = (int)s_row;
            if constexpr (JOIN) {
                if (bi % 2 == 1) {
                    // blocks s0 - NB and s0 together: 2*NB consecutive slices per half wavefront
                    const int s = s0 - OP::NB + lane % 32;
                    const int off = (s / ST) * sr + (int)h * ST + (s % ST) + (wq * QTW * OP::MB + 8 * (lane / 32)) * QREST * sr;
#pragma unroll
                    for (int qt = 0; qt < QTW; ++qt)
#pragma unroll
                        for (int v = 0; v < OP::NACC; ++v) {
                            join_blocks(acc[0][qt], acc[1][qt], v);
                            out_store<KEEP>(acc[0][qt][v], &Yrow[off + (qt * OP::MB + v) * QREST * sr]);
                            out_store<KEEP>(acc[1][qt][v], &Yrow[off + (qt * OP::MB + 4 + v) * QREST * sr]);
                        }
                }
            } else {
                const int s = s0 + j;
                const int off = (s / ST) * sr + (int)h * ST + (s % ST) + (wq * QTW * OP::MB + OP::row_lane(lane)) * QREST * sr;
#pragma unroll
                for (int qt = 0; qt < QTW; ++qt)
#pragma unroll
                    for (int v = 0; v < OP::NACC; ++v)
                        out_store<KEEP>(acc[0][qt][v], &Yrow[off + (qt * OP::MB + OP::row_reg(v)) * QREST * sr]);
            }
        }
    }
    if constexpr (!LAST) {
        __syncthreads();                               // the whole tile has been read
#pragma unroll
        for (int bi = 0; bi < BPW; ++bi) {
            const int s = (ws + bi * SG) * OP::NB + j;
#pragma unroll
            for (int qt = 0; qt < QTW; ++qt)
#pragma unroll
                for (int v = 0; v < OP::NACC; ++v) {
                    const int q = (wq * QTW + qt) * OP::MB + OP::row_lane(lane) + OP::row_reg(v);
                    const int c = q * SJ + s;          // position in the next stage's row of the tile
                    tile[(c / P) * RS + (c % P)] = acc[bi][qt][v];
                }
        }
        __syncthreads();
    }
}

// Single factor, split in two so that the caller can refill the other tile buffer between them:
// all products of this wavefront's slice blocks first (accumulators stay in registers) ...
template <class OP, int P, int Q, int ST, int NW, int QSPLIT>
__device__ __forceinline__ void mfma_single_compute(
    const typename OP::T* __restrict__ tile,
    const typename OP::T (&a)[MfmaShape<OP, P, Q, 1, ST, NW, QSPLIT>::QTW][MfmaShape<OP, P, Q, 1, ST, NW, QSPLIT>::PL],
    typename OP::Acc (&acc)[ST / OP::NB / MfmaShape<OP, P, Q, 1, ST, NW, QSPLIT>::SG][MfmaShape<OP, P, Q, 1, ST, NW, QSPLIT>::QTW])
{
    typedef MfmaShape<OP, P, Q, 1, ST, NW, QSPLIT> Sh;
    typedef typename OP::T T;
    typedef typename Vec16<T>::type V;
    constexpr int VN = Sh::VN, PL = Sh::PL, QTW = Sh::QTW, SG = Sh::SG, RS = Sh::RS;
    constexpr int BPW = ST / OP::NB / SG;
    static_assert(ST % OP::NB == 0 && (ST / OP::NB) % SG == 0, "slice blocks must divide among the wave groups");
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const int j = lane % OP::NB, g = lane / OP::NB;
    const int ws = wave / QSPLIT;
#pragma unroll
    for (int bi = 0; bi < BPW; ++bi) {
        const int s0 = Sh::block_of(ws, bi, BPW) * OP::NB;
        T b[PL];
        const V* src = reinterpret_cast<const V*>(tile + (s0 + j) * RS + g * PL);
#pragma unroll
        for (int c = 0; c < PL / VN; ++c) {
            const V v = src[c];
#pragma unroll
            for (int e = 0; e < VN; ++e) b[VN * c + e] = v[e];
        }
#pragma unroll
        for (int qt = 0; qt < QTW; ++qt) {
#pragma unroll
            for (int v = 0; v < OP::NACC; ++v) acc[bi][qt][v] = T(0);
#pragma unroll
            for (int t = 0; t < PL; ++t) acc[bi][qt] = OP::mma(a[qt][t], b[t], acc[bi][qt]);
        }
    }
}

// ... then the permuted store: (q, s) -> column q*s_row + h*ST + s.
template <class OP, int P, int Q, int ST, int NW, int QSPLIT, bool KEEP>
__device__ __forceinline__ void mfma_single_store(
    typename OP::T* __restrict__ Yrow, int64_t s_row, int64_t h,
    typename OP::Acc (&acc)[ST / OP::NB / MfmaShape<OP, P, Q, 1, ST, NW, QSPLIT>::SG][MfmaShape<OP, P, Q, 1, ST, NW, QSPLIT>::QTW])
{
    typedef MfmaShape<OP, P, Q, 1, ST, NW, QSPLIT> Sh;
    constexpr int QTW = Sh::QTW, SG = Sh::SG;
    constexpr int BPW = ST / OP::NB / SG;
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const int j = lane % OP::NB;
    const int wq = wave % QSPLIT, ws = wave / QSPLIT;
    // (in-row offsets fit 32 bits: the planner only picks this kernel for rows below 2^31 bytes)
    const int sr = (int)s_row;
    if constexpr (Sh::joined(BPW)) {
#pragma unroll
        for (int bi = 0; bi < BPW; bi += 2) {
            const int s = Sh::block_of(ws, bi, BPW) * OP::NB + lane % 32;
            const int off = (int)h * ST + s + (wq * QTW * OP::MB + 8 * (lane / 32)) * sr;
#pragma unroll
            for (int qt = 0; qt < QTW; ++qt)
#pragma unroll
                for (int v = 0; v < OP::NACC; ++v) {
                    join_blocks(acc[bi][qt], acc[bi + 1][qt], v);
                    out_store<KEEP>(acc[bi][qt][v], &Yrow[off + (qt * OP::MB + v) * sr]);
                    out_store<KEEP>(acc[bi + 1][qt][v], &Yrow[off + (qt * OP::MB + 4 + v) * sr]);
                }
        }
    } else {
#pragma unroll
        for (int bi = 0; bi < BPW; ++bi) {
            const int s = (ws + bi * SG) * OP::NB + j;
            const int off = (int)h * ST + s + (wq * QTW * OP::MB + OP::row_lane(lane)) * sr;
#pragma unroll
            for (int qt = 0; qt < QTW; ++qt)
#pragma unroll
                for (int v = 0; v < OP::NACC; ++v)
                    out_store<KEEP>(acc[bi][qt][v], &Yrow[off + (qt * OP::MB + OP::row_reg(v)) * sr]);
        }
    }
}

template <class OP, int P, int Q, int NF, int ST, int NW, int QSPLIT, bool KEEP>
__global__ __launch_bounds__(NW * 64, (NW >= 16 ? 4 : 2))   // second bound: wavefronts per SIMD to fit
void mfma_sliced_multiply(const typename OP::T* __restrict__ Xg, typename OP::T* __restrict__ Yg,
                          const typename OP::T* __restrict__ F0, const typename OP::T* __restrict__ F1,
                          int64_t k_in, int64_t k_out, int64_t tiles_per_row, int64_t num_tiles,
                          int64_t tiles_per_wg, int tile_order)
{
    typedef MfmaShape<OP, P, Q, NF, ST, NW, QSPLIT> Sh;
    typedef typename OP::T T;
    typedef typename Vec16<T>::type V;
    constexpr int VN = Sh::VN, PL = Sh::PL, QTW = Sh::QTW, RS = Sh::RS, NT = Sh::NT, RV = Sh::RV;
    extern __shared__ __attribute__((aligned(16))) unsigned char mfma_lds[];
    T* tile = reinterpret_cast<T*>(mfma_lds);

    const int tid = threadIdx.x;
    const int lane = tid % 64, wave = tid / 64;
    const int wq = wave % QSPLIT;
    const int ai = lane % OP::MB, ag = lane / OP::MB;

    // factor pieces of this lane: A[i][k] = F[p][q] with q = column block + ai, p = ag*PL + t
    T a0[QTW][PL], a1[NF > 1 ? QTW : 1][NF > 1 ? PL : 1];
#pragma unroll
    for (int qt = 0; qt < QTW; ++qt)
#pragma unroll
        for (int t = 0; t < PL; ++t) {
            const int q = (wq * QTW + qt) * OP::MB + ai;
            a0[qt][t] = F0[(ag * PL + t) * Q + q];
            if constexpr (NF > 1) a1[qt][t] = F1[(ag * PL + t) * Q + q];
        }

    const int64_t s_row = tiles_per_row * ST;
    // Tiles of this workgroup: t_begin, t_begin + t_step, ... below t_end.
    //  order 0: a contiguous range of tiles_per_wg tiles.
    //  order 1: two workgroups that the dispatcher places on the same XCD one after the other (ids b
    //           and b + 8) share a range of 2*tiles_per_wg tiles and take alternate ones, so that
    //           neighbouring tiles, whose short output runs fill the same cache lines, are written at
    //           about the same time into the same L2.
    //  order 2: tiles b, b + grid, b + 2*grid, ...: the workgroups resident at any moment work on
    //           consecutive tiles, so their output runs (one per factor column, a power-of-two stride
    //           apart within a tile) tile whole stretches of each output row instead of all falling
    //           on the same few memory channels.
    int64_t t_begin = (int64_t)blockIdx.x * tiles_per_wg, t_step = 1;
    int64_t t_end = t_begin + tiles_per_wg;
    if (tile_order == 1) {
        const int64_t b = blockIdx.x, xcd = b % 8, k = b / 8;
        t_begin = ((k >> 1) * 8 + xcd) * tiles_per_wg * 2 + (k & 1);
        t_step = 2;
        t_end = t_begin + 2 * tiles_per_wg;
    } else if (tile_order == 2) {
        t_begin = blockIdx.x;
        t_step = gridDim.x;
        t_end = num_tiles;
    } else if (tile_order == 3) {
        const int64_t per = num_tiles / 8, x = blockIdx.x % 8;
        t_begin = x * per + blockIdx.x / 8;
        t_step = gridDim.x / 8;
        t_end = (x + 1) * per;
    }
    if (t_end > num_tiles) t_end = num_tiles;

    auto tile_ptr = [&](int64_t t) {
        return reinterpret_cast<const V*>(Xg + (t / tiles_per_row) * k_in + (t % tiles_per_row) * Sh::TK);
    };
    V pf[RV];
    if (t_begin < t_end) {
        const V* src = tile_ptr(t_begin);
#pragma unroll
        for (int i = 0; i < RV; ++i) pf[i] = stream_load(&src[tid + i * NT]);
    }

    if constexpr (Sh::NBUF == 2) {
        // Two tile buffers, one barrier per tile.  While tile t is multiplied out of one buffer, tile
        // t+1 waits in registers; after the products it moves to the other buffer and the loads of
        // tile t+2 are issued, and only then are the results stored, so that waiting for a fetched
        // tile never means waiting for stores that were issued a moment ago.
        constexpr int BPW = ST / OP::NB / Sh::SG;
        if (t_begin < t_end) {
#pragma unroll
            for (int i = 0; i < RV; ++i) {
                const int e = (tid + i * NT) * VN;
                *reinterpret_cast<V*>(tile + (e / P) * RS + (e % P)) = pf[i];
            }
            if (t_begin + t_step < t_end) {
                const V* src = tile_ptr(t_begin + t_step);
#pragma unroll
                for (int i = 0; i < RV; ++i) pf[i] = stream_load(&src[tid + i * NT]);
            }
        }
        __syncthreads();
        int cur = 0;
        for (int64_t t = t_begin; t < t_end; t += t_step) {
            T* buf = tile + cur * Sh::BUF_ELEMS;
            T* other = tile + (cur ^ 1) * Sh::BUF_ELEMS;
            typename OP::Acc acc[BPW][QTW];
            mfma_single_compute<OP, P, Q, ST, NW, QSPLIT>(buf, a0, acc);
            if (t + t_step < t_end) {
#pragma unroll
                for (int i = 0; i < RV; ++i) {
                    const int e = (tid + i * NT) * VN;
                    *reinterpret_cast<V*>(other + (e / P) * RS + (e % P)) = pf[i];
                }
                if (t + 2 * t_step < t_end) {
                    const V* src = tile_ptr(t + 2 * t_step);
#pragma unroll
                    for (int i = 0; i < RV; ++i) pf[i] = stream_load(&src[tid + i * NT]);
                }
            }
            const int64_t row = t / tiles_per_row, h = t % tiles_per_row;
            mfma_single_store<OP, P, Q, ST, NW, QSPLIT, KEEP>(Yg + row * k_out, s_row, h, acc);
            __syncthreads();      // the other buffer is complete; this one has been read by everybody
            cur ^= 1;
        }
    } else {
        for (int64_t t = t_begin; t < t_end; t += t_step) {
            // registers -> LDS rows of P elements with stride RS
#pragma unroll
            for (int i = 0; i < RV; ++i) {
                const int e = (tid + i * NT) * VN;
                *reinterpret_cast<V*>(tile + (e / P) * RS + (e % P)) = pf[i];
            }
            __syncthreads();
            const int64_t row = t / tiles_per_row, h = t % tiles_per_row;
            T* Yrow = Yg + row * k_out;
            // With two factors the fetch of the next tile is issued after the first stage: its
            // registers then only coexist with the streaming second stage, not with the held
            // accumulators.
            if constexpr (NF == 1) {
                if (t + t_step < t_end) {
                    const V* src = tile_ptr(t + t_step);
#pragma unroll
                    for (int i = 0; i < RV; ++i) pf[i] = stream_load(&src[tid + i * NT]);
                }
                mfma_stage<OP, P, Q, NF, ST, NW, QSPLIT, 0, KEEP>(tile, a0, Yrow, s_row, h);
            } else {
                mfma_stage<OP, P, Q, NF, ST, NW, QSPLIT, 0, KEEP>(tile, a0, Yrow, s_row, h);
                if (t + t_step < t_end) {
                    const V* src = tile_ptr(t + t_step);
#pragma unroll
                    for (int i = 0; i < RV; ++i) pf[i] = stream_load(&src[tid + i * NT]);
                }
                mfma_stage<OP, P, Q, NF, ST, NW, QSPLIT, 1, KEEP>(tile, a1, Yrow, s_row, h);
            }
            __syncthreads();                           // tile fully consumed before it is overwritten
        }
    }
}

}  // namespace km
