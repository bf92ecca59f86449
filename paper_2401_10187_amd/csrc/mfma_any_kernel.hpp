// One sliced-multiply iteration on the matrix cores for a factor of any shape whose slices start on
// 16-byte boundaries (P a multiple of 4 floats or 2 doubles; run-time shapes: 20, 48, 80, 96, 100, ...
// and rectangles), are at most one chunk long (FLAT == 1 below: 13, 22, 33, 50, ...) or neither
// (FLAT == 2: 65, 99, 127, fp64 33, 45, ...), fp32 and fp64.  P and Q are padded with zeros to
// multiples of 16 on the way into LDS.
//
// The contraction of a slice with the factor (Algorithm 1's inner loop) is the dense product
//     D[q][s] = sum_p F[p][q] * X[s*P + p]
// done with the 16x16x4 MFMA of the element type: the factor is the A operand (rows q), slices are the
// B operand (columns s), so an accumulator register holds 16 consecutive slices of one factor column
// and stores are runs of the output row (the output column of (s, q) is q*(K/P)+s; section 4 of the
// paper, with the matrix cores in place of its thread tiles).
//
// A unit of work is 128 consecutive slices (256 in the narrow shape, see AnyShape), numbered through
// all rows as in the generic kernel, times CB*16 factor columns; workgroups stride over the units,
// units of the same slices being numbered so that they run on the same XCD (they share the slices
// through its L2 cache).  P is walked in chunks of 256 bytes per slice (64 floats, 32 doubles; narrow:
// 128 bytes; the last chunk may be shorter): a chunk of the slices and the matching rows of the
// factor, transposed, sit in LDS, rows padded to an odd number of 16-byte units so that the 16-byte
// operand reads of 16 consecutive lanes fall into different banks.  Each of the four wavefronts owns
// 32 slices (narrow: 64), MFMA blocks of 16 that are joined in pairs before the store in fp32 so that
// a half wavefront writes a whole 128-byte line, and all CB column blocks.  Loads and stores are
// bounds-checked against the slice, element and column counts; the factor is read with 16-byte loads
// when its rows start on 16-byte boundaries (f_aligned: base aligned and Q a whole number of vectors),
// element by element otherwise.  KEEP selects ordinary instead of non-temporal stores (out_store).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "fused_kernel.hpp"   // Vec16, stream_load / stream_store
#include "mfma_kernel.hpp"    // MfmaF32x16, MfmaF64x16, join_blocks
#include "plan.hpp"           // any_column_blocks

namespace km {

constexpr int ANY_NW = 4;                   // wavefronts per workgroup
constexpr int ANY_THREADS = 64 * ANY_NW;
constexpr int ANY_TS = 32 * ANY_NW;         // slices per unit of the wide shape (two 16-slice blocks per wavefront)
constexpr int ANY_ROW_BYTES = 256;          // bytes of a slice per LDS chunk of the wide shape (64 floats, 32 doubles)

template <typename T> struct AnyOp;
template <> struct AnyOp<float> { typedef MfmaF32x16 OP; };
template <> struct AnyOp<double> { typedef MfmaF64x16 OP; };

// NARROW (slices of at most 128 bytes): chunks of half the bytes and units of twice the slices, so
// that a unit still moves enough bytes to keep the memory system busy and fewer lanes idle in the loads.
template <typename T, int CB, bool NARROW>
struct AnyShape {
    static constexpr int VN = Vec16<T>::N;
    static constexpr int SB = NARROW ? 4 : 2;                   // 16-slice blocks per wavefront
    static constexpr int TS = 16 * SB * ANY_NW;                 // slices per unit
    static constexpr int KT = ANY_ROW_BYTES / (NARROW ? 2 : 1) / (int)sizeof(T);   // slice elements per LDS chunk
    static constexpr int ROW = KT + VN;                         // padded LDS row: an odd number of 16-byte units
    static constexpr int QG = CB * 16;                          // factor columns per unit
    static constexpr int X_ELEMS = TS * ROW, F_ELEMS = QG * ROW;
    static constexpr int LDS_BYTES = (X_ELEMS + F_ELEMS) * (int)sizeof(T);
    static constexpr int VPR = KT / VN;                         // 16-byte vectors per chunk row of a slice
    static constexpr int RP = ANY_THREADS / VPR;                // slices the workgroup fetches per pass
    static constexpr int XV = TS / RP;                          // vectors of the slice chunk per thread
    static constexpr int FVR = QG / VN;                         // 16-byte vectors per chunk row of the factor
    static constexpr int FV = (KT * FVR + ANY_THREADS - 1) / ANY_THREADS;   // vectors of the factor chunk per thread
    static_assert(TS == (NARROW ? 2 : 1) * ANY_TS && XV * RP == TS && KT % 16 == 0, "fetch passes cover the unit");
    static_assert(((ROW * sizeof(T)) / 16) % 2 == 1, "row stride must be an odd number of 16-byte units");
};

// (the second launch bound, wavefronts per SIMD, caps the registers: left alone the compiler spends
// several hundred of them on scheduling freedom and one workgroup fills a compute unit)
// FLAT == 1: for slices that do not start on 16-byte boundaries (P not a whole number of vectors) and
// fit one chunk (P <= KT).  The TS slices of a unit are contiguous in memory and the unit starts on a
// 16-byte boundary (TS * P elements per unit), so the unit is fetched as one run of 16-byte vectors and
// the elements are dealt to their LDS rows one by one (consecutive elements, consecutive banks).
// FLAT == 2: such slices of several chunks (wide shape only).  A chunk row of a slice then starts
// anywhere inside a 16-byte vector, so VPR + 1 aligned vectors cover it: that many threads fetch one
// row (15 rows per pass instead of 16), and every element is written to its LDS column on its own;
// elements of the vectors that belong to the neighbouring chunk or slice are dropped, columns past the
// end of the slice are zeroed.  Nothing outside X is read: a vector that would pass its end is fetched
// element by element.
template <typename T, int CB, bool NARROW, bool KEEP, int FLAT>
__global__ __launch_bounds__(ANY_THREADS, (CB >= 5 || (NARROW && sizeof(T) == 8 && CB >= 3) ? 2 : 3))
void mfma_any_sliced_multiply(const T* __restrict__ Xg, const T* __restrict__ Fg, T* __restrict__ Yg,
                              int64_t K, int P, int Q, int64_t num_slices, int64_t num_units, int f_aligned)
{
    typedef AnyShape<T, CB, NARROW> Sh;
    typedef typename AnyOp<T>::OP OP;
    typedef typename Vec16<T>::type V;
    constexpr int VN = Sh::VN, KT = Sh::KT, ROW = Sh::ROW, QG = Sh::QG, XV = Sh::XV, FVR = Sh::FVR, FV = Sh::FV;
    constexpr int SB = Sh::SB, TS = Sh::TS, RP = Sh::RP;
    constexpr bool GATHER = sizeof(T) == 8 || CB >= 5;  // how the factor chunk is transposed into LDS (below)
    constexpr bool SKEW = FLAT == 2;
    constexpr int VPX = Sh::VPR + 1;                   // aligned vectors that cover a chunk row starting anywhere
    constexpr int RPX = ANY_THREADS / VPX;             // rows per pass of the skewed fetch (the last threads idle)
    constexpr int XVX = (TS + RPX - 1) / RPX;
    constexpr int XN = SKEW ? XVX : XV;
    static_assert(!SKEW || !NARROW, "slices of several chunks take the wide shape");
    extern __shared__ __attribute__((aligned(16))) unsigned char any_lds[];
    T* Xs = reinterpret_cast<T*>(any_lds);            // [TS][ROW]: slice i, chunk element k
    T* Fs = Xs + Sh::X_ELEMS;                          // [QG][ROW]: factor column q (transposed), chunk element k

    const int64_t S = K / P;
    const int tid = threadIdx.x;
    const int lane = tid % 64, wave = tid / 64;
    const int j = lane % 16, g = lane / 16;            // operand row/column inside a block, k group
    const int q_groups = (Q + QG - 1) / QG;
    const int xrow = tid / Sh::VPR, xcol = (tid % Sh::VPR) * VN;   // fetch duty: column xcol of slices xrow, xrow + RP, ...
    const int srow = tid / VPX, svec = tid % VPX;      // skewed fetch: vector svec of slices srow, srow + RPX, ...

    // A factor of one column group and one chunk is the same LDS content for every unit of this
    // workgroup: it is staged with the first unit only (2048 x 36x36^3 0.700 -> 0.567 ms, 512 x 52x52^3
    // 0.580 -> 0.481, 512 x 60x60^3 0.814 -> 0.667, 1024 x 24x24^4 2.47 -> 2.23: the scalar, bank-conflicting LDS
    // writes of the transposition cost as much as staging the slices.  Variants measured slower: the
    // same as a compile-time form of the kernel that stages the factor ahead of the loop (0.620 for
    // 36x36^3), and a whole factor of several chunks in rows of run-time length, 3-5 % only).
    const bool f_stays = q_groups == 1 && P <= KT;

    if constexpr (FLAT == 1) {
        // elements P .. KT - 1 of every LDS row are read by the products (up to the next multiple of 16)
        // and never written by the unit loop: zeros, once
        const int pad = KT - P;
        for (int e = tid; e < TS * pad; e += ANY_THREADS) Xs[(e / pad) * ROW + P + e % pad] = T(0);
    }

    for (int64_t unit = blockIdx.x; unit < num_units; unit += gridDim.x) {
        const bool stage_f = !f_stays || unit == blockIdx.x;
        int64_t tile;
        int group;
        unit_of(unit, num_units / q_groups, q_groups, tile, group);
        const int64_t g0 = tile * TS;                // first slice of the unit, counted through all rows
        const int q0 = group * QG;

        typename OP::Acc acc[SB][CB];
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int v = 0; v < OP::NACC; ++v) acc[sb][cb][v] = T(0);

        for (int k0 = 0; k0 < P; k0 += KT) {
            const int kt = P - k0 < KT ? P - k0 : KT;
            // The chunk is fetched before the barrier that frees the LDS buffer, so its latency overlaps
            // with the other wavefronts' products; further overlap comes from the three workgroups that
            // share a compute unit.  Slices only this unit reads bypass the caches; with several column
            // groups they stay for the neighbouring units.
            V xr[XN], fr[FV];
            const T* xsrc = Xg + g0 * P + k0;            // uniform part of the slice addresses
            if constexpr (SKEW) {
                const int64_t total = num_slices * P;    // elements of X
#pragma unroll
                for (int i = 0; i < XVX; ++i) {
                    const int row = srow + RPX * i;
#pragma unroll
                    for (int k = 0; k < VN; ++k) xr[i][k] = T(0);
                    if (srow < RPX && row < TS && g0 + row < num_slices) {
                        const int64_t o = (g0 + row) * P + k0;                        // first element of the chunk row
                        const int64_t a = (o & ~(int64_t)(VN - 1)) + svec * VN;       // this thread's aligned vector
                        if (a - o < kt) {                                             // some of it lies inside the chunk row
                            if (a + VN <= total) {
                                const V* src = reinterpret_cast<const V*>(Xg + a);
                                xr[i] = q_groups == 1 ? stream_load(src) : *src;
                            } else {
#pragma unroll
                                for (int k = 0; k < VN; ++k) xr[i][k] = a + k < total ? Xg[a + k] : T(0);
                            }
                        }
                    }
                }
            } else if constexpr (FLAT == 1) {
                // vector v of the unit's TS * P contiguous elements; the last unit may hold fewer slices
                const int64_t left = (num_slices - g0) * P;
                const int valid = left < (int64_t)TS * P ? (int)left : TS * P;
#pragma unroll
                for (int i = 0; i < XV; ++i) {
                    const int e0 = (tid + i * ANY_THREADS) * VN;
                    if (e0 + VN <= valid) {
                        const V* src = reinterpret_cast<const V*>(xsrc + e0);
                        xr[i] = q_groups == 1 ? stream_load(src) : *src;
                    } else {
#pragma unroll
                        for (int k = 0; k < VN; ++k) xr[i][k] = e0 + k < valid ? xsrc[e0 + k] : T(0);
                    }
                }
            } else {
#pragma unroll
            for (int i = 0; i < XV; ++i) {
                const int row = xrow + RP * i;
                if (g0 + row < num_slices && xcol < kt) {
                    const V* src = reinterpret_cast<const V*>(xsrc + row * P + xcol);
                    xr[i] = q_groups == 1 ? stream_load(src) : *src;
                } else {
#pragma unroll
                    for (int k = 0; k < VN; ++k) xr[i][k] = T(0);
                }
            }
            }
            // The factor chunk goes into LDS transposed.  GATHER: a thread gathers VN consecutive rows p of
            // one column q (element-sized loads; lanes run along q, so each load instruction reads stretches
            // of factor rows) and writes them as one 16-byte vector of row q of Fs, free of bank conflicts
            // (512 x 40x40^3 fp64 0.413 -> 0.373 ms, 1024 x 44x44^3 fp64 1.016 -> 0.901, 128 x 72x72^3 0.490 -> 0.450).
            // Otherwise it loads a 16-byte vector of one factor row and scatters its elements over VN rows
            // of Fs with element-sized writes, four to a bank: the gathering form needs more address
            // registers, and the fp32 kernels of three and four column blocks spill with it (36x36^3 +30 %).
            const T* fsrc = Fg + (int64_t)k0 * Q + q0;   // uniform part of the factor addresses
            if (stage_f)
#pragma unroll
            for (int i = 0; i < FV; ++i) {
                const int e = tid + i * ANY_THREADS;
                if constexpr (GATHER) {
                    const int q = e % QG, p = (e / QG) * VN;
#pragma unroll
                    for (int k = 0; k < VN; ++k) fr[i][k] = (p + k < kt && q0 + q < Q) ? fsrc[(p + k) * Q + q] : T(0);
                } else {
                    const int p = e / FVR, q = (e % FVR) * VN;
                    if (f_aligned && p < kt && q0 + q < Q) fr[i] = *reinterpret_cast<const V*>(fsrc + p * Q + q);
                    else                                 // factor rows that do not start on 16-byte boundaries, padding
#pragma unroll
                        for (int k = 0; k < VN; ++k) fr[i][k] = (p < kt && q0 + q + k < Q) ? fsrc[p * Q + q + k] : T(0);
                }
            }
            __syncthreads();                             // the previous chunk (or unit) has been read by everybody
            if constexpr (SKEW) {
#pragma unroll
                for (int i = 0; i < XVX; ++i) {
                    const int row = srow + RPX * i;
                    if (srow < RPX && row < TS) {
                        const int mis = (int)(((g0 + row) * P + k0) & (VN - 1));
#pragma unroll
                        for (int k = 0; k < VN; ++k) {
                            const int col = svec * VN + k - mis;                      // column of the chunk row
                            if (col >= 0 && col < KT) Xs[row * ROW + col] = col < kt ? xr[i][k] : T(0);
                        }
                    }
                }
            } else if constexpr (FLAT == 1) {
#pragma unroll
                for (int i = 0; i < XV; ++i) {
                    const int e0 = (tid + i * ANY_THREADS) * VN;
                    if (e0 < TS * P) {
                        int row = e0 / P, col = e0 - row * P;
#pragma unroll
                        for (int k = 0; k < VN; ++k) {
                            Xs[row * ROW + col] = xr[i][k];
                            if (++col == P) { col = 0; ++row; }
                        }
                    }
                }
            } else {
#pragma unroll
                for (int i = 0; i < XV; ++i) *reinterpret_cast<V*>(Xs + (xrow + RP * i) * ROW + xcol) = xr[i];
            }
            if (stage_f)
#pragma unroll
            for (int i = 0; i < FV; ++i) {
                const int e = tid + i * ANY_THREADS;
                if constexpr (GATHER) {
                    const int q = e % QG, p = (e / QG) * VN;
                    if (p < KT) *reinterpret_cast<V*>(Fs + q * ROW + p) = fr[i];     // column q, elements p .. p + VN - 1
                } else {
                    const int p = e / FVR, q = (e % FVR) * VN;
                    if (p < KT)
#pragma unroll
                        for (int k = 0; k < VN; ++k) Fs[(q + k) * ROW + p] = fr[i][k];     // transposed: column q, element p
                }
            }
            __syncthreads();
            // 16 chunk elements per trip: lane group g takes elements 4g .. 4g+3 of them, one MFMA step each
#pragma unroll 1
            for (int kc = 0; kc < kt; kc += 16) {
                T b[SB][4], a[CB][4];
#pragma unroll
                for (int sb = 0; sb < SB; ++sb) {
                    const T* src = Xs + (wave * 16 * SB + sb * 16 + j) * ROW + kc + 4 * g;
#pragma unroll
                    for (int c = 0; c < 4 / VN; ++c) {
                        const V v = reinterpret_cast<const V*>(src)[c];
#pragma unroll
                        for (int k = 0; k < VN; ++k) b[sb][c * VN + k] = v[k];
                    }
                }
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    const T* src = Fs + (cb * 16 + j) * ROW + kc + 4 * g;
#pragma unroll
                    for (int c = 0; c < 4 / VN; ++c) {
                        const V v = reinterpret_cast<const V*>(src)[c];
#pragma unroll
                        for (int k = 0; k < VN; ++k) a[cb][c * VN + k] = v[k];
                    }
                }
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb) acc[sb][cb] = OP::mma(a[cb][t], b[sb][t], acc[sb][cb]);
            }
        }

        // permuted store: (slice s of row r, column q) -> Y[r*(S*Q) + q*S + s]
        if constexpr (OP::JOIN_BLOCKS) {
            static_assert(SB % 2 == 0, "joined stores take the slice blocks of a wavefront in pairs");
            // after the exchange, register v of a pair's first block holds column 8*(lane/32) + v of its column
            // block and the second block's register column 8*(lane/32) + 4 + v, both for slice lane % 32
#pragma unroll
            for (int sb = 0; sb < SB; sb += 2) {
                const int64_t slice = g0 + wave * 16 * SB + sb * 16 + lane % 32;
                const bool live = slice < num_slices;
                T* Ycol = Yg + (live ? (slice / S) * (S * (int64_t)Q) + slice % S : 0);
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int v = 0; v < OP::NACC; ++v) {
                        join_blocks(acc[sb][cb], acc[sb + 1][cb], v);
                        const int q = q0 + cb * 16 + 8 * (lane / 32) + v;
                        if (live && q < Q) out_store<KEEP>(acc[sb][cb][v], &Ycol[(int64_t)q * S]);
                        if (live && q + 4 < Q) out_store<KEEP>(acc[sb + 1][cb][v], &Ycol[(int64_t)(q + 4) * S]);
                    }
            }
        } else {
#pragma unroll
            for (int sb = 0; sb < SB; ++sb) {
                const int64_t slice = g0 + wave * 16 * SB + sb * 16 + j;
                const bool live = slice < num_slices;
                T* Ycol = Yg + (live ? (slice / S) * (S * (int64_t)Q) + slice % S : 0);
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int v = 0; v < OP::NACC; ++v) {
                        const int q = q0 + cb * 16 + OP::row_lane(lane) + OP::row_reg(v);
                        if (live && q < Q) out_store<KEEP>(acc[sb][cb][v], &Ycol[(int64_t)q * S]);
                    }
            }
        }
    }
}

}  // namespace km
