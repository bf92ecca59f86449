// Two fused sliced multiplies on the matrix cores with the intermediate kept in registers
// (fusion of section 4.2 of the paper with N_fused = 2; fp32, P x 32 factors, P = 16 or 32).
//
// A tile is ST*P*P contiguous elements of one row: X[a][p1][p2], a < ST.  The pair of factors maps
// it to Y[(q1, q2)][a], stored at column (q1*Q + q2)*(K_in/P^2) + h*ST + a of the output row (h =
// tile index in the row), exactly as the LDS-resident fused kernels do.
//
// For one `a` both contractions are dense products and the accumulator layout of the first is the
// B-operand layout of the second:
//   stage 0   D0[p1][q2] = sum_p2 X[a][p1][p2] * F0[p2][q2]      A = X_a  (rows p1), B = F0
//   stage 1   D1[q1][q2] = sum_p1 F1[p1][q1]   * D0[p1][q2]      A = F1^T (rows q1), B = D0
// v_mfma_f32_32x32x2_f32 leaves D0 with column q2 on lane%32 and row 8*(v/4) + 4*(lane/32) + v%4 in
// register v; taken as a B operand, register t of lane half g therefore supplies k = p1 =
// 8*(t/4) + 4*g + t%4, and the A operand (F1) is loaded in that same order.  The intermediate never
// leaves the registers: no LDS, no barrier, no transposition between the two stages.
// With P = 16 one 32-row stage-0 product covers two values of `a`.
//
// X is read straight from global memory into the A-operand registers (each lane takes P/2
// contiguous elements of its slice).  Only the result passes through LDS, to turn "one a per
// wavefront pass" into contiguous runs of ST elements along `a`: D1 of all the tile's `a` is written
// as rows (q1, q2) of ST elements, then read back 16 bytes per lane and stored with 16-byte global
// stores, half of the q1 range at a time so that two workgroups fit a compute unit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "fused_kernel.hpp"   // Vec16

namespace km {

template <int P, int ST, int NW, int PD = 1, int NPASS = 2>
struct MfmaPairShape {
    static constexpr int Q = 32;
    static constexpr int NT = NW * 64;
    static constexpr int AP = 32 / P;                 // values of `a` per 32-row stage-0 product
    static constexpr int KS = P / 2;                  // MFMA steps per product (2 k values per step)
    static constexpr int UNITS = ST / AP;             // stage-0 products per tile
    static constexpr int UPW = UNITS / NW;            // ... per wavefront
    static constexpr int APW = UPW * AP;              // values of `a` per wavefront
    static constexpr int TK = ST * P * P;
    static constexpr int STP = ST + 4;                // padded row of the output staging buffer
    // The output goes through the staging buffer in NPASS passes over the q1 range: with two passes
    // (72 KB) two workgroups fit a compute unit and each keeps the second half of its accumulators in
    // registers meanwhile; with one pass (144 KB) a single large workgroup keeps nothing.
    static constexpr int PASS_Q1 = Q / NPASS;         // q1 values per pass
    static constexpr int PASS_ROWS = PASS_Q1 * Q;     // rows (q1_local, q2) of one output pass
    static constexpr int LDS_BYTES = PASS_ROWS * STP * 4;
    static constexpr int RD = PASS_ROWS * (ST / 4) / NT;   // 16-byte reads per thread and pass
    static constexpr int WPS = NW >= 8 ? 4 : 2;       // wavefronts per SIMD the register budget is set for
    static_assert(P == 16 || P == 32, "P must be 16 or 32");
    static_assert(NPASS == 1 || NPASS == 2, "one or two output passes");
    static_assert(ST % (AP * NW) == 0 && ST % 4 == 0, "tile must split evenly over the wavefronts");
    static_assert((PASS_ROWS * (ST / 4)) % NT == 0, "output pass must split evenly over the threads");
    static constexpr int RING = PD + 1;               // operand buffers: PD units in flight + the one in use
    static_assert(PD >= 1 && PD < UPW && UPW % RING == 0, "the operand ring must wrap once per tile");
    static_assert(RD % 4 == 0, "output reads are issued four at a time");
};

typedef float pair_f32x16 __attribute__((ext_vector_type(16)));
typedef float pair_f32x4 __attribute__((ext_vector_type(4)));

template <int P, int ST, int NW, int PD, int NPASS, bool KEEP>
__global__ __launch_bounds__(NW * 64, (MfmaPairShape<P, ST, NW, PD, NPASS>::WPS))
void mfma_pair_sliced_multiply(const float* __restrict__ Xg, float* __restrict__ Yg,
                               const float* __restrict__ F0, const float* __restrict__ F1,   // in order of application
                               int64_t k_in, int64_t k_out, int64_t tiles_per_row, int64_t num_tiles,
                               int64_t tiles_per_wg, int tile_order)
{
    typedef MfmaPairShape<P, ST, NW, PD, NPASS> Sh;
    constexpr int Q = Sh::Q, KS = Sh::KS, AP = Sh::AP, UPW = Sh::UPW, STP = Sh::STP, NT = Sh::NT, RING = Sh::RING;
    extern __shared__ __attribute__((aligned(16))) unsigned char pair_lds[];
    float* stage = reinterpret_cast<float*>(pair_lds);

    const int tid = threadIdx.x;
    const int lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);    // wave-uniform: lets addresses be scalar base + lane offset
    const int col = lane % 32;        // stage 0: row (a_loc, p1) of A, column q2 of B; stage 1: row q1 of A
    const int g = lane / 32;          // which of the two k values of an MFMA step this lane holds

    // B operand of stage 0: F0[p2][q2], p2 = g*KS + t.   A operand of stage 1: F1[p1][q1] with
    // p1 = 8*(t/4) + 4*g + t%4, the row that accumulator register t of lane half g holds.
    float b0[KS], a1[KS];
#pragma unroll
    for (int t = 0; t < KS; ++t) {
        b0[t] = F0[(g * KS + t) * Q + col];
        a1[t] = F1[(8 * (t / 4) + 4 * g + (t % 4)) * Q + col];
    }

    const int64_t s_row = tiles_per_row * ST;
    // tile_order 0: a contiguous range of tiles per workgroup; 2: tiles b, b + grid, b + 2*grid, ...;
    // 3: the same stride inside the XCD's own eighth of the tiles
    int64_t t_begin = (int64_t)blockIdx.x * tiles_per_wg, t_step = 1;
    int64_t t_end = t_begin + tiles_per_wg;
    if (tile_order == 2) {
        t_begin = blockIdx.x;
        t_step = gridDim.x;
        t_end = num_tiles;
    } else if (tile_order == 3) {
        // each XCD (workgroup b runs on XCD b % 8) owns a contiguous eighth of the tiles and its
        // workgroups stride through it: neighbouring output runs meet in one L2
        const int64_t per = num_tiles / 8, x = blockIdx.x % 8;
        t_begin = x * per + blockIdx.x / 8;
        t_step = gridDim.x / 8;
        t_end = (x + 1) * per;
    }
    if (t_end > num_tiles) t_end = num_tiles;

    // element offset, inside a tile, of this lane's piece of unit u of this wavefront
    const unsigned lane_off = col * P + g * KS;
    // tile indices are wave-uniform; saying so keeps tile addresses in scalar registers
    auto uniform = [](int64_t v) {
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
        const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
        return (int64_t)(((uint64_t)hi << 32) | lo);
    };
    auto tile_src = [&](int64_t t) {
        return Xg + uniform(t / tiles_per_row) * k_in + uniform(t % tiles_per_row) * Sh::TK;
    };

    // A operand of stage 0: a ring of PD + 1 units, PD of them in flight while one is multiplied.
    // Unit v of every tile uses slot v % RING (UPW is a multiple of RING).
    pair_f32x4 xa[RING][KS / 4];
    if (t_begin < t_end) {
#pragma unroll
        for (int v = 0; v < PD; ++v) {
            const float* src = tile_src(t_begin) + ((wave + v * NW) * AP) * P * P;
#pragma unroll
            for (int c = 0; c < KS / 4; ++c) xa[v][c] = *reinterpret_cast<const pair_f32x4*>(src + (lane_off + 4 * c));
        }
    }

    for (int64_t t = t_begin; t < t_end; t += t_step) {
        const float* Xt = tile_src(t);
        // Registers 0-7 of a stage-1 accumulator hold q1 < 16 and go to the staging buffer at once
        // (it is free: the previous tile's last pass ended with a barrier); registers 8-15 (q1 >= 16)
        // wait here for the second pass.
        float keep[NPASS == 2 ? Sh::APW : 1][8];
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            // fetch unit u + PD (of this tile, or of the next one)
            {
                const int v = u + PD;
                if (v < UPW) {
                    const float* src = Xt + ((wave + v * NW) * AP) * P * P;
#pragma unroll
                    for (int c = 0; c < KS / 4; ++c)
                        xa[v % RING][c] = *reinterpret_cast<const pair_f32x4*>(src + (lane_off + 4 * c));
                } else if (t + t_step < t_end) {
                    const float* src = tile_src(t + t_step) + ((wave + (v - UPW) * NW) * AP) * P * P;
#pragma unroll
                    for (int c = 0; c < KS / 4; ++c)
                        xa[v % RING][c] = *reinterpret_cast<const pair_f32x4*>(src + (lane_off + 4 * c));
                }
            }
            pair_f32x16 d0;
#pragma unroll
            for (int v = 0; v < 16; ++v) d0[v] = 0.f;
#pragma unroll
            for (int s = 0; s < KS; ++s)
                d0 = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[u % RING][s / 4][s % 4], b0[s], d0, 0, 0, 0);
#pragma unroll
            for (int al = 0; al < AP; ++al) {
                pair_f32x16 acc;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
                for (int s = 0; s < KS; ++s)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[s], d0[al * KS + s], acc, 0, 0, 0);
                const int a = (wave + u * NW) * AP + al;
#pragma unroll
                for (int w = 0; w < 8; ++w) {
                    const int q1l = 8 * (w / 4) + 4 * g + (w % 4);           // q1 of register w (and of 8 + w, minus 16)
                    stage[(q1l * Q + col) * STP + a] = acc[w];
                    if constexpr (NPASS == 2) keep[u * AP + al][w] = acc[8 + w];
                    else stage[((16 + q1l) * Q + col) * STP + a] = acc[8 + w];
                }
            }
        }

        const int64_t row = uniform(t / tiles_per_row), h = uniform(t % tiles_per_row);
        float* Yrow = Yg + row * k_out + h * ST;
#pragma unroll
        for (int pass = 0; pass < NPASS; ++pass) {
            if (pass == 1) {
#pragma unroll
                for (int u = 0; u < UPW; ++u)
#pragma unroll
                    for (int al = 0; al < AP; ++al) {
                        const int a = (wave + u * NW) * AP + al;
#pragma unroll
                        for (int w = 0; w < 8; ++w) {
                            const int q1l = 8 * (w / 4) + 4 * g + (w % 4);
                            stage[(q1l * Q + col) * STP + a] = keep[u * AP + al][w];
                        }
                    }
            }
            __syncthreads();
            // row r = (q1l, q2) of the staging buffer -> output column ((PASS_Q1*pass + q1l)*Q + q2)*s_row + h*ST + a
            float* Ypass = Yrow + (int64_t)(Sh::PASS_Q1 * pass * Q) * s_row;
#pragma unroll
            for (int i0 = 0; i0 < Sh::RD; i0 += 4) {
                pair_f32x4 v[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int idx = tid + (i0 + i) * NT;
                    v[i] = *reinterpret_cast<const pair_f32x4*>(stage + (idx / (ST / 4)) * STP + 4 * (idx % (ST / 4)));
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int idx = tid + (i0 + i) * NT;
                    out_store<KEEP>(v[i], reinterpret_cast<pair_f32x4*>(Ypass + (int64_t)(idx / (ST / 4)) * s_row + 4 * (idx % (ST / 4))));
                }
            }
            __syncthreads();
        }
    }
}

}  // namespace km

namespace km {

// The same register-chained pair for rows that hold exactly one slice of the pair (K_in = P*P, the
// whole Kron-Matmul of two factors on a matrix with many rows): the slow index `a` of the tile is the
// row itself.  X rows are contiguous, so a tile of ST rows is read exactly as above; on the output
// side row a is (q1, q2) in memory order, which is how the stage-1 accumulator already lies (column
// q2 on lane % 32, one q1 per register), so every accumulator register is stored as full 128-byte
// lines straight from the registers: no LDS, no barrier.  The last tile may hold fewer than ST rows.
template <int P, int ST, int NW>
__global__ __launch_bounds__(NW * 64, 2)
void mfma_pair_rows_sliced_multiply(const float* __restrict__ Xg, float* __restrict__ Yg,
                                    const float* __restrict__ F0, const float* __restrict__ F1,   // in order of application
                                    int64_t M, int64_t num_tiles, int64_t tiles_per_wg, int tile_order)
{
    typedef MfmaPairShape<P, ST, NW, 1, 2> Sh;
    constexpr int Q = Sh::Q, KS = Sh::KS, AP = Sh::AP, UPW = Sh::UPW;
    constexpr int KIN = P * P, KOUT = Q * Q;

    const int tid = threadIdx.x;
    const int lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int col = lane % 32;
    const int g = lane / 32;

    float b0[KS], a1[KS];
#pragma unroll
    for (int t = 0; t < KS; ++t) {
        b0[t] = F0[(g * KS + t) * Q + col];
        a1[t] = F1[(8 * (t / 4) + 4 * g + (t % 4)) * Q + col];
    }

    int64_t t_begin = (int64_t)blockIdx.x * tiles_per_wg, t_step = 1;
    int64_t t_end = t_begin + tiles_per_wg;
    if (tile_order == 2) {
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

    // this lane's piece of unit u: row (of the tile) a_loc + first row of the unit, elements from lane_off
    const int a_loc = (col * P) / KIN;                    // 0, or 0/1 when a unit holds two rows (P = 16)
    const unsigned lane_off = col * P + g * KS;           // = a_loc * KIN + p1 * P + g * KS
    auto load_unit = [&](int64_t t, int u, pair_f32x4 (&dst)[KS / 4]) {
        const int64_t row0 = t * ST + (wave + u * NW) * AP;                 // first row of the unit
        const float* src = Xg + row0 * KIN;
        const bool live = row0 + a_loc < M;
#pragma unroll
        for (int c = 0; c < KS / 4; ++c) {
            if (live) dst[c] = *reinterpret_cast<const pair_f32x4*>(src + (lane_off + 4 * c));
            else dst[c] = pair_f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };

    pair_f32x4 xa[2][KS / 4];
    if (t_begin < t_end) load_unit(t_begin, 0, xa[0]);
    for (int64_t t = t_begin; t < t_end; t += t_step) {
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            if (u + 1 < UPW) load_unit(t, u + 1, xa[(u + 1) % 2]);
            else if (t + t_step < t_end) load_unit(t + t_step, 0, xa[(u + 1) % 2]);
            pair_f32x16 d0;
#pragma unroll
            for (int v = 0; v < 16; ++v) d0[v] = 0.f;
#pragma unroll
            for (int s = 0; s < KS; ++s)
                d0 = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[u % 2][s / 4][s % 4], b0[s], d0, 0, 0, 0);
#pragma unroll
            for (int al = 0; al < AP; ++al) {
                pair_f32x16 acc;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
                for (int s = 0; s < KS; ++s)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[s], d0[al * KS + s], acc, 0, 0, 0);
                const int64_t row = t * ST + (wave + u * NW) * AP + al;
                if (row < M) {
                    float* dst = Yg + row * KOUT + col;
#pragma unroll
                    for (int w = 0; w < 16; ++w) {
                        const int q1 = 8 * (w / 4) + 4 * g + (w % 4);
                        stream_store(acc[w], &dst[q1 * Q]);
                    }
                }
            }
        }
    }
}

}  // namespace km
