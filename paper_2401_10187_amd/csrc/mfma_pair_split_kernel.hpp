// The register-chained pair of sliced multiplies of mfma_pair_kernel.hpp with the work of a
// workgroup split between two kinds of wavefronts (fp32, P x 32 factors, P = 16 or 32).
//
// Waves 0-3 ("compute", one per SIMD) load X, run both MFMA stages and leave the results in LDS;
// waves 4-7 ("store", one per SIMD) copy finished results from LDS to global memory.  The two kinds
// never wait for each other's memory operations: a compute wave's loads are not queued behind
// stores, and the stores of one tile drain while the next tile is being multiplied.
//
// LDS holds two staging buffers of half a tile's output each (q1 < 16 in A, q1 >= 16 in B; rows
// (q1, q2) of ST values along `a`, as in mfma_pair_kernel.hpp).  Per tile:
//
//   compute waves                              store waves
//   MFMA units: q1 < 16 half -> A,             (storing B of the previous tile)
//               q1 >= 16 half kept in registers
//   ---------------------------------- barrier 1 ----------------------------------
//   kept half -> B                             A -> global
//   ---------------------------------- barrier 2 ----------------------------------
//   next tile's MFMA units -> A                B -> global
//
// A is written only between barrier 2 and barrier 1 and read only between barrier 1 and barrier 2;
// B the other way round.  Every wave passes the same two barriers per tile.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "fused_kernel.hpp"        // stream_store
#include "mfma_pair_kernel.hpp"    // pair_f32x4, pair_f32x16

namespace km {

template <int P, int ST, int PD>
struct MfmaPairSplitShape {
    static constexpr int Q = 32;
    static constexpr int NWC = 4, NWS = 4;             // compute and store wavefronts
    static constexpr int NT = (NWC + NWS) * 64;
    static constexpr int AP = 32 / P;                  // values of `a` per 32-row stage-0 product
    static constexpr int KS = P / 2;                   // MFMA steps per product
    static constexpr int UNITS = ST / AP;              // stage-0 products per tile
    static constexpr int UPW = UNITS / NWC;            // ... per compute wavefront
    static constexpr int APW = UPW * AP;               // values of `a` per compute wavefront
    static constexpr int TK = ST * P * P;
    static constexpr int STP = ST + 4;                 // padded row of a staging buffer
    static constexpr int PASS_ROWS = 16 * Q;           // rows (q1_local, q2) of one buffer
    static constexpr int BUF_ELEMS = PASS_ROWS * STP;
    static constexpr int LDS_BYTES = 2 * BUF_ELEMS * 4;
    static constexpr int RD = PASS_ROWS * (ST / 4) / (NWS * 64);   // 16-byte reads per store thread and buffer
    static constexpr int RING = PD + 1;
    static_assert(P == 16 || P == 32, "P must be 16 or 32");
    static_assert(ST % (AP * NWC) == 0 && ST % 4 == 0, "tile must split evenly over the compute wavefronts");
    static_assert((PASS_ROWS * (ST / 4)) % (NWS * 64) == 0 && RD % 4 == 0, "buffer must split evenly over the store threads");
    static_assert(PD >= 1 && PD < UPW && UPW % RING == 0, "the operand ring must wrap once per tile");
};

template <int P, int ST, int PD>
__global__ __launch_bounds__(512, 2)
void mfma_pair_split_sliced_multiply(const float* __restrict__ Xg, float* __restrict__ Yg,
                                     const float* __restrict__ F0, const float* __restrict__ F1,   // in order of application
                                     int64_t k_in, int64_t k_out, int64_t tiles_per_row, int64_t num_tiles,
                                     int64_t tiles_per_wg, int tile_order)
{
    typedef MfmaPairSplitShape<P, ST, PD> Sh;
    constexpr int Q = Sh::Q, KS = Sh::KS, AP = Sh::AP, UPW = Sh::UPW, STP = Sh::STP, RING = Sh::RING, NWC = Sh::NWC;
    extern __shared__ __attribute__((aligned(16))) unsigned char pair_split_lds[];
    float* buf_a = reinterpret_cast<float*>(pair_split_lds);
    float* buf_b = buf_a + Sh::BUF_ELEMS;

    const int tid = threadIdx.x;
    const int lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);    // wave-uniform

    const int64_t s_row = tiles_per_row * ST;
    // tile walk as in mfma_pair_kernel.hpp
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
    auto uniform = [](int64_t v) {
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
        const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
        return (int64_t)(((uint64_t)hi << 32) | lo);
    };

    if (wave < NWC) {
        // ---------------------------------------------------------------- compute wavefronts
        const int col = lane % 32;        // stage 0: row (a_loc, p1) of A, column q2 of B; stage 1: row q1 of A
        const int g = lane / 32;          // which of the two k values of an MFMA step this lane holds
        float b0[KS], a1[KS];
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            b0[t] = F0[(g * KS + t) * Q + col];
            a1[t] = F1[(8 * (t / 4) + 4 * g + (t % 4)) * Q + col];
        }
        const unsigned lane_off = col * P + g * KS;
        auto tile_src = [&](int64_t t) {
            return Xg + uniform(t / tiles_per_row) * k_in + uniform(t % tiles_per_row) * Sh::TK;
        };
        pair_f32x4 xa[RING][KS / 4];
        if (t_begin < t_end) {
#pragma unroll
            for (int v = 0; v < PD; ++v) {
                const float* src = tile_src(t_begin) + ((wave + v * NWC) * AP) * P * P;
#pragma unroll
                for (int c = 0; c < KS / 4; ++c) xa[v][c] = *reinterpret_cast<const pair_f32x4*>(src + (lane_off + 4 * c));
            }
        }
        for (int64_t t = t_begin; t < t_end; t += t_step) {
            const float* Xt = tile_src(t);
            float keep[Sh::APW][8];
#pragma unroll
            for (int u = 0; u < UPW; ++u) {
                {
                    const int v = u + PD;
                    if (v < UPW) {
                        const float* src = Xt + ((wave + v * NWC) * AP) * P * P;
#pragma unroll
                        for (int c = 0; c < KS / 4; ++c)
                            xa[v % RING][c] = *reinterpret_cast<const pair_f32x4*>(src + (lane_off + 4 * c));
                    } else if (t + t_step < t_end) {
                        const float* src = tile_src(t + t_step) + ((wave + (v - UPW) * NWC) * AP) * P * P;
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
                    const int a = (wave + u * NWC) * AP + al;
#pragma unroll
                    for (int w = 0; w < 8; ++w) {
                        const int q1l = 8 * (w / 4) + 4 * g + (w % 4);           // q1 of register w (and of 8 + w, minus 16)
                        buf_a[(q1l * Q + col) * STP + a] = acc[w];
                        keep[u * AP + al][w] = acc[8 + w];
                    }
                }
            }
            __syncthreads();                              // barrier 1: A is complete, B has been stored
#pragma unroll
            for (int u = 0; u < UPW; ++u)
#pragma unroll
                for (int al = 0; al < AP; ++al) {
                    const int a = (wave + u * NWC) * AP + al;
#pragma unroll
                    for (int w = 0; w < 8; ++w) {
                        const int q1l = 8 * (w / 4) + 4 * g + (w % 4);
                        buf_b[(q1l * Q + col) * STP + a] = keep[u * AP + al][w];
                    }
                }
            __syncthreads();                              // barrier 2: B is complete, A has been stored
        }
    } else {
        // ---------------------------------------------------------------- store wavefronts
        const int stid = tid - NWC * 64;
        constexpr int SNT = Sh::NWS * 64;
        for (int64_t t = t_begin; t < t_end; t += t_step) {
            const int64_t row = uniform(t / tiles_per_row), h = uniform(t % tiles_per_row);
            float* Yrow = Yg + row * k_out + h * ST;
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
                __syncthreads();                          // barrier 1 (pass 0) / barrier 2 (pass 1)
                const float* buf = pass == 0 ? buf_a : buf_b;
                // row r = (q1l, q2) of the buffer -> output column ((16*pass + q1l)*Q + q2)*s_row + h*ST + a
                float* Ypass = Yrow + (int64_t)(16 * pass * Q) * s_row;
#pragma unroll
                for (int i0 = 0; i0 < Sh::RD; i0 += 4) {
                    pair_f32x4 v[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int idx = stid + (i0 + i) * SNT;
                        v[i] = *reinterpret_cast<const pair_f32x4*>(buf + (idx / (ST / 4)) * STP + 4 * (idx % (ST / 4)));
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int idx = stid + (i0 + i) * SNT;
                        stream_store(v[i], reinterpret_cast<pair_f32x4*>(Ypass + (int64_t)(idx / (ST / 4)) * s_row + 4 * (idx % (ST / 4))));
                    }
                }
            }
        }
    }
}

}  // namespace km
