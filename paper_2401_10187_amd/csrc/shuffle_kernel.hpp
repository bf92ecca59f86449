// One sliced multiply with an 8x8 fp32 factor without LDS: the P-reduction is done with wavefront
// lane exchanges (DPP).
//
// Lanes map one to one onto the contiguous elements of X: lane l of a chunk loads 16 bytes, i.e.
// elements p = 4*(l%2) .. 4*(l%2)+3 of slice l/2, so global reads are perfectly coalesced and nothing
// is staged.  Each lane multiplies its four elements with the matching four rows of F (kept in
// registers) for all eight columns; the two lanes of a slice then add their partial sums with one
// quad-permute DPP exchange per column (the "reduction over P" of Algorithm 1's inner loop).  The
// even lane of the pair stores columns 0-3, the odd lane columns 4-7: for one register the even
// lanes of a wavefront hold 32 consecutive slices of one column, i.e. a contiguous 128-byte run of
// the output row (column q of slice s goes to q*(K/P) + s), and so do the odd lanes.
//
// This is the variant the shuffle idea pays for: a single factor.  A second factor would have to
// reduce across eight lane pairs (three exchange steps per column and register), which costs more
// vector instructions than the LDS exchange of fused_kernel.hpp.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "fused_kernel.hpp"   // stream_load / stream_store

namespace km {

constexpr int SHF_P = 8, SHF_Q = 8;
constexpr int SHF_NT = 256;            // threads per workgroup
constexpr int SHF_R = 4;               // 16-byte chunks per thread
constexpr int SHF_ST = SHF_NT * SHF_R * 4 / SHF_P;     // slices per workgroup tile (512)

typedef float shf_f32x4 __attribute__((ext_vector_type(4)));

// value of `v` in the other lane of the pair (lanes 2k and 2k+1): DPP quad_perm [1,0,3,2]
__device__ __forceinline__ float shf_pair_exchange(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
}

// (a template only so that the header can be included by several translation units)
template <int NT_>
__global__ __launch_bounds__(NT_)
void shuffle_sliced_multiply_8x8(const float* __restrict__ Xg, float* __restrict__ Yg,
                                 const float* __restrict__ Fg, int64_t k_in, int64_t tiles_per_row,
                                 int64_t num_tiles)
{
    constexpr int P = SHF_P, Q = SHF_Q, NT = NT_, R = SHF_R;
    static_assert(NT_ == SHF_NT, "one workgroup size");
    const int64_t t = xcd_contiguous_tile(blockIdx.x, num_tiles);
    const int64_t row = t / tiles_per_row;
    const int64_t h = t % tiles_per_row;
    const int64_t S = k_in / P;                            // slices per row; k_out = S * Q = k_in
    const int tid = threadIdx.x;
    const int half = tid & 1;                              // which four elements of the slice this lane holds

    // the four rows of F this lane multiplies with
    float f[4][Q];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int q = 0; q < Q; ++q) f[i][q] = Fg[(4 * half + i) * Q + q];

    const shf_f32x4* src = reinterpret_cast<const shf_f32x4*>(Xg + row * k_in + h * (SHF_ST * P));
    shf_f32x4 x[R];
#pragma unroll
    for (int r = 0; r < R; ++r) x[r] = stream_load(&src[tid + r * NT]);

    float* Yrow = Yg + row * k_in;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float mine[4];
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            float part = x[r][0] * f[0][q];
            part += x[r][1] * f[1][q];
            part += x[r][2] * f[2][q];
            part += x[r][3] * f[3][q];
            const float sum = part + shf_pair_exchange(part);     // both lanes of the slice now hold it
            if (q < 4) { if (!half) mine[q] = sum; }
            else       { if (half) mine[q - 4] = sum; }
        }
        // slice of this lane within the row, and its four columns 4*half + j
        const int64_t s = h * SHF_ST + (int64_t)(tid + r * NT) / 2;
        float* dst = Yrow + (int64_t)(4 * half) * S + s;
#pragma unroll
        for (int j = 0; j < 4; ++j) stream_store(mine[j], &dst[(int64_t)j * S]);
    }
}

}  // namespace km
