// One sliced-multiply iteration for any factor shape (Algorithm 1, inner loops; the four steps of
// the kernel in section 4: global->LDS, LDS->registers, multiply-accumulate, permuted store).
//
// A workgroup owns GEN_TS consecutive slices and walks the factor columns in groups of GEN_TQ and
// the slice elements in chunks of GEN_TP.  Slices are numbered through all rows (row r, slice s is
// slice r*S + s and starts at element (r*S + s)*P of X, rows being contiguous), so a tile may span
// rows and short rows (S small, down to one slice per row when N = 1) still fill the workgroup.  Lanes run along the slice index, so for a
// fixed factor column a wavefront stores one contiguous run of the output row: the output column of
// (slice s, column q) is q*(K/P)+s.  A thread keeps GEN_RS slices x GEN_QR consecutive columns in
// registers; per 16-byte read of its slices' elements it reads the matching factor rows, which are
// wave-uniform (broadcast reads).  Every access is bounds-checked: no divisibility is assumed.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "fused_kernel.hpp"   // Vec16

namespace km {

constexpr int GEN_RS = 2;                  // slices per thread
constexpr int GEN_TS = 64 * GEN_RS;        // slices per workgroup
constexpr int GEN_QW = 4;                  // wavefronts per workgroup, each takes GEN_QR columns of a group
constexpr int GEN_QR = 8;                  // columns per thread
constexpr int GEN_TQ = GEN_QW * GEN_QR;    // factor columns per pass
constexpr int GEN_TP = 16;                 // slice elements staged per chunk
constexpr int GEN_THREADS = 64 * GEN_QW;

template <typename T>
constexpr int gen_lds_bytes()
{
    return (int)sizeof(T) * (GEN_TS * (GEN_TP + Vec16<T>::N) + GEN_TP * GEN_TQ);
}

template <typename T>
__global__ __launch_bounds__(GEN_THREADS)
void sliced_multiply_generic(const T* __restrict__ Xg, const T* __restrict__ Fg, T* __restrict__ Yg,
                             int64_t K, int P, int Q, int64_t num_slices, int64_t num_tiles)
{
    typedef typename Vec16<T>::type V;
    constexpr int VN = Vec16<T>::N;
    constexpr int XROW = GEN_TP + VN;      // padded: 16-byte reads of consecutive lanes spread over the banks
    __shared__ __attribute__((aligned(16))) T Xs[GEN_TS][XROW];
    __shared__ __attribute__((aligned(16))) T Fs[GEN_TP][GEN_TQ];

    const int64_t S = K / P;
    const int tid = threadIdx.x;
    const int lane = tid % 64, wave = tid / 64;
    // 16-byte global loads are possible when every slice chunk starts on a 16-byte boundary
    const bool vec_ok = (P % VN == 0) && (K % VN == 0);

    // the grid may be smaller than the number of tiles (launches are limited to 2^32 work-items)
    for (int64_t tile = blockIdx.x; tile < num_tiles; tile += gridDim.x) {
        const int64_t g0 = tile * GEN_TS;                // first slice of the tile, counted through all rows
        for (int q0 = 0; q0 < Q; q0 += GEN_TQ) {
            T acc[GEN_RS][GEN_QR];
#pragma unroll
            for (int r = 0; r < GEN_RS; ++r)
#pragma unroll
                for (int j = 0; j < GEN_QR; ++j) acc[r][j] = T(0);

            for (int p0 = 0; p0 < P; p0 += GEN_TP) {
                // stage GEN_TS x GEN_TP elements of X: thread t takes half a chunk row (8 elements) of slice t/2
                {
                    const int s = tid / 2;
                    const int pp = (tid % 2) * (GEN_TP / 2);
                    const bool live = g0 + s < num_slices;
                    const T* src = Xg + (g0 + s) * P + p0 + pp;
                    if (live && vec_ok && p0 + pp + GEN_TP / 2 <= P) {
#pragma unroll
                        for (int c = 0; c < GEN_TP / 2 / VN; ++c)
                            *reinterpret_cast<V*>(&Xs[s][pp + c * VN]) = reinterpret_cast<const V*>(src)[c];
                    } else {
#pragma unroll
                        for (int e = 0; e < GEN_TP / 2; ++e)
                            Xs[s][pp + e] = (live && p0 + pp + e < P) ? src[e] : T(0);
                    }
                }
                // stage GEN_TP x GEN_TQ elements of F
                for (int e = tid; e < GEN_TP * GEN_TQ; e += GEN_THREADS) {
                    const int p = e / GEN_TQ, q = e % GEN_TQ;
                    Fs[p][q] = (p0 + p < P && q0 + q < Q) ? Fg[(int64_t)(p0 + p) * Q + q0 + q] : T(0);
                }
                __syncthreads();
#pragma unroll
                for (int pv = 0; pv < GEN_TP; pv += VN) {
                    V x[GEN_RS];
#pragma unroll
                    for (int r = 0; r < GEN_RS; ++r) x[r] = *reinterpret_cast<const V*>(&Xs[lane + 64 * r][pv]);
#pragma unroll
                    for (int e = 0; e < VN; ++e) {
                        T f[GEN_QR];
#pragma unroll
                        for (int c = 0; c < GEN_QR / VN; ++c) {
                            const V fv = *reinterpret_cast<const V*>(&Fs[pv + e][wave * GEN_QR + c * VN]);
#pragma unroll
                            for (int k = 0; k < VN; ++k) f[c * VN + k] = fv[k];
                        }
#pragma unroll
                        for (int r = 0; r < GEN_RS; ++r)
#pragma unroll
                            for (int j = 0; j < GEN_QR; ++j) acc[r][j] += x[r][e] * f[j];
                    }
                }
                __syncthreads();
            }
#pragma unroll
            for (int r = 0; r < GEN_RS; ++r) {
                const int64_t g = g0 + lane + 64 * r;
                if (g < num_slices) {
                    T* Yrow = Yg + (g / S) * (S * Q) + g % S;        // row of the slice, and the slice within it
#pragma unroll
                    for (int j = 0; j < GEN_QR; ++j) {
                        const int q = q0 + wave * GEN_QR + j;
                        if (q < Q) Yrow[(int64_t)q * S] = acc[r][j];
                    }
                }
            }
        }
    }
}

}  // namespace km
