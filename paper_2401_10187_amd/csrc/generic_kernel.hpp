// One sliced-multiply iteration for any factor shape (Algorithm 1, inner loops; the four steps of
// the kernel in section 4: global->LDS, LDS->registers, multiply-accumulate, permuted store).
//
// A workgroup owns GEN_TS consecutive slices of one row and walks the factor columns in groups of
// GEN_TQ and the slice elements in chunks of GEN_TP.  Lanes run along the slice index, so for a
// fixed factor column a wavefront stores one contiguous run of the output row: the output column of
// (slice s, column q) is q*(K/P)+s.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace km {

constexpr int GEN_TS = 64;     // slices per workgroup (one per lane of a wavefront)
constexpr int GEN_QL = 4;      // wavefronts per workgroup, each takes every 4th column of a group
constexpr int GEN_QR = 8;      // accumulators per thread
constexpr int GEN_TQ = GEN_QL * GEN_QR;   // factor columns per pass
constexpr int GEN_TP = 16;     // slice elements staged per chunk
constexpr int GEN_THREADS = GEN_TS * GEN_QL;

template <typename T>
__global__ __launch_bounds__(GEN_THREADS)
void sliced_multiply_generic(const T* __restrict__ Xg, const T* __restrict__ Fg, T* __restrict__ Yg,
                             int64_t K, int P, int Q, int64_t tiles_per_row)
{
    __shared__ T Xs[GEN_TS][GEN_TP + 1];
    __shared__ T Fs[GEN_TP][GEN_TQ];

    const int64_t S = K / P;
    const int64_t row = blockIdx.x / tiles_per_row;
    const int64_t s0 = (blockIdx.x % tiles_per_row) * GEN_TS;
    const int tid = threadIdx.x;
    const int sl = tid % GEN_TS;          // slice within the tile
    const int ql = tid / GEN_TS;          // column lane
    const T* Xrow = Xg + row * K;
    T* Yrow = Yg + row * (S * Q);

    for (int q0 = 0; q0 < Q; q0 += GEN_TQ) {
        T acc[GEN_QR];
#pragma unroll
        for (int i = 0; i < GEN_QR; ++i) acc[i] = T(0);

        for (int p0 = 0; p0 < P; p0 += GEN_TP) {
            // stage GEN_TS x GEN_TP elements of X: thread t takes 4 consecutive elements of a slice
            {
                const int s = tid / (GEN_TP / 4);
                const int pp = (tid % (GEN_TP / 4)) * 4;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int p = p0 + pp + e;
                    T v = T(0);
                    if (s0 + s < S && p < P) v = Xrow[(s0 + s) * P + p];
                    Xs[s][pp + e] = v;
                }
            }
            // stage GEN_TP x GEN_TQ elements of F
            for (int e = tid; e < GEN_TP * GEN_TQ; e += GEN_THREADS) {
                const int p = e / GEN_TQ, q = e % GEN_TQ;
                T v = T(0);
                if (p0 + p < P && q0 + q < Q) v = Fg[(int64_t)(p0 + p) * Q + q0 + q];
                Fs[p][q] = v;
            }
            __syncthreads();
#pragma unroll
            for (int p = 0; p < GEN_TP; ++p) {
                const T x = Xs[sl][p];
#pragma unroll
                for (int i = 0; i < GEN_QR; ++i) acc[i] += x * Fs[p][ql + i * GEN_QL];
            }
            __syncthreads();
        }
        if (s0 + sl < S) {
#pragma unroll
            for (int i = 0; i < GEN_QR; ++i) {
                const int q = q0 + ql + i * GEN_QL;
                if (q < Q) Yrow[(int64_t)q * S + s0 + sl] = acc[i];
            }
        }
    }
}

}  // namespace km
