// One sliced-multiply iteration for any factor shape (Algorithm 1, inner loops; the four steps of
// the kernel in section 4: global->LDS, LDS->registers, multiply-accumulate, permuted store).
//
// A unit of work is GEN_TS consecutive slices times GEN_TQ consecutive factor columns; workgroups
// stride over the units, units of the same slices being numbered so that they run on the same XCD
// (they share the slices through its L2 cache), so that small problems still spread over many
// compute units.  Within a unit the
// slice elements are walked in chunks of GEN_TP: the next chunk of X and F is fetched into registers
// while the current one is multiplied out of LDS, and two LDS buffers leave one barrier per chunk.
// Slices are numbered through all rows (row r, slice s is slice r*S + s and starts at element
// (r*S + s)*P of X, rows being contiguous), so a tile may span rows and short rows (S small, down to
// one slice per row when N = 1) still fill the workgroup.  Lanes run along the slice index, so for a
// fixed factor column a wavefront stores one contiguous run of the output row: the output column of
// (slice s, column q) is q*(K/P)+s.  A thread keeps GEN_RS slices x GEN_QR consecutive columns in
// registers; per 16-byte read of its slices' elements it reads the matching factor rows, which are
// wave-uniform (broadcast reads).  Every access is bounds-checked: no divisibility is assumed.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "fused_kernel.hpp"   // Vec16
#include "plan.hpp"           // unit_of

namespace km {

constexpr int GEN_RS = 2;                  // slices per thread
constexpr int GEN_TS = 64 * GEN_RS;        // slices per workgroup
constexpr int GEN_QW = 4;                  // wavefronts per workgroup, each takes GEN_QR columns of a group
constexpr int GEN_QR = 8;                  // columns per thread
constexpr int GEN_TQ = GEN_QW * GEN_QR;    // factor columns per unit
constexpr int GEN_TP = 16;                 // slice elements staged per chunk
constexpr int GEN_THREADS = 64 * GEN_QW;
constexpr int GEN_FR = GEN_TP * GEN_TQ / GEN_THREADS;   // factor elements staged per thread and chunk

template <typename T>
constexpr int gen_lds_bytes()
{
    return 2 * (int)sizeof(T) * (GEN_TS * (GEN_TP + Vec16<T>::N) + GEN_TP * GEN_TQ);
}

template <typename T>
__global__ __launch_bounds__(GEN_THREADS)
void sliced_multiply_generic(const T* __restrict__ Xg, const T* __restrict__ Fg, T* __restrict__ Yg,
                             int64_t K, int P, int Q, int64_t num_slices, int64_t num_units)
{
    typedef typename Vec16<T>::type V;
    constexpr int VN = Vec16<T>::N;
    constexpr int XROW = GEN_TP + VN;      // padded: 16-byte reads of consecutive lanes spread over the banks
    constexpr int XV = GEN_TP / 2 / VN;    // 16-byte vectors of X per thread and chunk
    __shared__ __attribute__((aligned(16))) T Xs[2][GEN_TS][XROW];
    __shared__ __attribute__((aligned(16))) T Fs[2][GEN_TP][GEN_TQ];

    const int64_t S = K / P;
    const int tid = threadIdx.x;
    const int lane = tid % 64, wave = tid / 64;
    // 16-byte global loads are possible when every slice chunk starts on a 16-byte boundary
    const bool vec_ok = (P % VN == 0) && (K % VN == 0);
    const int q_groups = (Q + GEN_TQ - 1) / GEN_TQ;
    // staging duty of this thread: half a chunk row (GEN_TP/2 elements) of slice tid/2 ...
    const int xs = tid / 2, xp = (tid % 2) * (GEN_TP / 2);

    // the grid may be smaller than the number of units (launches are limited to 2^32 work-items)
    for (int64_t unit = blockIdx.x; unit < num_units; unit += gridDim.x) {
        int64_t tile;
        int group;
        unit_of(unit, num_units / q_groups, q_groups, tile, group);
        const int64_t g0 = tile * GEN_TS;                // first slice of the unit, counted through all rows
        const int q0 = group * GEN_TQ;
        const bool live = g0 + xs < num_slices;
        const T* xsrc = Xg + (g0 + xs) * P + xp;

        V xr[XV];
        T fr[GEN_FR];
        auto fetch = [&](int p0) {
            if (live && vec_ok && p0 + xp + GEN_TP / 2 <= P) {
#pragma unroll
                for (int c = 0; c < XV; ++c) xr[c] = reinterpret_cast<const V*>(xsrc + p0)[c];
            } else {
#pragma unroll
                for (int c = 0; c < XV; ++c)
#pragma unroll
                    for (int e = 0; e < VN; ++e)
                        xr[c][e] = (live && p0 + xp + c * VN + e < P) ? xsrc[p0 + c * VN + e] : T(0);
            }
            // ... and GEN_FR elements of the factor chunk
#pragma unroll
            for (int i = 0; i < GEN_FR; ++i) {
                const int e = tid + i * GEN_THREADS;
                const int p = e / GEN_TQ, q = e % GEN_TQ;
                fr[i] = (p0 + p < P && q0 + q < Q) ? Fg[(int64_t)(p0 + p) * Q + q0 + q] : T(0);
            }
        };

        T acc[GEN_RS][GEN_QR];
#pragma unroll
        for (int r = 0; r < GEN_RS; ++r)
#pragma unroll
            for (int j = 0; j < GEN_QR; ++j) acc[r][j] = T(0);

        fetch(0);
        int buf = 0;
        for (int p0 = 0; p0 < P; p0 += GEN_TP) {
            // A buffer is rewritten two chunks after it was read; the barrier of the chunk in between
            // orders the two.  (Across units: the last chunk's readers and the next unit's first
            // writers use different buffers or are separated by the barrier below.)
#pragma unroll
            for (int c = 0; c < XV; ++c) *reinterpret_cast<V*>(&Xs[buf][xs][xp + c * VN]) = xr[c];
#pragma unroll
            for (int i = 0; i < GEN_FR; ++i) {
                const int e = tid + i * GEN_THREADS;
                Fs[buf][e / GEN_TQ][e % GEN_TQ] = fr[i];
            }
            __syncthreads();
            if (p0 + GEN_TP < P) fetch(p0 + GEN_TP);
#pragma unroll
            for (int pv = 0; pv < GEN_TP; pv += VN) {
                V x[GEN_RS];
#pragma unroll
                for (int r = 0; r < GEN_RS; ++r) x[r] = *reinterpret_cast<const V*>(&Xs[buf][lane + 64 * r][pv]);
#pragma unroll
                for (int e = 0; e < VN; ++e) {
                    T f[GEN_QR];
#pragma unroll
                    for (int c = 0; c < GEN_QR / VN; ++c) {
                        const V fv = *reinterpret_cast<const V*>(&Fs[buf][pv + e][wave * GEN_QR + c * VN]);
#pragma unroll
                        for (int k = 0; k < VN; ++k) f[c * VN + k] = fv[k];
                    }
#pragma unroll
                    for (int r = 0; r < GEN_RS; ++r)
#pragma unroll
                        for (int j = 0; j < GEN_QR; ++j) acc[r][j] += x[r][e] * f[j];
                }
            }
            buf ^= 1;
        }
        __syncthreads();      // the next unit starts writing at buffer 0 again, whatever the chunk count was
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

}  // namespace km
