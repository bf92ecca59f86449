// Fused sliced multiplies with the tile resident in LDS (section 4.2 of the paper).
//
// A workgroup takes one contiguous tile of T_K = ST * P^NF elements of one row, applies NF
// consecutive P x Q factors to it (each application is the sliced multiply of Algorithm 1 restricted
// to the tile: slice s, column q -> local position q*S + s) and scatters the result: the tile's
// final contents, ordered (fused column qq, slice r < ST), go to column qq*(K_in/P^NF) + h*ST + r of
// the output row, h being the tile's index in the row (the store of Figure 7).
//
// gfx950 mapping, which differs from the paper's register/shared-memory tiling:
//  * every thread owns whole slices: it reads the P contiguous elements of a slice from LDS with
//    16-byte reads and keeps all Q results of that slice in registers; lanes run along the slice
//    index, so LDS writes (stride 1 between lanes) and the global stores of one factor column are
//    contiguous across a wavefront;
//  * factor elements are wave-uniform, so they are fetched with scalar loads (constant address
//    space) and used as the scalar operand of the FMA: no LDS or vector registers are spent on F;
//  * the tile is updated in place: all reads of a stage, barrier, all writes, barrier.
//  * workgroup ids are remapped so that the tiles of one row, whose partial output lines interleave,
//    run on the same XCD (one L2) at about the same time.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace km {

constexpr int64_t ipow(int64_t b, int e) { return e <= 0 ? 1 : b * ipow(b, e - 1); }
constexpr int64_t cmax(int64_t a, int64_t b) { return a > b ? a : b; }

// 16-byte vectors (native vector types, so that arrays of them stay in registers)
template <typename T> struct Vec16;
template <> struct Vec16<float> { typedef float type __attribute__((ext_vector_type(4))); static constexpr int N = 4; };
template <> struct Vec16<double> { typedef double type __attribute__((ext_vector_type(2))); static constexpr int N = 2; };

// X is read once and Y written once per launch: non-temporal accesses (measured 7 % faster than
// default caching on the 8x8 workload).
template <typename V> __device__ __forceinline__ V stream_load(const V* p) { return __builtin_nontemporal_load(p); }
template <typename V> __device__ __forceinline__ void stream_store(V v, V* p) { __builtin_nontemporal_store(v, p); }
// Output that the next launch reads back and that fits the chip's last-level cache (256 MB) is
// written with ordinary stores instead (KEEP): the next launch then finds part of it on chip
// (measured: 16 x 128x128^3 fp64 0.462 -> 0.437 ms, 256 x 8x8^6 0.198 -> 0.190; beyond 400 MB per
// launch ordinary stores are 2-8 % slower than non-temporal ones).
template <bool KEEP, typename V> __device__ __forceinline__ void out_store(V v, V* p)
{
    if constexpr (KEEP) *p = v;
    else __builtin_nontemporal_store(v, p);
}

// read-only data that is uniform across a wavefront: scalar loads
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wold-style-cast"
template <typename T>
__device__ __forceinline__ const T __attribute__((address_space(4)))* as_constant(const T* p)
{
    return (const T __attribute__((address_space(4)))*)p;
}
#pragma clang diagnostic pop

// XCD-aware order: workgroup b runs on XCD b % 8; each XCD gets a contiguous range of tiles (the first
// num_tiles % 8 ranges one tile longer), so that the tiles of one row, whose partial output lines
// interleave, meet in one L2 (1010 x 9^6, 81810 tiles of 36-byte runs: 4.79 ms per Kron-Matmul while
// only tile counts divisible by 8 were reordered, 2000 rows of the same took 4.45).
__device__ __forceinline__ int64_t xcd_contiguous_tile(int64_t b, int64_t num_tiles)
{
    const int64_t base = num_tiles / 8, rem = num_tiles % 8, x = b % 8;
    return x * base + (x < rem ? x : rem) + b / 8;
}

template <typename T, int P, int Q, int NF, int ST, int NT>
struct FusedShape {
    static constexpr int size(int j) { return (int)(ST * ipow(P, NF - j) * ipow(Q, j)); }   // tile elements after j factors
    static constexpr int TK = size(0);
    static constexpr int lds_elems()
    {
        int m = 0;
        for (int j = 0; j < NF; ++j) m = size(j) > m ? size(j) : m;
        return m;
    }
    static constexpr int LDS_BYTES = lds_elems() * (int)sizeof(T);
    static constexpr int VN = Vec16<T>::N;
    static constexpr bool VEC_TILE = TK % VN == 0;     // tile start stays 16-byte aligned
    static constexpr bool VEC_SLICE = P % VN == 0;     // a slice is a whole number of 16-byte vectors
};

// One stage: factor `Fc` applied to the tile held in `tile` (size(J) elements).
template <typename T, int P, int Q, int NF, int ST, int NT, int J, bool KEEP>
__device__ __forceinline__ void fused_stage(T* __restrict__ tile, const T* Fg, T* __restrict__ Yrow,
                                            int64_t s_row, int64_t h)
{
    typedef FusedShape<T, P, Q, NF, ST, NT> Sh;
    typedef typename Vec16<T>::type V;
    constexpr int VN = Sh::VN;
    constexpr int SJ = Sh::size(J) / P;                 // slices in the tile at this stage
    constexpr int R = (SJ + NT - 1) / NT;               // slices per thread
    constexpr bool FULL = SJ % NT == 0;
    constexpr bool LAST = J == NF - 1;
    const auto Fc = as_constant(Fg);
    const int tid = threadIdx.x;

    T out[R][Q];
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int s = tid + i * NT;
        T x[P];
        if (FULL || s < SJ) {
            if constexpr (Sh::VEC_SLICE) {
                const V* src = reinterpret_cast<const V*>(tile + s * P);
#pragma unroll
                for (int c = 0; c < P / VN; ++c) {
                    const V v = src[c];
#pragma unroll
                    for (int e = 0; e < VN; ++e) x[VN * c + e] = v[e];
                }
            } else {
#pragma unroll
                for (int p = 0; p < P; ++p) x[p] = tile[s * P + p];
            }
        } else {
#pragma unroll
            for (int p = 0; p < P; ++p) x[p] = T(0);
        }
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            T acc = x[0] * Fc[q];
#pragma unroll
            for (int p = 1; p < P; ++p) acc += x[p] * Fc[p * Q + q];
            out[i][q] = acc;
        }
    }
    if constexpr (!LAST) {
        __syncthreads();                                 // every slice has been read
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int s = tid + i * NT;
            if (FULL || s < SJ) {
#pragma unroll
                for (int q = 0; q < Q; ++q) tile[q * SJ + s] = out[i][q];
            }
        }
        __syncthreads();
    } else {
        // local (q, s) with s = qq_rest*ST + r  ->  column (q*Q^(NF-1) + qq_rest)*s_row + h*ST + r
        // One 64-bit pointer per slice, advanced by a wave-uniform stride per column (measured faster
        // than 32-bit offsets from the row base).
        constexpr int QREST = (int)ipow(Q, NF - 1);
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int s = tid + i * NT;
            if (FULL || s < SJ) {
                T* dst = Yrow + (int64_t)(s / ST) * s_row + h * ST + (s % ST);
#pragma unroll
                for (int q = 0; q < Q; ++q) out_store<KEEP>(out[i][q], &dst[(int64_t)(q * QREST) * s_row]);
            }
        }
    }
}

template <typename T, int P, int Q, int NF, int ST, int NT, bool KEEP>
__global__ __launch_bounds__(NT)
void fused_sliced_multiply(const T* __restrict__ Xg, T* __restrict__ Yg,
                           const T* F0, const T* F1, const T* F2,   // in order of application
                           int64_t k_in, int64_t k_out, int64_t tiles_per_row, int64_t num_tiles)
{
    typedef FusedShape<T, P, Q, NF, ST, NT> Sh;
    typedef typename Vec16<T>::type V;
    constexpr int VN = Sh::VN;
    extern __shared__ __attribute__((aligned(16))) unsigned char fused_lds[];
    T* tile = reinterpret_cast<T*>(fused_lds);

    const int64_t t = xcd_contiguous_tile(blockIdx.x, num_tiles);
    const int64_t row = t / tiles_per_row;
    const int64_t h = t % tiles_per_row;
    const T* src = Xg + row * k_in + h * Sh::TK;
    T* Yrow = Yg + row * k_out;
    const int64_t s_row = tiles_per_row * ST;           // K_in / P^NF
    const int tid = threadIdx.x;

    if constexpr (Sh::VEC_TILE) {
        constexpr int NV = Sh::TK / VN;
        constexpr int RV = (NV + NT - 1) / NT;
        V tmp[RV];
#pragma unroll
        for (int i = 0; i < RV; ++i) {
            const int v = tid + i * NT;
            if (NV % NT == 0 || v < NV) tmp[i] = stream_load(&reinterpret_cast<const V*>(src)[v]);
        }
#pragma unroll
        for (int i = 0; i < RV; ++i) {
            const int v = tid + i * NT;
            if (NV % NT == 0 || v < NV) reinterpret_cast<V*>(tile)[v] = tmp[i];
        }
    } else {
        for (int e = tid; e < Sh::TK; e += NT) tile[e] = src[e];
    }
    __syncthreads();

    fused_stage<T, P, Q, NF, ST, NT, 0, KEEP>(tile, F0, Yrow, s_row, h);
    if constexpr (NF > 1) fused_stage<T, P, Q, NF, ST, NT, 1, KEEP>(tile, F1, Yrow, s_row, h);
    if constexpr (NF > 2) fused_stage<T, P, Q, NF, ST, NT, 2, KEEP>(tile, F2, Yrow, s_row, h);
}

}  // namespace km
