// Launcher of the run-time-shape MFMA kernel (declared in launch.hpp).
#pragma once
#include "launch.hpp"
#include "mfma_any_kernel.hpp"

namespace km {

template <typename T, int CB, bool NARROW, bool KEEP, int FLAT>
static hipError_t launch_mfma_any_shape(const LaunchArgs& a, int64_t slices)
{
    typedef AnyShape<T, CB, NARROW> Sh;
    const km_plan_step& st = *a.st;
    const int f = st.first_factor;
    auto kern = mfma_any_sliced_multiply<T, CB, NARROW, KEEP, FLAT>;
    static unsigned char lds_ok[64];
    hipError_t e = allow_lds((const void*)kern, Sh::LDS_BYTES, lds_ok);
    if (e != hipSuccess || a.prepare_only) return e;
    const int Q = a.pr->Q[f];
    if (FLAT == 0 ? a.pr->P[f] % Sh::VN != 0 : (FLAT == 1 && a.pr->P[f] > Sh::KT)) return hipErrorInvalidValue;
    const int64_t units = ((slices + Sh::TS - 1) / Sh::TS) * ((Q + Sh::QG - 1) / Sh::QG);
    if (st.lds_bytes != Sh::LDS_BYTES || st.tile_slices != Sh::TS || st.grid < 1 || st.grid > units) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)st.grid), dim3(ANY_THREADS), Sh::LDS_BYTES, a.stream,
                       (const T*)a.src, (const T*)a.factors[f], (T*)a.dst, st.k_in, a.pr->P[f], a.pr->Q[f], slices, units,
                       (int)(((uintptr_t)a.factors[f] & 15) == 0 && a.pr->Q[f] % Sh::VN == 0));
    return hipGetLastError();
}

template <typename T, int CB>
static hipError_t launch_mfma_any_cb(const LaunchArgs& a, int64_t slices)
{
    // slices of at most half a wide chunk take the narrow shape
    const bool narrow = (size_t)a.pr->P[a.st->first_factor] * sizeof(T) * 2 <= (size_t)ANY_ROW_BYTES;
    // Output runs (16 or 32 consecutive slices of a column: 128 bytes) that do not start on 64-byte
    // boundaries would reach memory as partial lines if they bypassed the cache: ordinary stores
    // (measured: 1024 x 30x30^3 fp64 0.417 -> 0.348 ms, 8192 x 20x15^3 0.302 -> 0.237)
    const bool keep = a.keep_output || (a.st->k_in / a.pr->P[a.st->first_factor]) * (int64_t)sizeof(T) % 64 != 0;
    // slices that do not start on 16-byte boundaries: the form that fetches a unit as one contiguous run
    // when a slice is one chunk, the form of skewed chunk rows otherwise
    const int P = a.pr->P[a.st->first_factor];
    const int flat = P % (16 / (int)sizeof(T)) == 0 ? 0 : ((size_t)P * sizeof(T) <= (size_t)ANY_ROW_BYTES ? 1 : 2);
    hipError_t e = hipSuccess;
    for (int k = 0; k < 6 && e == hipSuccess; ++k) {
        const bool kp = (k & 1) != 0;
        const int fl = k >> 1;
        if (!a.prepare_only && (kp != keep || fl != flat)) continue;     // preparing takes every form
        if (narrow) {
            if (fl == 2) continue;                                       // (no skewed form of the narrow shape: its slices are one chunk)
            e = fl ? (kp ? launch_mfma_any_shape<T, CB, true, true, 1>(a, slices) : launch_mfma_any_shape<T, CB, true, false, 1>(a, slices))
                   : (kp ? launch_mfma_any_shape<T, CB, true, true, 0>(a, slices) : launch_mfma_any_shape<T, CB, true, false, 0>(a, slices));
        } else {
            e = fl == 2 ? (kp ? launch_mfma_any_shape<T, CB, false, true, 2>(a, slices) : launch_mfma_any_shape<T, CB, false, false, 2>(a, slices))
              : fl == 1 ? (kp ? launch_mfma_any_shape<T, CB, false, true, 1>(a, slices) : launch_mfma_any_shape<T, CB, false, false, 1>(a, slices))
                        : (kp ? launch_mfma_any_shape<T, CB, false, true, 0>(a, slices) : launch_mfma_any_shape<T, CB, false, false, 0>(a, slices));
        }
    }
    return e;
}

template <typename T>
hipError_t launch_mfma_any(const LaunchArgs& a)
{
    const km_plan_step& st = *a.st;
    const int f = st.first_factor;
    const int P = a.pr->P[f], Q = a.pr->Q[f];
    if (st.num_factors != 1 || st.k_in % P || st.block != ANY_THREADS) return hipErrorInvalidValue;
    const int64_t slices = a.pr->M * (st.k_in / P);      // counted through all rows
    const int cb = any_column_blocks(Q);
    switch (cb) {
        case 1: return launch_mfma_any_cb<T, 1>(a, slices);
        case 2: return launch_mfma_any_cb<T, 2>(a, slices);
        case 3: return launch_mfma_any_cb<T, 3>(a, slices);
        case 4: return launch_mfma_any_cb<T, 4>(a, slices);
        case 5: return launch_mfma_any_cb<T, 5>(a, slices);
    }
    return hipErrorInvalidValue;
}

}  // namespace km
