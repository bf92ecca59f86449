// Launcher of the run-time-shape MFMA kernel (declared in launch.hpp).
#pragma once
#include "launch.hpp"
#include "mfma_any_kernel.hpp"

namespace km {

template <typename T, int CB>
static hipError_t launch_mfma_any_cb(const LaunchArgs& a, int64_t slices, int64_t units)
{
    typedef AnyShape<T, CB> Sh;
    const km_plan_step& st = *a.st;
    const int f = st.first_factor;
    auto kern = mfma_any_sliced_multiply<T, CB>;
    static unsigned char lds_ok[64];
    hipError_t e = allow_lds((const void*)kern, Sh::LDS_BYTES, lds_ok);
    if (e != hipSuccess || a.prepare_only) return e;
    if (st.lds_bytes != Sh::LDS_BYTES) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)st.grid), dim3(ANY_THREADS), Sh::LDS_BYTES, a.stream,
                       (const T*)a.src, (const T*)a.factors[f], (T*)a.dst, st.k_in, a.pr->P[f], a.pr->Q[f], slices, units,
                       (int)(((uintptr_t)a.factors[f] & 15) == 0));
    return hipGetLastError();
}

template <typename T>
hipError_t launch_mfma_any(const LaunchArgs& a)
{
    const km_plan_step& st = *a.st;
    const int f = st.first_factor;
    const int P = a.pr->P[f], Q = a.pr->Q[f];
    if (st.num_factors != 1 || P % 16 || Q % 16 || st.k_in % P || st.block != ANY_THREADS) return hipErrorInvalidValue;
    const int64_t slices = a.pr->M * (st.k_in / P);      // counted through all rows
    const int cb = any_column_blocks(Q);
    const int64_t units = ((slices + ANY_TS - 1) / ANY_TS) * ((Q + cb * 16 - 1) / (cb * 16));
    if (st.grid < 1 || st.grid > units) return hipErrorInvalidValue;
    switch (cb) {
        case 3: return launch_mfma_any_cb<T, 3>(a, slices, units);
        case 4: return launch_mfma_any_cb<T, 4>(a, slices, units);
        case 5: return launch_mfma_any_cb<T, 5>(a, slices, units);
    }
    return hipErrorInvalidValue;
}

}  // namespace km
