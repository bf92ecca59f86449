// Launchers of the dedicated small-factor kernel and the lane-exchange kernel (declared in launch.hpp): argument checks against what the kernel
// and its grid assume, the LDS attribute, the launch.  Included only by the translation units that
// instantiate these kernels.
#pragma once
#include "launch.hpp"
#include "fused_kernel.hpp"
#include "shuffle_kernel.hpp"

namespace km {

template <typename T, int P, int Q, int NF, int ST, int NT>
struct FusedLauncher {
template <bool KEEP>
static hipError_t run(const LaunchArgs& a)
{
    typedef FusedShape<T, P, Q, NF, ST, NT> Sh;
    const km_plan_step& st = *a.st;
    auto kern = fused_sliced_multiply<T, P, Q, NF, ST, NT, KEEP>;
    static unsigned char lds_ok[64];
    hipError_t e = allow_lds((const void*)kern, Sh::LDS_BYTES, lds_ok);
    if (e != hipSuccess || a.prepare_only) return e;
    const T* f[3] = {nullptr, nullptr, nullptr};
    for (int j = 0; j < NF; ++j) f[j] = (const T*)a.factors[st.first_factor + NF - 1 - j];   // order of application
    const int64_t tiles_per_row = st.k_in / Sh::TK;
    hipLaunchKernelGGL(kern, dim3((unsigned)st.grid), dim3(NT), Sh::LDS_BYTES, a.stream,
                       (const T*)a.src, (T*)a.dst, f[0], f[1], f[2], st.k_in, st.k_out, tiles_per_row,
                       (int64_t)st.grid);
    return hipGetLastError();
}
};

template <typename T, int P, int Q, int NF, int ST, int NT>
hipError_t launch_fused(const LaunchArgs& a) { return launch_either<FusedLauncher<T, P, Q, NF, ST, NT>>(a); }

inline hipError_t launch_shuffle_impl(const LaunchArgs& a)
{
    const km_plan_step& st = *a.st;
    const int64_t tiles_per_row = st.k_in / ((int64_t)SHF_ST * SHF_P);
    if (a.prepare_only) return hipSuccess;
    hipLaunchKernelGGL(shuffle_sliced_multiply_8x8<SHF_NT>, dim3((unsigned)st.grid), dim3(SHF_NT), 0, a.stream,
                       (const float*)a.src, (float*)a.dst, (const float*)a.factors[st.first_factor], st.k_in,
                       tiles_per_row, (int64_t)st.grid);
    return hipGetLastError();
}

}  // namespace km
