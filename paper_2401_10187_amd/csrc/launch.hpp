// What the C-ABI unit knows of the compiled kernel instances: one launcher per instance, declared
// here and defined (with the kernels) in the translation unit of its family.
#pragma once
#include <hip/hip_runtime.h>
#include "plan.hpp"

namespace km {

struct LaunchArgs {
    const void* src;
    void* dst;
    const void* const* factors;   // host array of device pointers, all N of the problem
    const Problem* pr;
    const km_plan_step* st;
    hipStream_t stream;
    bool prepare_only;            // set the kernel's attributes on the current device, launch nothing
    bool keep_output;             // the next launch reads dst back and it fits the last-level cache: ordinary
                                  // instead of non-temporal stores (kernels that have both forms)
};

// Launchers of kernels with both store forms: prepares both, launches the one the arguments ask for.
template <class Impl>
inline hipError_t launch_either(const LaunchArgs& a)
{
    if (a.prepare_only) {
        hipError_t e = Impl::template run<false>(a);
        return e != hipSuccess ? e : Impl::template run<true>(a);
    }
    return a.keep_output ? Impl::template run<true>(a) : Impl::template run<false>(a);
}
typedef hipError_t (*LaunchFn)(const LaunchArgs&);

// Kernels that need more than 48 KB of dynamic LDS must raise their limit once per device.
inline hipError_t allow_lds(const void* kernel, int bytes, unsigned char (&done)[64])
{
    if (bytes <= 48 * 1024) return hipSuccess;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (done[dev]) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done[dev] = 1;     // racing threads at worst set the same value twice
    return e;
}

template <typename T, int P, int Q, int NF, int ST, int NT> hipError_t launch_fused(const LaunchArgs& a);
template <class Sh> hipError_t launch_multi(const LaunchArgs& a);      // Sh: a MixedShape of fused_multi_kernel.hpp
template <class OP, int P, int Q, int NF, int ST, int NW, int QSPLIT> hipError_t launch_mfma(const LaunchArgs& a);
template <int P, int ST, int NW, int PD, int NPASS> hipError_t launch_mfma_pair(const LaunchArgs& a);
template <int P, int ST, int NW> hipError_t launch_mfma_pair_rows(const LaunchArgs& a);
hipError_t launch_shuffle(const LaunchArgs& a);
template <typename T> hipError_t launch_mfma_any(const LaunchArgs& a);

}  // namespace km
