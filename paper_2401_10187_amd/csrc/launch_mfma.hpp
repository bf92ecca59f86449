// Launchers of the LDS-staged MFMA kernel (declared in launch.hpp): argument checks against what the kernel
// and its grid assume, the LDS attribute, the launch.  Included only by the translation units that
// instantiate these kernels.
#pragma once
#include "launch.hpp"
#include "mfma_kernel.hpp"

namespace km {

template <class OP, int P, int Q, int NF, int ST, int NW, int QSPLIT>
struct MfmaLauncher {
template <bool KEEP>
static hipError_t run(const LaunchArgs& a)
{
    typedef MfmaShape<OP, P, Q, NF, ST, NW, QSPLIT> Sh;
    typedef typename OP::T T;
    const km_plan_step& st = *a.st;
    auto kern = mfma_sliced_multiply<OP, P, Q, NF, ST, NW, QSPLIT, KEEP>;
    static unsigned char lds_ok[64];
    hipError_t e = allow_lds((const void*)kern, Sh::LDS_BYTES, lds_ok);
    if (e != hipSuccess || a.prepare_only) return e;
    const T* f[2] = {nullptr, nullptr};
    for (int j = 0; j < NF; ++j) f[j] = (const T*)a.factors[st.first_factor + NF - 1 - j];   // order of application
    const int64_t tiles_per_row = st.k_in / Sh::TK;
    const int64_t num_tiles = a.pr->M * tiles_per_row;
    const int64_t tpw = st.tiles_per_wg;
    if (tpw < 1 || (num_tiles + tpw - 1) / tpw != st.grid) return hipErrorInvalidValue;
    if (st.tile_order < 0 || st.tile_order > 3) return hipErrorInvalidValue;
    if (st.tile_order == 1 && !pair_order_fits(num_tiles, tpw)) return hipErrorInvalidValue;
    if (st.tile_order == 3 && !xcd_order_fits(num_tiles, st.grid)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)st.grid), dim3(Sh::NT), Sh::LDS_BYTES, a.stream,
                       (const T*)a.src, (T*)a.dst, f[0], f[1], st.k_in, st.k_out, tiles_per_row, num_tiles, tpw,
                       st.tile_order);
    return hipGetLastError();
}
};

template <class OP, int P, int Q, int NF, int ST, int NW, int QSPLIT>
hipError_t launch_mfma(const LaunchArgs& a) { return launch_either<MfmaLauncher<OP, P, Q, NF, ST, NW, QSPLIT>>(a); }

}  // namespace km
