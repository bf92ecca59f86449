// Launchers of the register-chained MFMA pair kernels (declared in launch.hpp): argument checks against what the kernel
// and its grid assume, the LDS attribute, the launch.  Included only by the translation units that
// instantiate these kernels.
#pragma once
#include "launch.hpp"
#include "mfma_pair_kernel.hpp"

namespace km {

template <int P, int ST, int NW, int PD, int NPASS>
struct PairLauncher {
template <bool KEEP>
static hipError_t run(const LaunchArgs& a)
{
    typedef MfmaPairShape<P, ST, NW, PD, NPASS> Sh;
    const km_plan_step& st = *a.st;
    auto kern = mfma_pair_sliced_multiply<P, ST, NW, PD, NPASS, KEEP>;
    static unsigned char lds_ok[64];
    hipError_t e = allow_lds((const void*)kern, Sh::LDS_BYTES, lds_ok);
    if (e != hipSuccess || a.prepare_only) return e;
    const float* f0 = (const float*)a.factors[st.first_factor + 1];    // applied first
    const float* f1 = (const float*)a.factors[st.first_factor];
    const int64_t tiles_per_row = st.k_in / Sh::TK;
    const int64_t num_tiles = a.pr->M * tiles_per_row;
    const int64_t tpw = st.tiles_per_wg;
    if (tpw < 1 || (num_tiles + tpw - 1) / tpw != st.grid) return hipErrorInvalidValue;
    if (st.tile_order != 0 && st.tile_order != 2 && st.tile_order != 3) return hipErrorInvalidValue;
    if (st.tile_order == 3 && !xcd_order_fits(num_tiles, st.grid)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)st.grid), dim3(Sh::NT), Sh::LDS_BYTES, a.stream,
                       (const float*)a.src, (float*)a.dst, f0, f1, st.k_in, st.k_out, tiles_per_row, num_tiles, tpw,
                       st.tile_order);
    return hipGetLastError();
}
};

template <int P, int ST, int NW, int PD, int NPASS>
hipError_t launch_mfma_pair(const LaunchArgs& a) { return launch_either<PairLauncher<P, ST, NW, PD, NPASS>>(a); }

template <int P, int ST, int NW>
hipError_t launch_mfma_pair_rows(const LaunchArgs& a)
{
    const km_plan_step& st = *a.st;
    auto kern = mfma_pair_rows_sliced_multiply<P, ST, NW>;
    if (st.k_in != (int64_t)P * P || st.k_out != 32 * 32 || st.tile_rows != ST || st.tile_slices != 1)
        return hipErrorInvalidValue;
    const float* f0 = (const float*)a.factors[st.first_factor + 1];    // applied first
    const float* f1 = (const float*)a.factors[st.first_factor];
    const int64_t num_tiles = (a.pr->M + ST - 1) / ST;
    const int64_t tpw = st.tiles_per_wg;
    if (tpw < 1 || (num_tiles + tpw - 1) / tpw != st.grid) return hipErrorInvalidValue;
    if (st.tile_order != 0 && st.tile_order != 2 && st.tile_order != 3) return hipErrorInvalidValue;
    if (st.tile_order == 3 && !xcd_order_fits(num_tiles, st.grid)) return hipErrorInvalidValue;
    if (a.prepare_only) return hipSuccess;
    hipLaunchKernelGGL(kern, dim3((unsigned)st.grid), dim3(NW * 64), 0, a.stream,
                       (const float*)a.src, (float*)a.dst, f0, f1, a.pr->M, num_tiles, tpw, st.tile_order);
    return hipGetLastError();
}

}  // namespace km
