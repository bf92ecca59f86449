// Launchers of the small-factor kernel with several factors per LDS pass (declared in launch.hpp): argument checks against what the kernel
// and its grid assume, the LDS attribute, the launch.  Included only by the translation units that
// instantiate these kernels.
#pragma once
#include "launch.hpp"
#include "fused_multi_kernel.hpp"

namespace km {

template <class Sh>
struct MultiLauncher {
template <bool KEEP>
static hipError_t run(const LaunchArgs& a)
{
    typedef typename Sh::T T;
    constexpr int STMAX = Sh::STMAX, NT = Sh::NT;
    const km_plan_step& st = *a.st;
    auto kern = fused_multi_sliced_multiply<Sh, KEEP>;
    static unsigned char lds_ok[64];
    hipError_t e = allow_lds((const void*)kern, Sh::LDS_BYTES, lds_ok);
    if (e != hipSuccess || a.prepare_only) return e;
    const int rows = st.tile_rows;
    if (rows < 1 || st.tile_slices < 1 || (int64_t)st.tile_slices * rows > STMAX) return hipErrorInvalidValue;
    const int slices = st.tile_slices * rows;            // what the kernel treats as one tile
    if (st.num_factors != Sh::NF) return hipErrorInvalidValue;
    FactorPtrs<Sh::NF> fp;
    for (int j = 0; j < Sh::NF; ++j) fp.f[j] = a.factors[st.first_factor + Sh::NF - 1 - j];   // order of application
    // stage j takes the next g(j) factors in that order: each must have the shape the stage is compiled for
    for (int j = 0, at = 0; j < Sh::NS; ++j)
        for (int k = 0; k < Sh::g(j); ++k, ++at) {
            const int f = st.first_factor + Sh::NF - 1 - at;
            if (a.pr->P[f] != Sh::p(j) || a.pr->Q[f] != Sh::q(j)) return hipErrorInvalidValue;
        }
    const int64_t tk_row = (int64_t)st.tile_slices * Sh::per_slice(0);
    if (st.k_in % tk_row) return hipErrorInvalidValue;
    const int64_t tiles_per_row = st.k_in / tk_row;
    // tiles of several rows hold whole rows
    if (rows > 1 && tiles_per_row != 1) return hipErrorInvalidValue;
    const int64_t tiles = rows > 1 ? (a.pr->M + rows - 1) / rows : a.pr->M * tiles_per_row;
    if (tiles != st.grid) return hipErrorInvalidValue;
    if (st.lds_bytes < Sh::LDS_PER_SLICE * slices + Sh::LDS_SLACK || st.lds_bytes > Sh::LDS_BYTES) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)st.grid), dim3(NT), (size_t)st.lds_bytes, a.stream,
                       (const T*)a.src, (T*)a.dst, fp, st.k_in, st.k_out, tiles_per_row, (int64_t)st.grid,
                       slices, rows, a.pr->M);
    return hipGetLastError();
}
};

template <class Sh>
hipError_t launch_multi(const LaunchArgs& a) { return launch_either<MultiLauncher<Sh>>(a); }

}  // namespace km
