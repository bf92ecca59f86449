// C-ABI of the Kron-Matmul library (see include/kronmatmul.h) and the launch loop of Algorithm 1:
// one launch per plan step, buffers swapped between launches, everything on the caller's stream.
#include <hip/hip_runtime.h>
#include <mutex>
#include <vector>
#include <string.h>

#include "../../include/kronmatmul.h"
#include "plan.hpp"
#include "launch.hpp"
#include "instances.hpp"
#include "generic_kernel.hpp"
#include "row_kernel.hpp"
#include "fused_kernel.hpp"          // the kernel headers below are only needed for their shape structs
#include "fused_multi_kernel.hpp"
#include "mfma_kernel.hpp"
#include "mfma_pair_kernel.hpp"
#include "shuffle_kernel.hpp"
#include "mfma_any_kernel.hpp"

namespace km {

// ---------------------------------------------------------------------------------------------
// compiled kernel instances (launchers: launch.hpp; the list: instances.hpp)
// ---------------------------------------------------------------------------------------------
#define KM_FUSED_ROW(T, DT, P, Q, NF, ST, NT) \
    {KM_KERNEL_FUSED, DT, P, Q, NF, ST, NT, FusedShape<T, P, Q, NF, ST, NT>::LDS_BYTES, 1, 0, 0, 1.0f, "fused", 0, 0, \
     sizeof(T) == 8 ? 8192 : 0,    /* fp64: 10-20 % faster than the several-factors-per-pass kernel up to 4096 slices per row, 10 % slower at 32768 */ \
     NT == 1024 ? 8192 : 0},       /* 1024-thread workgroups only from 8192 tiles up: below, the 256-thread instance of the same tile is \
                                      2-5 % faster (128 x 8x8^6 0.110 vs 0.104 ms), above 1-2 % slower (2048 x 8x8^6 1.426 vs 1.454) */
/* (walk -1, one round of resident workgroups: measured for every single-factor instance; it pays for the
   shapes named here, e.g. 4096 x 64x64^2 0.100 -> 0.071 ms, 20000 x 64x64^2 0.327 -> 0.275, 1024 x 48x48^3 fp64
   1.08 -> 1.02, and costs on others: 200000 x 16x16^2 0.148 -> 0.181, 1024 x 64x64^2 fp64 0.038 -> 0.048) */
#define KM_MFMA_ROW(OP, DT, P, Q, NF, ST, NW, QS) \
    {KM_KERNEL_MFMA, DT, P, Q, NF, ST, NW * 64, MfmaShape<OP, P, Q, NF, ST, NW, QS>::LDS_BYTES, 1, 1, 0, 1.0f, "mfma", \
     0, 0, 0, 0, (P == 80 || P == 96 || P == 112 || P >= 144 || (P == 64 && Q == 64 && DT == KM_F32) || (P == 48 && DT == KM_F64)) ? -1 : 0 /* walk: one round of resident workgroups */},
/* One workgroup per compute unit with the whole output tile staged at once (NPASS == 1): 7-12 % faster
   than two 4-wave workgroups where output rows lie up to 8 KB apart and every compute unit gets 8 tiles
   and more (1024 x 32x32^4: 1.75 -> 1.54 ms per launch); 15 % slower on rows of 32^5 elements (128 KB
   between output rows) and on launches of a few hundred tiles.  Walks of 8 tiles, XCD-contiguous. */
#define KM_PAIR_ROW(P, ST, NW, PD, NPASS) \
    {KM_KERNEL_MFMA, KM_F32, P, 32, 2, ST, NW * 64, MfmaPairShape<P, ST, NW, PD, NPASS>::LDS_BYTES, 1, 2, 0, 1.0f, "mfma-pair", \
     0, 0, NPASS == 1 ? 2048 : 0, NPASS == 1 ? 2048 : 0, NPASS == 1 ? 8 : 0, NPASS == 1 ? 1 : 0},
#define KM_MULTI_ROW(T, DT, P, Q, G0, G1, G2, ST, NT) \
    {KM_KERNEL_FUSED, DT, P, Q, G0 + G1 + G2, ST, NT, MultiShape<T, P, Q, G0, G1, G2, ST, NT>::LDS_BYTES, 1, 0, 1, \
     (G0 == 1 && P < 8) ? 1.6f                           /* one tiny factor per LDS pass is instruction-bound */ \
     : (P == 3 && G0 + G1 + G2 >= 5) ? 1.2f              /* 3^5 and more elements per slice: long runs need tiles that leave two workgroups per compute unit */ \
     : (P == 5 && G0 + G1 + G2 >= 4) ? 1.1f : 1.0f,      /* 62 KB tiles: 5^6 as 3 + 3 factors 7 % faster than as 4 + 2, 5^8 as 4 + 4 still 7 % faster than as 3 + 3 + 2 */ \
     "fused-multi", MultiShape<T, P, Q, G0, G1, G2, ST, NT>::LDS_PER_SLICE, (int)ipow(P, G0), 0, 0, 0, 0, \
     MultiShape<T, P, Q, G0, G1, G2, ST, NT>::LDS_SLACK, {0, 0, 0, 0, 0, 0, 0, 0, 0}},
#define KM_MULTI4_ROW(T, DT, P, Q, G0, G1, G2, G3, ST, NT) \
    {KM_KERNEL_FUSED, DT, P, Q, G0 + G1 + G2 + G3, ST, NT, MultiShape<T, P, Q, G0, G1, G2, ST, NT, G3>::LDS_BYTES, 1, 0, 1, \
     1.0f, "fused-multi", MultiShape<T, P, Q, G0, G1, G2, ST, NT, G3>::LDS_PER_SLICE, (int)ipow(P, G0), ST /* whole rows only */, 0, 0, 0, \
     MultiShape<T, P, Q, G0, G1, G2, ST, NT, G3>::LDS_SLACK, {0, 0, 0, 0, 0, 0, 0, 0, 0}},
#define KM_MULTI4_FN(T, DT, P, Q, G0, G1, G2, G3, ST, NT) launch_multi<MultiShape<T, P, Q, G0, G1, G2, ST, NT, G3>>,
#define KM_MIXED_SHAPE(T, P0, Q0, G0, P1, Q1, G1, P2, Q2, G2, ST, NT) MixedShape<T, P0, Q0, G0, P1, Q1, G1, P2, Q2, G2, ST, NT>
#define KM_MIXED_ROW(T, DT, P0, Q0, G0, P1, Q1, G1, P2, Q2, G2, ST, NT) \
    {KM_KERNEL_FUSED, DT, P0, Q0, G0 + G1 + G2, ST, NT, KM_MIXED_SHAPE(T, P0, Q0, G0, P1, Q1, G1, P2, Q2, G2, ST, NT)::LDS_BYTES, 1, 0, 1, \
     (G0 == 1 && P0 < 8) ? 1.6f : 1.0f, "fused-mixed", \
     KM_MIXED_SHAPE(T, P0, Q0, G0, P1, Q1, G1, P2, Q2, G2, ST, NT)::LDS_PER_SLICE, (int)ipow(P0, G0), 0, 0, 0, 0, \
     KM_MIXED_SHAPE(T, P0, Q0, G0, P1, Q1, G1, P2, Q2, G2, ST, NT)::LDS_SLACK, {P0, Q0, G0, P1, Q1, G1, P2, Q2, G2}},
#define KM_MIXED_FN(T, DT, P0, Q0, G0, P1, Q1, G1, P2, Q2, G2, ST, NT) launch_multi<KM_MIXED_SHAPE(T, P0, Q0, G0, P1, Q1, G1, P2, Q2, G2, ST, NT)>,
#define KM_ROWS_ROW(P, ST, NW) \
    {KM_KERNEL_MFMA, KM_F32, P, 32, 2, 1, NW * 64, 0, ST, 2, 0, 1.0f, "mfma-pair-rows"},
#define KM_ROWS_FN(P, ST, NW) launch_mfma_pair_rows<P, ST, NW>,
#define KM_MULTI_FN(T, DT, P, Q, G0, G1, G2, ST, NT) launch_multi<MultiShape<T, P, Q, G0, G1, G2, ST, NT>>,
#define KM_PAIR_FN(P, ST, NW, PD, NPASS) launch_mfma_pair<P, ST, NW, PD, NPASS>,
#define KM_FUSED_FN(T, DT, P, Q, NF, ST, NT) launch_fused<T, P, Q, NF, ST, NT>,
#define KM_MFMA_FN(OP, DT, P, Q, NF, ST, NW, QS) launch_mfma<OP, P, Q, NF, ST, NW, QS>,

static const Variant g_variants[] = {
    {KM_KERNEL_SHUFFLE, KM_F32, SHF_P, SHF_Q, 1, SHF_ST, SHF_NT, 0, 1, 0, 0, 1.0f, "shuffle"},
    KM_INSTANCES(KM_FUSED_ROW, KM_MFMA_ROW, KM_PAIR_ROW, KM_MULTI_ROW, KM_ROWS_ROW, KM_MIXED_ROW, KM_MULTI4_ROW) };
static const LaunchFn g_launchers[] = {
    launch_shuffle,
    KM_INSTANCES(KM_FUSED_FN, KM_MFMA_FN, KM_PAIR_FN, KM_MULTI_FN, KM_ROWS_FN, KM_MIXED_FN, KM_MULTI4_FN) };
static const int g_num_variants = (int)(sizeof(g_variants) / sizeof(g_variants[0]));

template <typename T>
static hipError_t launch_generic(const LaunchArgs& a)
{
    const km_plan_step& st = *a.st;
    const int f = st.first_factor;
    const int P = a.pr->P[f], Q = a.pr->Q[f];
    const int64_t S = st.k_in / P;
    const int64_t slices = a.pr->M * S;                  // counted through all rows
    const int64_t units = ((slices + GEN_TS - 1) / GEN_TS) * ((Q + GEN_TQ - 1) / GEN_TQ);
    if (st.grid < 1 || st.grid > units) return hipErrorInvalidValue;
    if (a.prepare_only) return hipSuccess;
    hipLaunchKernelGGL((sliced_multiply_generic<T>), dim3((unsigned)st.grid), dim3(GEN_THREADS), 0, a.stream,
                       (const T*)a.src, (const T*)a.factors[f], (T*)a.dst, st.k_in, P, Q, slices, units);
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_rows(const LaunchArgs& a)
{
    const km_plan_step& st = *a.st;
    const Problem& pr = *a.pr;
    const int n = st.num_factors;
    if (st.first_factor != 0 || n != pr.N || n > ROW_MAXF) return hipErrorInvalidValue;
    RowFactors fa{};
    fa.n = n;
    int64_t w = st.k_in, maxw = st.k_in, fel = 0;
    for (int i = 0; i < n; ++i) {                        // order of application: last factor first
        const int f = n - 1 - i;
        fa.f[i] = a.factors[f];
        fa.P[i] = pr.P[f];
        fa.Q[i] = pr.Q[f];
        if (w % pr.P[f]) return hipErrorInvalidValue;
        const int64_t s_blocks = (w / pr.P[f] + ROW_SB - 1) / ROW_SB;
        fa.magic[i] = ((1ull << 40) + (unsigned long long)s_blocks - 1) / (unsigned long long)s_blocks;
        w = w / pr.P[f] * pr.Q[f];
        if (w > maxw) maxw = w;
        fel += (int64_t)pr.P[f] * pr.Q[f];
    }
    const int64_t need = row_lds_bytes(maxw, fel, (int)sizeof(T));
    if (w != st.k_out || need > ROW_LDS_LIMIT || st.lds_bytes < need) return hipErrorInvalidValue;
    if (st.grid < 1 || st.grid > pr.M) return hipErrorInvalidValue;
    if (st.block != ROW_THREADS_MANY && st.block != ROW_THREADS_FEW) return hipErrorInvalidValue;
    auto kern = st.block == ROW_THREADS_FEW ? row_sliced_multiply<T, ROW_THREADS_FEW> : row_sliced_multiply<T, ROW_THREADS_MANY>;
    static unsigned char lds_ok[2][64];
    hipError_t e = allow_lds((const void*)kern, ROW_LDS_LIMIT, lds_ok[st.block == ROW_THREADS_FEW]);
    if (e != hipSuccess || a.prepare_only) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)st.grid), dim3((unsigned)st.block), (size_t)st.lds_bytes, a.stream,
                       (const T*)a.src, (T*)a.dst, fa, (int)st.k_in, (int)st.k_out, (int)maxw, pr.M);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// library state
// ---------------------------------------------------------------------------------------------
struct DeviceState {
    void* ws = nullptr;
    size_t ws_bytes = 0;
    void* scratch_ptr = nullptr;     // this device's copy of `scratch`, resolved once
    // Profiling history since KM_OPT_PROFILE was last switched on: call c with n launches owns
    // events [first[c], first[c] + n].  Events are pooled and reused after the history is cleared.
    std::vector<hipEvent_t> events;
    std::vector<int> call_first, call_steps;
    int events_used = 0;
};
constexpr int MAX_PROFILED_CALLS = 4096;

// Workspace of kronmatmul_static: one array per GPU, held from the moment the library's code is
// loaded on that GPU until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels are given the address that call returns on the device in use.
static __device__ __align__(256) unsigned char scratch[KM_STATIC_SCRATCH_BYTES];

static std::mutex g_mutex;
static Options g_options;
static int g_profile = 0;
// Launches other than a call's last whose output is between KEEP_MIN_MIB and g_keep_mib MiB write it
// with ordinary stores (KM_OPT_KEEP_MIB; the chip's last-level cache holds 256 MB).  Measured, whole
// call without -> with: 256 x 16x32^4 0.299 -> 0.266 ms, 256 x 8x8^6 0.201 -> 0.181, 16 x 32x32^4 (64 MiB)
// 0.065 -> 0.059, 256 x 64x64^3 0.317 -> 0.306; 32 x 8x8^6 (32 MiB) 0.035 -> 0.037, 512 MB and more: 1-8 %
// slower on the MFMA kernels.
static int g_keep_mib = 320;
constexpr double KEEP_MIN_MIB = 48.0;
static DeviceState g_dev[64];

static GenericKernel generic_kernel(int dtype)
{
    return GenericKernel{GEN_THREADS, GEN_TS, GEN_TQ, dtype == KM_F32 ? gen_lds_bytes<float>() : gen_lds_bytes<double>(),
                         ROW_THREADS_MANY, ROW_THREADS_FEW, ROW_FEW_ROWS, ROW_LDS_LIMIT, ROW_MAXF,
                         ANY_THREADS, ANY_TS, ANY_ROW_BYTES};
}

// Plans are memoised: iterative callers repeat the same small problem thousands of times and the
// planner should not show up next to a 6-microsecond kernel.
struct CachedPlan {
    int64_t M; int N; int dtype;
    std::vector<int> P, Q;
    Options opt;
    Plan plan;
    bool tuned;          // measured by kronmatmul_tune: kept until kronmatmul_release
};
static std::vector<CachedPlan> g_plan_cache;      // most recently used first, guarded by g_mutex
constexpr size_t PLAN_CACHE_ENTRIES = 16, PLAN_CACHE_TUNED = 64;

// Puts a plan at the head of the cache (g_mutex held).  A tuned plan replaces the entry of the same
// problem; computed plans are dropped oldest first, tuned ones only when PLAN_CACHE_TUNED are held.
static void cache_plan(const Problem& pr, const Options& opt, const Plan& plan, bool tuned);

static bool same_options(const Options& a, const Options& b)
{
    return a.kernels == b.kernels && a.max_fuse == b.max_fuse && a.prefer_tile == b.prefer_tile &&
           a.prefer_threads == b.prefer_threads && a.tiles_per_wg == b.tiles_per_wg &&
           a.pair_interleave == b.pair_interleave && a.tile_order == b.tile_order &&
           a.prefer_instance == b.prefer_instance;
}

// HIP takes a launch only if its work-items, grid x block, number fewer than 2^32.
static bool launchable(const km_plan_step& st)
{
    return st.grid > 0 && st.block > 0 && (double)st.grid * (double)st.block < 4294967296.0;
}

static km_status plan_for(const Problem& pr, Plan& plan)
{
    Options opt;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        opt = g_options;
        for (size_t i = 0; i < g_plan_cache.size(); ++i) {
            const CachedPlan& c = g_plan_cache[i];
            if (c.M == pr.M && c.N == pr.N && c.dtype == pr.dtype && same_options(c.opt, opt) && c.P == pr.P && c.Q == pr.Q) {
                plan = c.plan;
                if (i) std::swap(g_plan_cache[0], g_plan_cache[i]);
                return KM_OK;
            }
        }
    }
    km_status s = make_plan(pr, opt, g_variants, g_num_variants, generic_kernel(pr.dtype), plan);
    if (s != KM_OK) return s;
    for (const km_plan_step& st : plan.steps)
        if (!launchable(st)) return KM_EUNSUPPORTED;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        cache_plan(pr, opt, plan, false);
    }
    return KM_OK;
}

static void cache_plan(const Problem& pr, const Options& opt, const Plan& plan, bool tuned)
{
    size_t computed = 0, kept = 0;
    for (size_t i = 0; i < g_plan_cache.size();) {
        const CachedPlan& c = g_plan_cache[i];
        const bool same = c.M == pr.M && c.N == pr.N && c.dtype == pr.dtype && same_options(c.opt, opt) &&
                          c.P == pr.P && c.Q == pr.Q;
        if (same) {
            if (c.tuned && !tuned) return;               // never replace a measured plan by a computed one
            g_plan_cache.erase(g_plan_cache.begin() + i);
            continue;
        }
        (c.tuned ? kept : computed) += 1;
        ++i;
    }
    const size_t limit = tuned ? PLAN_CACHE_TUNED : PLAN_CACHE_ENTRIES;
    if ((tuned ? kept : computed) >= limit)
        for (size_t i = g_plan_cache.size(); i-- > 0;)
            if (g_plan_cache[i].tuned == tuned) { g_plan_cache.erase(g_plan_cache.begin() + i); break; }
    g_plan_cache.insert(g_plan_cache.begin(), CachedPlan{pr.M, pr.N, pr.dtype, pr.P, pr.Q, opt, plan, tuned});
}

static hipError_t launch_step(const Problem& pr, const km_plan_step& st, const void* src, void* dst,
                              const void* const* F, hipStream_t stream, bool prepare_only = false,
                              bool keep_output = false)
{
    LaunchArgs a{src, dst, F, &pr, &st, stream, prepare_only, keep_output};
    if (st.kernel == KM_KERNEL_GENERIC)
        return pr.dtype == KM_F32 ? launch_generic<float>(a) : launch_generic<double>(a);
    if (st.kernel == KM_KERNEL_ROWS)
        return pr.dtype == KM_F32 ? launch_rows<float>(a) : launch_rows<double>(a);
    if (st.kernel == KM_KERNEL_MFMA_ANY)
        return pr.dtype == KM_F32 ? launch_mfma_any<float>(a) : launch_mfma_any<double>(a);
    if (st.variant < 0 || st.variant >= g_num_variants) return hipErrorInvalidValue;
    return g_launchers[st.variant](a);
}

static km_status run(const Problem& pr, const Plan& plan, const void* X, const void* const* F, void* Y,
                     void* ws, hipStream_t stream, bool allow_profile = true)
{
    char* ws0 = (char*)ws;
    char* ws1 = ws0 + plan.ws0_bytes;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return KM_ELAUNCH;
    DeviceState& ds = g_dev[dev];
    const int n = (int)plan.steps.size();
    int profile;
    int ev0 = 0;
    std::vector<hipEvent_t> ev;      // this call's events, copied while the lock is held: another thread may grow ds.events
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        profile = allow_profile && g_profile && (int)ds.call_first.size() < MAX_PROFILED_CALLS;
        if (profile) {
            ev0 = ds.events_used;
            while ((int)ds.events.size() < ev0 + n + 1) {
                hipEvent_t e;
                if (hipEventCreate(&e) != hipSuccess) return KM_ELAUNCH;
                ds.events.push_back(e);
            }
            ds.events_used = ev0 + n + 1;
            ev.assign(ds.events.begin() + ev0, ds.events.begin() + ev0 + n + 1);
        }
    }
    if (profile && hipEventRecord(ev[0], stream) != hipSuccess) return KM_ELAUNCH;
    for (int i = 0; i < n; ++i) {
        const km_plan_step& st = plan.steps[i];
        auto buf = [&](int b) -> void* {
            switch (b) {
                case KM_BUF_X: return (void*)X;
                case KM_BUF_Y: return Y;
                case KM_BUF_WS0: return ws0;
                default: return ws1;
            }
        };
        // an intermediate that fits the last-level cache is written so that it stays there for the next launch
        const double out_mib = (double)pr.M * (double)st.k_out * (double)pr.esize / 1048576.0;
        // (the small-factor kernel still gains 1-2 % at 1 GiB, where a quarter of the intermediate stays on
        // chip: 1024 x 8x8^6 0.724 -> 0.715 ms, 16 x 8x8^8 1.255 -> 1.225, 65536 x 8x8^4 0.714 -> 0.697; level at
        // 2 GiB, 1.6 % slower at 4 GiB; the MFMA kernels lose from 400 MB on)
        const double keep_max = (double)g_keep_mib * (st.kernel == KM_KERNEL_FUSED ? 4.0 : 1.0);
        const bool keep = i + 1 < n && out_mib >= KEEP_MIN_MIB && out_mib <= keep_max;
        if (launch_step(pr, st, buf(st.src), buf(st.dst), F, stream, false, keep) != hipSuccess) return KM_ELAUNCH;
        if (profile && hipEventRecord(ev[i + 1], stream) != hipSuccess) return KM_ELAUNCH;
    }
    if (profile) {
        std::lock_guard<std::mutex> lock(g_mutex);
        ds.call_first.push_back(ev0);
        ds.call_steps.push_back(n);
    }
    return KM_OK;
}

static bool aligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// Sleeps until the constant 100 MHz clock has advanced by `wall_ticks`, in steps of a few
// microseconds and at most 2^21 of them, then reports how far both clocks moved.
__global__ void clock_probe_kernel(unsigned long long* ticks, unsigned long long wall_ticks)
{
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    for (int i = 0; i < (1 << 21); ++i) {
        __builtin_amdgcn_s_sleep(127);
        if (wall_clock64() - w0 >= wall_ticks) break;
    }
    if (threadIdx.x == 0) {
        ticks[0] = clock64() - c0;
        ticks[1] = wall_clock64() - w0;
    }
}

static bool overlap(const void* a, size_t na, const void* b, size_t nb)
{
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return na > 0 && nb > 0 && a0 < b0 + nb && b0 < a0 + na;
}

static km_status check_pointers(const Problem& pr, const void* X, const void* const* F, void* Y)
{
    if (!F) return KM_EINVAL;
    if (pr.M == 0) return KM_OK;
    if (!X || !Y) return KM_EINVAL;
    if (!aligned(X, 16) || !aligned(Y, 16)) return KM_EINVAL;      // kernels use 16-byte accesses
    for (int i = 0; i < pr.N; ++i)
        if (!F[i] || !aligned(F[i], pr.esize)) return KM_EINVAL;
    // Y is written while X is still being read (and used for intermediates): they must be apart
    if (overlap(X, (size_t)(pr.M * pr.k_in) * pr.esize, Y, (size_t)(pr.M * pr.k_out) * pr.esize)) return KM_EINVAL;
    return KM_OK;
}

// The workspace (ws_bytes of it are used) must be apart from X and from Y.
static km_status check_workspace(const Problem& pr, const void* X, const void* Y, const void* ws, size_t ws_bytes)
{
    if (overlap(ws, ws_bytes, X, (size_t)(pr.M * pr.k_in) * pr.esize) ||
        overlap(ws, ws_bytes, Y, (size_t)(pr.M * pr.k_out) * pr.esize))
        return KM_EINVAL;
    return KM_OK;
}

// ---------------------------------------------------------------------------------------------
// autotuner: measures every instance that fits each group of factors and plans on the measurements
// ---------------------------------------------------------------------------------------------
// Fills a buffer with values in [-0.5, 0.5) so that timed launches work on ordinary numbers.
template <typename T>
__global__ void tune_fill(T* dst, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint32_t h = (uint32_t)i * 2654435761u;
        dst[i] = (T)((h >> 8) & 0xffff) * (T)(1.0 / 65536.0) - (T)0.5;
    }
}

struct TuneScratch {
    void* a = nullptr;       // rows read by the timed launch (X of a timed plan)
    void* b = nullptr;       // rows written (Y of a timed plan)
    void* f = nullptr;       // one buffer that stands in for every factor
    void* ws = nullptr;      // workspace of a timed plan
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ~TuneScratch()
    {
        if (a) (void)hipFree(a);
        if (b) (void)hipFree(b);
        if (f) (void)hipFree(f);
        if (ws) (void)hipFree(ws);
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
};

// Milliseconds per repetition of `body` (which enqueues work on `stream`), best of two rounds.
template <class Body>
static float time_body(TuneScratch& sc, hipStream_t stream, int reps, Body body)
{
    float best = -1.f;
    for (int round = 0; round < 2; ++round) {
        if (hipEventRecord(sc.e0, stream) != hipSuccess) return -1.f;
        for (int i = 0; i < reps; ++i)
            if (!body()) return -1.f;
        if (hipEventRecord(sc.e1, stream) != hipSuccess) return -1.f;
        if (hipEventSynchronize(sc.e1) != hipSuccess) return -1.f;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, sc.e0, sc.e1) != hipSuccess) return -1.f;
        ms /= (float)reps;
        if (best < 0.f || ms < best) best = ms;
    }
    return best;
}

static int reps_for(float ms_once)
{
    // about 3 ms of work per round, between 2 and 20 launches
    int reps = ms_once > 0.f ? (int)(3.0f / ms_once) : 20;
    return reps < 2 ? 2 : (reps > 20 ? 20 : reps);
}

static km_status tune(const Problem& pr, const Options& opt, hipStream_t stream, Plan& chosen,
                      float* tuned_ms, float* default_ms)
{
    const int N = pr.N;
    std::vector<int64_t> width;
    row_widths(pr, width);
    int64_t widest = 0, fmax = 0;
    for (int r = 0; r <= N; ++r) widest = width[r] > widest ? width[r] : widest;
    for (int i = 0; i < N; ++i) fmax = (int64_t)pr.P[i] * pr.Q[i] > fmax ? (int64_t)pr.P[i] * pr.Q[i] : fmax;

    Plan deflt;
    km_status s = make_plan(pr, opt, g_variants, g_num_variants, generic_kernel(pr.dtype), deflt);
    if (s != KM_OK) return s;

    TuneScratch sc;
    const size_t row_bytes = round_up((size_t)(pr.M * widest) * pr.esize, 256);
    if (hipMalloc(&sc.a, row_bytes) != hipSuccess || hipMalloc(&sc.b, row_bytes) != hipSuccess ||
        hipMalloc(&sc.f, (size_t)fmax * pr.esize) != hipSuccess) {
        (void)hipGetLastError();
        return KM_ENOMEM;
    }
    if (hipEventCreate(&sc.e0) != hipSuccess || hipEventCreate(&sc.e1) != hipSuccess) return KM_ELAUNCH;
    if (pr.dtype == KM_F32) {
        hipLaunchKernelGGL(tune_fill<float>, dim3(4096), dim3(256), 0, stream, (float*)sc.a, pr.M * widest);
        hipLaunchKernelGGL(tune_fill<float>, dim3(64), dim3(256), 0, stream, (float*)sc.f, fmax);
    } else {
        hipLaunchKernelGGL(tune_fill<double>, dim3(4096), dim3(256), 0, stream, (double*)sc.a, pr.M * widest);
        hipLaunchKernelGGL(tune_fill<double>, dim3(64), dim3(256), 0, stream, (double*)sc.f, fmax);
    }
    if (hipGetLastError() != hipSuccess) return KM_ELAUNCH;
    std::vector<const void*> F(N, sc.f);

    // cost[r][nf]: measured milliseconds of the best launch that applies factors r-nf .. r-1
    std::vector<double> best(N + 1, 0.0);
    std::vector<int> take(N + 1, 1);
    std::vector<Choice> pick(N + 1);
    std::vector<Choice> cands;
    for (int r = 1; r <= N; ++r) {
        best[r] = -1;
        for (int nf = 1; nf <= r && nf <= opt.max_fuse; ++nf) {
            enumerate_choices(g_variants, g_num_variants, pr, r - 1, nf, width[r], opt, cands);
            if (nf == 1) cands.push_back(Choice());            // the generic kernel
            if (nf == 1 && any_mfma_fits(pr, r - 1, opt)) {     // the run-time-shape MFMA kernel
                Choice any;
                any.any_mfma = true;
                cands.push_back(any);
            }
            float group_best = -1.f;
            Choice group_pick;
            for (const Choice& ch : cands) {
                const km_plan_step st = build_step(pr, opt, g_variants, r, nf, ch, width, generic_kernel(pr.dtype));
                if (!launchable(st)) continue;
                auto body = [&]() { return launch_step(pr, st, sc.a, sc.b, F.data(), stream) == hipSuccess; };
                const float once = time_body(sc, stream, 1, body);       // also the warm-up
                if (once < 0.f) return KM_ELAUNCH;
                if (group_best > 0.f && once > 2.f * group_best) continue;   // hopeless: skip the careful timing
                const float ms = time_body(sc, stream, reps_for(once), body);
                if (ms < 0.f) return KM_ELAUNCH;
                if (group_best < 0.f || ms < group_best) { group_best = ms; group_pick = ch; }
            }
            if (group_best < 0.f) continue;
            const double c = (double)group_best + best[r - nf];
            if (best[r] < 0 || c < best[r]) { best[r] = c; take[r] = nf; pick[r] = group_pick; }
        }
        if (best[r] < 0) return KM_EUNSUPPORTED;
    }
    Plan tuned;
    s = finish_plan(pr, opt, g_variants, take, pick, width, generic_kernel(pr.dtype), tuned);
    if (s != KM_OK) return s;

    // Launches timed alone can rank differently than in sequence: keep the measured plan only if the
    // whole sequence beats the planner's own.
    // A third candidate: the whole-row kernel wherever it fits, if the planner did not take it itself.
    Plan rows;
    bool have_rows = false;
    if (deflt.steps.size() != 1 || deflt.steps[0].kernel != KM_KERNEL_ROWS) {
        Options force = opt;
        force.prefer_instance = g_num_variants + 1;
        have_rows = make_plan(pr, force, g_variants, g_num_variants, generic_kernel(pr.dtype), rows) == KM_OK &&
                    rows.steps.size() == 1 && rows.steps[0].kernel == KM_KERNEL_ROWS && launchable(rows.steps[0]);
    }
    const size_t need_d = deflt.ws0_bytes + deflt.ws1_bytes, need_t = tuned.ws0_bytes + tuned.ws1_bytes;
    const size_t need = need_d > need_t ? need_d : need_t;
    if (need > 0 && hipMalloc(&sc.ws, need) != hipSuccess) { (void)hipGetLastError(); return KM_ENOMEM; }
    const Plan* plans[3] = {&deflt, &tuned, have_rows ? &rows : nullptr};
    float t[3] = {-1.f, -1.f, -1.f};
    float quickest = -1.f;
    for (int k = 0; k < 3; ++k) {
        if (!plans[k]) continue;
        auto body = [&]() { return run(pr, *plans[k], sc.a, F.data(), sc.b, sc.ws, stream, false) == KM_OK; };
        t[k] = time_body(sc, stream, 1, body);
        if (t[k] < 0.f) return KM_ELAUNCH;
        if (quickest < 0.f || t[k] < quickest) quickest = t[k];
    }
    const int reps = reps_for(quickest);
    for (int round = 0; round < 2; ++round)
        for (int k = 0; k < 3; ++k) {
            if (!plans[k]) continue;
            auto body = [&]() { return run(pr, *plans[k], sc.a, F.data(), sc.b, sc.ws, stream, false) == KM_OK; };
            const float ms = time_body(sc, stream, reps, body);
            if (ms < 0.f) return KM_ELAUNCH;
            if (round == 0 || ms < t[k]) t[k] = ms;
        }
    // The planner's own unless another is 1 % faster and needs no more workspace: a caller that sized
    // its workspace before tuning must not find it too small afterwards.
    int keep = 0;
    for (int k = 1; k < 3; ++k)
        if (plans[k] && t[k] < 0.99f * t[0] && t[k] < t[keep] &&
            plans[k]->ws0_bytes + plans[k]->ws1_bytes <= need_d) keep = k;
    chosen = *plans[keep];
    if (tuned_ms) *tuned_ms = t[keep];
    if (default_ms) *default_ms = t[0];
    if (hipStreamSynchronize(stream) != hipSuccess) return KM_ELAUNCH;
    return KM_OK;
}

// ---------------------------------------------------------------------------------------------
// factors given transposed
// ---------------------------------------------------------------------------------------------
// Copies of the factors in the layout the kernels read (P x Q row-major) sit behind the plan's own
// workspace, each on a 256-byte boundary.
static size_t factor_copy_bytes(const Problem& pr)
{
    size_t b = 0;
    for (int i = 0; i < pr.N; ++i) b += round_up((size_t)pr.P[i] * pr.Q[i] * pr.esize, 256);
    return b;
}

struct TransposeArgs {
    const void* src[64];      // stored Q x P, row-major
    void* dst[64];            // P x Q, row-major
    int p[64], q[64];
};

// one workgroup per factor
template <typename T>
__global__ __launch_bounds__(256) void transpose_factors(TransposeArgs a)
{
    const int f = blockIdx.x;
    const T* src = static_cast<const T*>(a.src[f]);
    T* dst = static_cast<T*>(a.dst[f]);
    const int P = a.p[f], Q = a.q[f];
    for (int e = threadIdx.x; e < P * Q; e += blockDim.x) {
        const int pp = e / Q, qq = e % Q;             // element (pp, qq) of the P x Q result
        dst[e] = src[(int64_t)qq * P + pp];
    }
}

// Library-managed workspace of at least `need` bytes on the current device (grown on demand).
static km_status library_workspace(size_t need, void** ws)
{
    *ws = nullptr;
    if (need == 0) return KM_OK;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return KM_ELAUNCH;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState& ds = g_dev[dev];
    if (ds.ws_bytes < need) {
        if (ds.ws) {
            // work already enqueued may still read the old buffer
            if (hipDeviceSynchronize() != hipSuccess) return KM_ELAUNCH;
            (void)hipFree(ds.ws);
            ds.ws = nullptr; ds.ws_bytes = 0;
        }
        if (hipMalloc(&ds.ws, need) != hipSuccess) { (void)hipGetLastError(); ds.ws = nullptr; return KM_ENOMEM; }
        ds.ws_bytes = need;
    }
    *ws = ds.ws;
    return KM_OK;
}

// Address of the current device's copy of `scratch` (resolved on first use, then remembered).
static km_status static_scratch(void** ptr)
{
    *ptr = nullptr;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return KM_ELAUNCH;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState& ds = g_dev[dev];
    if (!ds.scratch_ptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return KM_ELAUNCH; }
        ds.scratch_ptr = p;
    }
    *ptr = ds.scratch_ptr;
    return KM_OK;
}

// Where a call's workspace comes from: the library's cached allocation, the caller, or the static array.
enum WsKind { WS_LIBRARY, WS_CALLER, WS_STATIC };

// The body of every compute entry point.
static km_status execute(int M, int N, const int* P, const int* Q, const void* X, const void* const* F, void* Y,
                         km_dtype dtype, WsKind kind, void* workspace, size_t workspace_bytes, void* stream,
                         bool transposed)
{
    Problem pr;
    km_status s = make_problem(M, N, P, Q, (int)dtype, pr);
    if (s != KM_OK) return s;
    s = check_pointers(pr, X, F, Y);
    if (s != KM_OK) return s;
    if (pr.M == 0) return KM_OK;
    Plan plan;
    s = plan_for(pr, plan);
    if (s != KM_OK) return s;
    const size_t plan_need = round_up(plan.ws0_bytes + plan.ws1_bytes, 256);
    const size_t need = transposed ? plan_need + factor_copy_bytes(pr) : plan.ws0_bytes + plan.ws1_bytes;
    void* ws = workspace;
    if (kind == WS_CALLER) {
        if (need > 0 && (!workspace || workspace_bytes < need)) return KM_ENOMEM;
        if (need > 0 && !aligned(workspace, 16)) return KM_EINVAL;
        if (need > 0 && check_workspace(pr, X, Y, workspace, need) != KM_OK) return KM_EINVAL;
    } else if (kind == WS_STATIC) {
        // sizes are checked before anything touches the device; nothing on this path allocates
        if (need > KM_STATIC_SCRATCH_BYTES) return KM_ENOMEM;
        s = static_scratch(&ws);
        if (s != KM_OK) return s;
        return run(pr, plan, X, F, Y, ws, (hipStream_t)stream, false);     // unprofiled: events would be created
    } else {
        s = library_workspace(need, &ws);
        if (s != KM_OK) return s;
    }
    if (!transposed) return run(pr, plan, X, F, Y, ws, (hipStream_t)stream);

    TransposeArgs ta;
    const void* fcopy[64];
    char* at = (char*)ws + plan_need;
    for (int i = 0; i < pr.N; ++i) {
        ta.src[i] = F[i];
        ta.dst[i] = at;
        ta.p[i] = pr.P[i];
        ta.q[i] = pr.Q[i];
        fcopy[i] = at;
        at += round_up((size_t)pr.P[i] * pr.Q[i] * pr.esize, 256);
    }
    if (pr.dtype == KM_F32)
        hipLaunchKernelGGL(transpose_factors<float>, dim3(pr.N), dim3(256), 0, (hipStream_t)stream, ta);
    else
        hipLaunchKernelGGL(transpose_factors<double>, dim3(pr.N), dim3(256), 0, (hipStream_t)stream, ta);
    if (hipGetLastError() != hipSuccess) return KM_ELAUNCH;
    return run(pr, plan, X, fcopy, Y, ws, (hipStream_t)stream);
}

}  // namespace km

using namespace km;

extern "C" {

km_status kronmatmul_workspace_size(int M, int N, const int* P, const int* Q, km_dtype dtype, size_t* bytes)
{
    if (!bytes) return KM_EINVAL;
    Problem pr;
    km_status s = make_problem(M, N, P, Q, (int)dtype, pr);
    if (s != KM_OK) return s;
    *bytes = 0;
    if (pr.M == 0) return KM_OK;
    Plan plan;
    s = plan_for(pr, plan);
    if (s != KM_OK) return s;
    *bytes = plan.ws0_bytes + plan.ws1_bytes;
    return KM_OK;
}

km_status kronmatmul_ws(int M, int N, const int* P, const int* Q, const void* X, const void* const* F,
                        void* Y, km_dtype dtype, void* workspace, size_t workspace_bytes, void* stream)
{
    return execute(M, N, P, Q, X, F, Y, dtype, WS_CALLER, workspace, workspace_bytes, stream, false);
}

km_status kronmatmul(int M, int N, const int* P, const int* Q, const void* X, const void* const* F,
                     void* Y, km_dtype dtype, void* stream)
{
    return execute(M, N, P, Q, X, F, Y, dtype, WS_LIBRARY, nullptr, 0, stream, false);
}

km_status kronmatmul_static(int M, int N, const int* P, const int* Q, const void* X, const void* const* F,
                            void* Y, km_dtype dtype, void* stream)
{
    return execute(M, N, P, Q, X, F, Y, dtype, WS_STATIC, nullptr, 0, stream, false);
}

km_status kronmatmul_transposed_workspace_size(int M, int N, const int* P, const int* Q, km_dtype dtype,
                                               size_t* bytes)
{
    if (!bytes) return KM_EINVAL;
    Problem pr;
    km_status s = make_problem(M, N, P, Q, (int)dtype, pr);
    if (s != KM_OK) return s;
    *bytes = 0;
    if (pr.M == 0) return KM_OK;
    Plan plan;
    s = plan_for(pr, plan);
    if (s != KM_OK) return s;
    *bytes = round_up(plan.ws0_bytes + plan.ws1_bytes, 256) + factor_copy_bytes(pr);
    return KM_OK;
}

km_status kronmatmul_transposed_ws(int M, int N, const int* P, const int* Q, const void* X,
                                   const void* const* Ft, void* Y, km_dtype dtype, void* workspace,
                                   size_t workspace_bytes, void* stream)
{
    return execute(M, N, P, Q, X, Ft, Y, dtype, WS_CALLER, workspace, workspace_bytes, stream, true);
}

km_status kronmatmul_transposed(int M, int N, const int* P, const int* Q, const void* X,
                                const void* const* Ft, void* Y, km_dtype dtype, void* stream)
{
    return execute(M, N, P, Q, X, Ft, Y, dtype, WS_LIBRARY, nullptr, 0, stream, true);
}

km_status kronmatmul_tune(int M, int N, const int* P, const int* Q, km_dtype dtype, void* stream,
                          float* tuned_ms, float* default_ms)
{
    Problem pr;
    km_status s = make_problem(M, N, P, Q, (int)dtype, pr);
    if (s != KM_OK) return s;
    if (tuned_ms) *tuned_ms = 0.f;
    if (default_ms) *default_ms = 0.f;
    if (pr.M == 0) return KM_OK;
    Options opt;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        opt = g_options;
    }
    Plan plan;
    s = tune(pr, opt, (hipStream_t)stream, plan, tuned_ms, default_ms);
    if (s != KM_OK) return s;
    for (const km_plan_step& st : plan.steps)
        if (!launchable(st)) return KM_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mutex);
    cache_plan(pr, opt, plan, true);
    return KM_OK;
}

km_status kronmatmul_prepare(int M, int N, const int* P, const int* Q, km_dtype dtype)
{
    Problem pr;
    km_status s = make_problem(M, N, P, Q, (int)dtype, pr);
    if (s != KM_OK) return s;
    if (pr.M == 0) return KM_OK;
    Plan plan;
    s = plan_for(pr, plan);
    if (s != KM_OK) return s;
    std::vector<const void*> none(pr.N, nullptr);
    for (const km_plan_step& st : plan.steps)
        if (launch_step(pr, st, nullptr, nullptr, none.data(), nullptr, true) != hipSuccess) return KM_ELAUNCH;
    void* unused;
    return static_scratch(&unused);          // kronmatmul_static finds its array's address resolved
}

km_status kronmatmul_plan(int M, int N, const int* P, const int* Q, km_dtype dtype,
                          km_plan_step* steps, int cap, int* nsteps)
{
    if (!nsteps || cap < 0 || (cap > 0 && !steps)) return KM_EINVAL;
    Problem pr;
    km_status s = make_problem(M, N, P, Q, (int)dtype, pr);
    if (s != KM_OK) return s;
    *nsteps = 0;
    if (pr.M == 0) return KM_OK;                 // nothing to launch
    Plan plan;
    s = plan_for(pr, plan);
    if (s != KM_OK) return s;
    *nsteps = (int)plan.steps.size();
    for (int i = 0; i < *nsteps && i < cap; ++i) steps[i] = plan.steps[i];
    return KM_OK;
}

long long kronmatmul_store_column(long long k_in, long long p_group, long long tile_k,
                                  long long tile_index, long long local_col)
{
    return store_column(k_in, p_group, tile_k, tile_index, local_col);
}

km_status kronmatmul_cost(int M, int N, const int* P, const int* Q, km_dtype dtype,
                          double* flops, double* planned_bytes)
{
    Problem pr;
    km_status s = make_problem(M, N, P, Q, (int)dtype, pr);
    if (s != KM_OK) return s;
    if (pr.M == 0) {
        if (flops) *flops = 0;
        if (planned_bytes) *planned_bytes = 0;
        return KM_OK;
    }
    Plan plan;
    s = plan_for(pr, plan);
    if (s != KM_OK) return s;
    if (flops) *flops = plan.flops;
    if (planned_bytes) *planned_bytes = plan.bytes;
    return KM_OK;
}

km_status kronmatmul_set_option(km_option option, int value)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    switch (option) {
        case KM_OPT_KERNELS:
            if (value < 0 || value > 63) return KM_EINVAL;
            g_options.kernels = value | 1;
            return KM_OK;
        case KM_OPT_MAX_FUSE:
            if (value < 1 || value > 16) return KM_EINVAL;
            g_options.max_fuse = value;
            return KM_OK;
        case KM_OPT_PREFER_TILE:
            if (value < 0) return KM_EINVAL;
            g_options.prefer_tile = value;
            return KM_OK;
        case KM_OPT_PREFER_THREADS:
            if (value < 0 || value > 1024) return KM_EINVAL;
            g_options.prefer_threads = value;
            return KM_OK;
        case KM_OPT_TILES_PER_WG:
            if (value < 0 || value > 4096) return KM_EINVAL;
            g_options.tiles_per_wg = value;
            return KM_OK;
        case KM_OPT_PAIR_INTERLEAVE:
            if (value != 0 && value != 1) return KM_EINVAL;
            g_options.pair_interleave = value;
            return KM_OK;
        case KM_OPT_TILE_ORDER:
            if (value != -1 && value != 0 && value != 2 && value != 3) return KM_EINVAL;
            g_options.tile_order = value;
            return KM_OK;
        case KM_OPT_PREFER_INSTANCE:
            if (value < 0 || value > g_num_variants + 1) return KM_EINVAL;
            g_options.prefer_instance = value;
            return KM_OK;
        case KM_OPT_INSTANCE_COUNT:
            return KM_EINVAL;                      // read-only
        case KM_OPT_KEEP_MIB:
            if (value < 0 || value > (1 << 20)) return KM_EINVAL;
            g_keep_mib = value;
            return KM_OK;
        case KM_OPT_PROFILE:
            if (value != 0 && value != 1) return KM_EINVAL;
            if (value == 1 && g_profile == 0)      // a fresh history on every device
                for (DeviceState& ds : g_dev) { ds.call_first.clear(); ds.call_steps.clear(); ds.events_used = 0; }
            g_profile = value;
            return KM_OK;
    }
    return KM_EINVAL;
}

km_status kronmatmul_get_option(km_option option, int* value)
{
    if (!value) return KM_EINVAL;
    std::lock_guard<std::mutex> lock(g_mutex);
    switch (option) {
        case KM_OPT_KERNELS: *value = g_options.kernels; return KM_OK;
        case KM_OPT_MAX_FUSE: *value = g_options.max_fuse; return KM_OK;
        case KM_OPT_PROFILE: *value = g_profile; return KM_OK;
        case KM_OPT_KEEP_MIB: *value = g_keep_mib; return KM_OK;
        case KM_OPT_PREFER_TILE: *value = g_options.prefer_tile; return KM_OK;
        case KM_OPT_PREFER_THREADS: *value = g_options.prefer_threads; return KM_OK;
        case KM_OPT_TILES_PER_WG: *value = g_options.tiles_per_wg; return KM_OK;
        case KM_OPT_PAIR_INTERLEAVE: *value = g_options.pair_interleave; return KM_OK;
        case KM_OPT_TILE_ORDER: *value = g_options.tile_order; return KM_OK;
        case KM_OPT_PREFER_INSTANCE: *value = g_options.prefer_instance; return KM_OK;
        case KM_OPT_INSTANCE_COUNT: *value = g_num_variants; return KM_OK;
    }
    return KM_EINVAL;
}

static km_status profile_query(bool mean, float* ms, int cap, int* nsteps, int* ncalls)
{
    if (!nsteps || cap < 0 || (cap > 0 && !ms)) return KM_EINVAL;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return KM_ELAUNCH;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState& ds = g_dev[dev];
    const int calls = (int)ds.call_first.size();
    if (calls == 0) return KM_EINVAL;
    const int n = ds.call_steps[calls - 1];
    const int c0 = mean ? 0 : calls - 1;
    for (int c = c0; c < calls; ++c)
        if (ds.call_steps[c] != n) return KM_EINVAL;     // a mean needs calls of one plan
    if (hipEventSynchronize(ds.events[ds.call_first[calls - 1] + n]) != hipSuccess) return KM_ELAUNCH;
    *nsteps = n;
    if (ncalls) *ncalls = calls - c0;
    for (int i = 0; i < n && i < cap; ++i) {
        double sum = 0;
        for (int c = c0; c < calls; ++c) {
            float t = 0;
            const int e = ds.call_first[c] + i;
            if (hipEventElapsedTime(&t, ds.events[e], ds.events[e + 1]) != hipSuccess) return KM_ELAUNCH;
            sum += t;
        }
        ms[i] = (float)(sum / (calls - c0));
    }
    return KM_OK;
}

km_status kronmatmul_last_profile(float* ms, int cap, int* nsteps)
{
    return profile_query(false, ms, cap, nsteps, nullptr);
}

km_status kronmatmul_mean_profile(float* ms, int cap, int* nsteps, int* ncalls)
{
    return profile_query(true, ms, cap, nsteps, ncalls);
}

km_status kronmatmul_clock_probe(unsigned long long* ticks, int micros, void* stream)
{
    if (!ticks || !aligned(ticks, 8) || micros < 1 || micros > 1000000) return KM_EINVAL;
    hipLaunchKernelGGL(clock_probe_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, ticks,
                       (unsigned long long)micros * 100ull);
    return hipGetLastError() == hipSuccess ? KM_OK : KM_ELAUNCH;
}

km_status kronmatmul_release(void)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return KM_ELAUNCH;
    DeviceState& ds = g_dev[dev];
    if (hipDeviceSynchronize() != hipSuccess) return KM_ELAUNCH;
    if (ds.ws) (void)hipFree(ds.ws);
    ds.ws = nullptr; ds.ws_bytes = 0;
    for (hipEvent_t e : ds.events) (void)hipEventDestroy(e);
    ds.events.clear();
    ds.call_first.clear(); ds.call_steps.clear(); ds.events_used = 0;
    g_plan_cache.clear();        // measured plans included: they were timed on this device
    return KM_OK;
}

const char* kronmatmul_status_string(km_status status)
{
    switch (status) {
        case KM_OK: return "ok";
        case KM_EINVAL: return "invalid argument";
        case KM_ENOMEM: return "workspace too small or allocation failed";
        case KM_ELAUNCH: return "HIP launch or runtime error";
        case KM_EUNSUPPORTED: return "shape not supported";
    }
    return "unknown status";
}

const char* kronmatmul_kernel_name(int kernel)
{
    switch (kernel) {
        case KM_KERNEL_GENERIC: return "generic";
        case KM_KERNEL_FUSED: return "fused";
        case KM_KERNEL_MFMA: return "mfma";
        case KM_KERNEL_SHUFFLE: return "shuffle";
        case KM_KERNEL_ROWS: return "rows";
        case KM_KERNEL_MFMA_ANY: return "mfma-any";
    }
    return "unknown";
}

}  // extern "C"
