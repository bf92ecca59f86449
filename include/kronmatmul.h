/*
 * kronmatmul -- Kronecker matrix-matrix multiplication on AMD MI355X (gfx950).
 *
 *     Y = X * (F[0] (x) F[1] (x) ... (x) F[N-1])
 *
 * X is M x prod(P[i]), F[i] is P[i] x Q[i], Y is M x prod(Q[i]) (the "Kron-Matmul" of the paper's
 * section 2).  The product is evaluated by the paper's sliced-multiply iteration (section 3,
 * Algorithm 1): factors are applied from the last to the first; applying a P x Q factor to a row of
 * width K contracts each of the K/P contiguous length-P slices with each factor column and stores
 * the value for (slice s, column q) at column q*(K/P)+s, which is already the layout the next
 * iteration reads.  Runs of consecutive factors are fused into one kernel whose intermediates stay
 * in LDS (section 4.2).
 *
 * Conventions for every entry point
 *   - All matrices are dense, row-major, without padding.
 *   - P, Q and the array F itself are HOST memory; X, Y, the workspace and every F[i] are DEVICE
 *     memory on the current HIP device.  F[0] is the leftmost factor (slowest index digit).
 *   - X, Y and the workspace must be 16-byte aligned (hipMalloc and torch allocations are); factors
 *     need only their element's alignment.  KM_EINVAL otherwise.
 *   - The caller owns every buffer.  X and the factors are only read, and nothing outside the
 *     M x prod(P) elements of X, the P[i] x Q[i] elements of F[i], the M x prod(Q) elements of Y and
 *     the stated workspace bytes is read or written.  Y may be used as scratch for intermediates
 *     before it receives the result.  X, Y and the workspace must not overlap: KM_EINVAL if they do.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is enqueued
 *     on it; no entry point synchronises with the device unless stated.
 *   - Errors are returned, never thrown; nothing calls exit().  M == 0 is a successful no-op.
 *   - Entry points are thread-safe with respect to each other; concurrent calls that share the
 *     library-managed workspace (kronmatmul) on different streams are serialised by the caller.
 *     Options (kronmatmul_set_option) are process-wide, not per thread: a call uses the values in
 *     force when it starts.
 *   - Graph capture: kronmatmul_ws and kronmatmul_transposed_ws only enqueue kernels, with one
 *     exception: the first launch of a kernel instance on a device raises that kernel's LDS limit
 *     (hipFuncSetAttribute).  Call kronmatmul_prepare for the problem before capturing, or make one
 *     uncaptured call first.
 */
#ifndef KRONMATMUL_H
#define KRONMATMUL_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { KM_F32 = 0, KM_F64 = 1 } km_dtype;

typedef enum {
    KM_OK = 0,
    KM_EINVAL = 1,       /* bad shape, null pointer, unknown dtype/option, size overflow          */
    KM_ENOMEM = 2,       /* workspace too small, or the library could not allocate its own        */
    KM_ELAUNCH = 3,      /* HIP reported an error on launch / event / query                        */
    KM_EUNSUPPORTED = 4  /* no kernel can run this shape on this device                            */
} km_status;

/* Kernel families a plan step can use. */
typedef enum {
    KM_KERNEL_GENERIC = 0,  /* one factor, any P and Q: LDS-tiled FMA kernel                       */
    KM_KERNEL_FUSED = 1,    /* up to 12 consecutive small factors, tile resident in LDS (section 4.2) */
    KM_KERNEL_MFMA = 2,     /* factors with P and Q multiples of 16: slice contraction on MFMA     */
    KM_KERNEL_SHUFFLE = 3,  /* one 8x8 fp32 factor, no LDS: P-reduction by wavefront lane exchanges */
    KM_KERNEL_ROWS = 4,     /* every factor of a short row in one launch, any shapes: the row and its
                               intermediates stay in LDS (section 4.2's fusion with the row as tile) */
    KM_KERNEL_MFMA_ANY = 5  /* one factor of run-time shape on MFMA (zero-padded to 16s; slices of any alignment) */
} km_kernel;

/* Buffers a plan step reads or writes. */
typedef enum { KM_BUF_X = 0, KM_BUF_Y = 1, KM_BUF_WS0 = 2, KM_BUF_WS1 = 3 } km_buffer;

/* One kernel launch of a plan.  Factors first_factor .. first_factor+num_factors-1 (indices into
 * F, applied last to first) map rows of width k_in to rows of width k_out. */
typedef struct {
    int kernel;            /* km_kernel                                                            */
    int first_factor;      /* lowest factor index in this step                                     */
    int num_factors;       /* factors fused in this launch (N_fused of section 4.2)                */
    int tile_slices;       /* contiguous output run per tile and fused column (T_K / prod P)       */
    long long k_in;        /* row width read                                                       */
    long long k_out;       /* row width written                                                    */
    int src;               /* km_buffer read                                                       */
    int dst;               /* km_buffer written                                                    */
    long long grid;        /* workgroups launched                                                  */
    int block;             /* threads per workgroup                                                */
    int lds_bytes;         /* LDS per workgroup                                                    */
    int variant;           /* index of the compiled kernel instance, for reports                   */
    int tiles_per_wg;      /* tiles one workgroup walks over (0: one tile per workgroup)           */
    int tile_order;        /* walk: 0 contiguous range, 1 interleaved pairs, 2 strided by the grid,
                              3 strided inside the XCD's eighth of the tiles                       */
    int tile_rows;         /* rows per tile (the T_M of section 4); above 1 only when a tile holds
                              whole rows, tile_slices then being the slices of one row            */
} km_plan_step;

/* Bytes of device workspace kronmatmul_ws needs for this problem (0 when one launch suffices).
 * Follows Algorithm 1's two swapped intermediates, except that Y stands in for one of them when it
 * is wide enough and X is read in place.  Pure host computation. */
km_status kronmatmul_workspace_size(int M, int N, const int* P, const int* Q, km_dtype dtype,
                                    size_t* bytes);

/* Y = X * (F[0] (x) ... (x) F[N-1]) with a workspace the library allocates on first use and keeps
 * (one per device, grown on demand with hipMalloc, which may synchronise the device; freed by
 * kronmatmul_release). */
km_status kronmatmul(int M, int N, const int* P, const int* Q,
                     const void* X, const void* const* F, void* Y,
                     km_dtype dtype, void* stream);

/* Set-up for a problem on the current HIP device, outside any timed or captured region: plans it
 * (the plan is memoised) and sets the attributes of every kernel instance the plan launches, so that
 * later kronmatmul_ws calls for this problem do nothing but enqueue kernels.  Also looks up the
 * address of kronmatmul_static's array on this device.  Launches nothing. */
km_status kronmatmul_prepare(int M, int N, const int* P, const int* Q, km_dtype dtype);

/* Same, with a caller-provided device workspace of at least kronmatmul_workspace_size bytes
 * (may be NULL when that size is 0).  Never allocates.  KM_ENOMEM if workspace_bytes is too small. */
km_status kronmatmul_ws(int M, int N, const int* P, const int* Q,
                        const void* X, const void* const* F, void* Y,
                        km_dtype dtype, void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid it): kronmatmul_ws with the workspace taken from an array that is part of the
 * library's device code, KM_STATIC_SCRATCH_BYTES per GPU, held from the moment the library's code is
 * loaded on a GPU until the process ends.  Calls no hipMalloc / hipFree and creates no events; the
 * caller still passes X, F and Y.  KM_ENOMEM, before anything is enqueued, if the problem's
 * intermediates (kronmatmul_workspace_size) exceed KM_STATIC_SCRATCH_BYTES.  The array's address on
 * a device is looked up on the first call there, or by kronmatmul_prepare.  Every call on a GPU uses
 * that GPU's one array: calls that overlap in time on one GPU (different streams or threads) race
 * and must be serialised by the caller.  Nothing in it needs clearing between calls: every
 * intermediate element is written by one launch before the next launch reads it.  Calls made while
 * KM_OPT_PROFILE is 1 are not profiled. */
#define KM_STATIC_SCRATCH_BYTES (16u << 20)
km_status kronmatmul_static(int M, int N, const int* P, const int* Q,
                            const void* X, const void* const* F, void* Y,
                            km_dtype dtype, void* stream);

/* The same product with every factor given transposed: Ft[i] is the Q[i] x P[i] row-major array
 * whose transpose is the factor applied, Y = X * (Ft[0]^T (x) ... (x) Ft[N-1]^T); X is M x prod(P),
 * Y is M x prod(Q) as before.  (The operation is the paper's, section 2; this form serves callers
 * that hold the transposes, e.g. the gradient dX = dY * (F[0]^T (x) ...) of a Kron-Matmul.)  The
 * factors, which are small, are first copied in P x Q layout behind the plan's workspace by one
 * extra launch on `stream`; everything after that is the path of kronmatmul.  The workspace is
 * larger by those copies: kronmatmul_transposed_workspace_size.  kronmatmul_transposed uses the
 * library's cached workspace, kronmatmul_transposed_ws the caller's and never allocates. */
km_status kronmatmul_transposed_workspace_size(int M, int N, const int* P, const int* Q, km_dtype dtype,
                                               size_t* bytes);
km_status kronmatmul_transposed(int M, int N, const int* P, const int* Q,
                                const void* X, const void* const* Ft, void* Y,
                                km_dtype dtype, void* stream);
km_status kronmatmul_transposed_ws(int M, int N, const int* P, const int* Q,
                                   const void* X, const void* const* Ft, void* Y,
                                   km_dtype dtype, void* workspace, size_t workspace_bytes, void* stream);

/* The launches kronmatmul would issue for this problem, in order.  Writes at most `cap` steps and
 * the total count to *nsteps.  Pure host computation (no device needed). */
km_status kronmatmul_plan(int M, int N, const int* P, const int* Q, km_dtype dtype,
                          km_plan_step* steps, int cap, int* nsteps);

/* Autotuning (the search over tile sizes of section 4.3, done at run time on the device that will
 * run the problem): times every compiled instance, tile length and tile walk that fits each group
 * of consecutive factors on synthetic rows of the problem's size, plans on the measured times, and
 * keeps that plan for later kronmatmul / kronmatmul_ws / kronmatmul_plan calls with this problem and
 * the options in force now, if its launches in sequence beat the cost-model plan and need no more
 * workspace than that plan (otherwise that one is kept: a workspace sized with
 * kronmatmul_workspace_size before tuning stays large enough).  The plan stays until
 * kronmatmul_release.  Allocates and frees device memory (two
 * buffers of M x the widest intermediate, plus the plan's workspace; KM_ENOMEM if that fails),
 * enqueues on `stream` and waits for it: not for use under graph capture.  Results do not depend on
 * the plan beyond rounding order.  tuned_ms / default_ms (host, may be NULL) receive the time of the
 * kept plan and of the cost-model plan, in milliseconds per call. */
km_status kronmatmul_tune(int M, int N, const int* P, const int* Q, km_dtype dtype, void* stream,
                          float* tuned_ms, float* default_ms);

/* Output column, within a row of the intermediate, of element `local_col` of a tile after a fused
 * group of factors with prod(P) = p_group was applied to a row of width k_in cut into contiguous
 * tiles of tile_k elements (section 4.2, the store of Figure 7; with one factor it is the store of
 * Figure 3).  local_col counts the tile's final contents in (fused column, slice) order.  Returns -1
 * on invalid arguments.  Pure host computation, exported so the index map can be tested. */
long long kronmatmul_store_column(long long k_in, long long p_group, long long tile_k,
                                  long long tile_index, long long local_col);

/* Floating-point operations (2 per multiply-add, summed over the N iterations of Algorithm 1) and
 * the bytes the planned launches must move (rows read + rows written per launch, plus factors). */
km_status kronmatmul_cost(int M, int N, const int* P, const int* Q, km_dtype dtype,
                          double* flops, double* planned_bytes);

/* Options (process-wide).  KM_OPT_KERNELS, KM_OPT_MAX_FUSE and KM_OPT_PROFILE are for users; the
 * options called "tuning aid" force the planner's hand and exist for tests and sweeps only: they are
 * not meant to be changed while other threads are making calls.  KM_OPT_KERNELS: bit mask of km_kernel families the planner may use (bit k = family k;
 * the generic family is always allowed; default 55: the shuffle family is off because the LDS-tiled
 * kernels measured faster).  KM_OPT_MAX_FUSE: upper limit on factors per launch (1 to 16, default 16).
 * KM_OPT_PROFILE: when 1, every launch is bracketed by HIP events on the caller's stream.
 * KM_OPT_PREFER_TILE / KM_OPT_PREFER_THREADS: tuning aids; when non-zero the planner prefers compiled
 * instances with that tile_slices / workgroup size where one fits the shape (0 = automatic).
 * KM_OPT_TILES_PER_WG: tuning aid; consecutive tiles per workgroup of the MFMA kernels (0 = automatic).
 * KM_OPT_PAIR_INTERLEAVE: tuning aid (default 1); MFMA kernels whose output runs are shorter than a
 * cache line give alternate tiles to pairs of workgroups that share an XCD.
 * KM_OPT_TILE_ORDER: tuning aid (default -1); persistent MFMA kernels walk over a contiguous range of
 * tiles (0), over tiles strided by the grid size (2), or strided inside a contiguous eighth of the
 * tiles per XCD (3; taken as 2 when tiles or grid do not split by 8); -1 leaves the choice between 2
 * and 3 to the compiled instance.
 * KM_OPT_PREFER_INSTANCE: tuning aid; k > 0 makes the planner take compiled instance k - 1 (the
 * `variant` of a plan step) wherever it fits the shape (0 = automatic); k = instance count + 1
 * makes it take the whole-row kernel (KM_KERNEL_ROWS) whenever the rows fit LDS.
 * KM_OPT_INSTANCE_COUNT: read-only; the number of compiled instances.
 * KM_OPT_KEEP_MIB: tuning aid (default 320); a launch that is not a call's last and writes between 48
 * and this many MiB (four times as many for the KM_KERNEL_FUSED family) uses ordinary instead of
 * non-temporal stores, so that the next launch finds part of the intermediate in the chip's
 * last-level cache (256 MB); 0 = non-temporal always.  It takes effect on the next call and changes
 * no result. */
typedef enum { KM_OPT_KERNELS = 0, KM_OPT_MAX_FUSE = 1, KM_OPT_PROFILE = 2, KM_OPT_PREFER_TILE = 3,
               KM_OPT_PREFER_THREADS = 4, KM_OPT_TILES_PER_WG = 5, KM_OPT_PAIR_INTERLEAVE = 6, KM_OPT_TILE_ORDER = 7,
               KM_OPT_PREFER_INSTANCE = 8, KM_OPT_INSTANCE_COUNT = 9, KM_OPT_KEEP_MIB = 10 } km_option;
km_status kronmatmul_set_option(km_option option, int value);
km_status kronmatmul_get_option(km_option option, int* value);

/* Per-launch durations (milliseconds) of the most recent profiled call on the current device, in
 * plan order.  Synchronises with the events of that call.  KM_EINVAL if nothing was profiled. */
km_status kronmatmul_last_profile(float* ms, int cap, int* nsteps);

/* Per-launch durations averaged over every call made on the current device since KM_OPT_PROFILE was
 * last switched from 0 to 1 (at most 4096 calls are kept; later ones run unprofiled).  All those
 * calls must have had the same number of launches, else KM_EINVAL.  *ncalls receives their count. */
km_status kronmatmul_mean_profile(float* ms, int cap, int* nsteps, int* ncalls);

/* Measurement aid: enqueues on `stream` a one-wavefront kernel that sleeps for about `micros`
 * microseconds (1 to 1,000,000) and writes to `ticks` (device memory, two 64-bit unsigned integers,
 * 8-byte aligned) how far the shader clock and the constant 100 MHz clock advanced meanwhile:
 * shader MHz = 100 * ticks[0] / ticks[1].  Launched on a second stream next to Kron-Matmul calls
 * it shows the clock the chip sustains under their load, which is what the matrix cores' peak
 * (quoted at the maximum clock) has to be scaled by.  The kernel ends by itself after `micros`, or
 * after a fixed number of sleep steps (a few seconds) whatever the clocks read.  Does not
 * synchronise.  KM_EINVAL for a null or misaligned pointer or micros out of range. */
km_status kronmatmul_clock_probe(unsigned long long* ticks, int micros, void* stream);

/* Frees the library-managed workspaces and profiling events (synchronises the device). */
km_status kronmatmul_release(void);

const char* kronmatmul_status_string(km_status status);
const char* kronmatmul_kernel_name(int kernel);

#ifdef __cplusplus
}
#endif
#endif /* KRONMATMUL_H */
