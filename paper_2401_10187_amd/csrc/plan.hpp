// Host-side planner: turns a problem (M, factor shapes, dtype) into the list of kernel launches
// that evaluates Algorithm 1, last factor first, and assigns the buffers the launches read and
// write (the two swapped intermediates of Algorithm 1; Y stands in for one of them when it is wide
// enough, and the first launch reads X in place).  Pure host code, no HIP calls.
#pragma once
#include <stdint.h>
#include <stddef.h>
#include <vector>
#include "../../include/kronmatmul.h"

namespace km {

// One compiled kernel instance the planner can choose.
struct Variant {
    int kernel;        // km_kernel family
    int dtype;         // km_dtype
    int P, Q;          // factor shape it is compiled for (0 = any)
    int num_factors;   // factors per launch
    int tile_slices;   // S_t: run of consecutive output columns a tile produces per fused column
    int threads;       // workgroup size
    int lds_bytes;     // LDS per workgroup
    int rows_per_tile; // rows of X a workgroup handles together
    int persistent;    // >0: a workgroup walks over several tiles (see tiles_per_wg); 1: in any of the
                       // three tile orders, 2: contiguous or grid-strided only
    int flexible;      // 1: tile_slices is an upper limit; the launch picks a divisor of K/prod(P)
    float slowdown;    // measured cost relative to an HBM-bound launch of the same bytes (planner weight)
    const char* name;
    int lds_per_slice; // flexible instances: LDS bytes per slice of the tile (lds_bytes is the maximum)
    int thread_elems;  // flexible instances: contiguous elements of a tile that one thread multiplies first
    int max_srow;      // > 0: only for rows of at most this many slices of the group (K / prod P)
    int min_tiles;     // > 0: only planned for launches of at least this many tiles (the tuner still tries it)
    int walk;          // > 0: tiles per workgroup of a persistent instance, instead of the rule of tiles_per_wg();
                       // -1: as many as make the grid one round of the workgroups the chip holds at once
    int xcd_order;     // 1: persistent instance that prefers tile order 3 (each XCD walks its own eighth of the tiles)
    int lds_slack;     // flexible instances: LDS bytes a launch needs on top of lds_per_slice * tile_slices
    int mix[9];        // instances whose stages have their own factor shapes: (P, Q, factors) of up to three
                       // stages in order of application (P, Q above are the first stage's); all 0 otherwise
};

// Do factors [f - nf + 1, f] (applied from f downwards) have the shapes instance c is compiled for?
inline bool shapes_match(const Variant& c, const std::vector<int>& P, const std::vector<int>& Q, int f, int nf)
{
    if (c.num_factors != nf) return false;
    if (c.mix[2] == 0) {                                  // one shape for every factor of the group
        for (int i = f - nf + 1; i <= f; ++i)
            if (P[i] != c.P || Q[i] != c.Q) return false;
        return true;
    }
    int at = f;
    for (int j = 0; j < 3; ++j)
        for (int k = 0; k < c.mix[3 * j + 2]; ++k, --at)
            if (at < f - nf + 1 || P[at] != c.mix[3 * j] || Q[at] != c.mix[3 * j + 1]) return false;
    return at == f - nf;
}

// LDS a launch of the instance asks for when its tiles hold `tile_slices` slices.
inline int launch_lds_bytes(const Variant& c, int tile_slices)
{
    if (!c.flexible || c.lds_per_slice <= 0) return c.lds_bytes;
    const int64_t b = ((int64_t)c.lds_per_slice * tile_slices + 15) / 16 * 16 + c.lds_slack;
    return b < c.lds_bytes ? (int)b : c.lds_bytes;
}

// Tiles handled by one workgroup of a persistent instance; `hint` > 0 forces the value.
// Measured with the autotuner on this chip: a workgroup loads its factors once, so with large
// factors (16 KB and more) long walks pay (64x64 fp32: walks of 32-64 tiles are 7 % faster than
// walks of 5), while with small factors every tile beyond the amortisation point costs workgroups
// in flight (16x16: walks of 3-4 tiles are 10 % slower than one tile per workgroup).  Walks are
// powers of two so that the usual power-of-two tile counts split evenly over the grid.
// Instances that fill most of a compute unit's LDS run one or two workgroups per unit and need the
// walk to overlap their loads with their stores: at least 4 tiles above 64 KB, 32 above 80 KB.
inline int64_t tiles_per_wg(int64_t num_tiles, int hint, int64_t factor_elems, int64_t tile_elems,
                            int lds_bytes, size_t esize, int instance_walk = 0)
{
    if (hint > 0) return hint;
    const int64_t want = (10 * factor_elems + tile_elems - 1) / tile_elems;
    int64_t t = 1;
    while (t < want && t < 32) t *= 2;
    if ((size_t)factor_elems * esize >= 16 * 1024) t = 32;
    if (lds_bytes > 64 * 1024 && t < 4) t = 4;
    if (lds_bytes > 80 * 1024) t = 32;
    if (instance_walk > 0) t = instance_walk;          // measured per instance
    // two workgroups per compute unit at least; four when the instance is light (small factor, at most
    // 64 KB of LDS): 1024 x 64x64^2 is 28 % faster with 1024 workgroups than with 512; but one per unit
    // is enough when loading the factor costs a workgroup as much as a tile does (16 x 64x64^3 fp64:
    // 256 workgroups walking 4 tiles each are 28 % faster than 1024 with one tile)
    const bool heavy = (size_t)factor_elems * esize >= 64 * 1024 || lds_bytes > 64 * 1024;
    // (factors of 16 KB and more: with 32x32 factors, whose tiles are as large as the factor too, four
    // workgroups per unit win again: 4096 x 32x32^2 fp64 0.044 -> 0.027 ms, 16 x 32x32^3 0.014 -> 0.011)
    const int64_t fewest = heavy ? 512 : ((size_t)factor_elems * esize >= 16 * 1024 && factor_elems >= tile_elems ? 256 : 1024);
    while (t > 1 && num_tiles / t < fewest) t /= 2;
    return t;
}

struct Problem {
    int64_t M = 0;
    int N = 0;
    std::vector<int> P, Q;
    int dtype = 0;
    int64_t k_in = 1, k_out = 1;   // prod P, prod Q
    size_t esize = 4;
};

struct Plan {
    std::vector<km_plan_step> steps;
    size_t ws0_bytes = 0, ws1_bytes = 0;   // the two intermediates (ws1 unused when Y can serve)
    double flops = 0, bytes = 0;
};

struct Options {
    int kernels = 0x37;   // bit mask of km_kernel families
    int max_fuse = 16;
    int prefer_tile = 0;      // tuning: choose instances with this tile_slices when one fits
    int prefer_threads = 0;   // tuning: ... with this workgroup size
    int tiles_per_wg = 0;     // tuning: tiles per workgroup of persistent instances (0 = automatic)
    int pair_interleave = 1;  // neighbouring tiles with short output runs go to workgroup pairs
    int prefer_instance = 0;  // tuning: k > 0 = take compiled instance k - 1 wherever it fits
    int tile_order = -1;      // persistent kernels: 0 = contiguous tile ranges, 2 = tiles strided by the grid,
                              // 3 = strided inside the XCD's own eighth of the tiles, -1 = the instance's
                              // preference (3 where it asks for it and the tiles split by 8, else 2)
};

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

#if defined(__HIPCC__)
#define KM_HOST_DEVICE __host__ __device__
#else
#define KM_HOST_DEVICE
#endif
// A run of `valid` elements that starts `mis` elements (0 <= mis < vn) above a 16-byte boundary is
// moved in vectors of vn elements counted from that boundary: unaligned_vectors() of them touch the
// run; the first unaligned_whole_vectors() are loaded or stored whole.  Those lie inside
// [-mis, valid): the elements below the run exist whenever mis > 0 (buffers start on 16-byte
// boundaries), so a whole vector never leaves the buffer.  What is left, the part of the last vector
// that belongs to the run, is moved element by element.
KM_HOST_DEVICE inline int unaligned_vectors(int valid, int mis, int vn) { return (valid + mis + vn - 1) / vn; }
KM_HOST_DEVICE inline int unaligned_whole_vectors(int valid, int mis, int vn) { return (valid + mis) / vn; }

// Validates the shapes and fills the derived sizes.  Products must stay below 2^62 elements.
inline km_status make_problem(int M, int N, const int* P, const int* Q, int dtype, Problem& pr)
{
    if (M < 0 || N < 1 || N > 64 || !P || !Q) return KM_EINVAL;
    if (dtype != KM_F32 && dtype != KM_F64) return KM_EINVAL;
    pr.M = M; pr.N = N; pr.dtype = dtype; pr.esize = dtype == KM_F32 ? 4 : 8;
    pr.P.assign(P, P + N); pr.Q.assign(Q, Q + N);
    const int64_t lim = (int64_t)1 << 40;   // elements per row; M * width * esize must fit in int64
    int64_t kin = 1, kout = 1;
    for (int i = 0; i < N; ++i) {
        if (P[i] < 1 || Q[i] < 1) return KM_EINVAL;
        if (kin > lim / P[i] || kout > lim / Q[i]) return KM_EINVAL;
        kin *= P[i]; kout *= Q[i];
    }
    // every intermediate width Q_N..Q_f * P_1..P_{f-1}
    int64_t w = kin;
    for (int f = N - 1; f >= 0; --f) {
        w = w / P[f];
        if (w > lim / Q[f]) return KM_EINVAL;
        w *= Q[f];
        if (M > 0 && w > ((int64_t)1 << 59) / M) return KM_EINVAL;
    }
    if (M > 0 && kin > ((int64_t)1 << 59) / M) return KM_EINVAL;
    pr.k_in = kin; pr.k_out = kout;
    return KM_OK;
}

// Output column of local element c of tile `tile_index` after a fused group (section 4.2): the
// tile's final contents are ordered (fused column qq, slice r) with r < S_t = tile_k / p_group, and
// the row of the intermediate holds, for each qq, all K_in / p_group slices contiguously.
inline int64_t store_column(int64_t k_in, int64_t p_group, int64_t tile_k, int64_t tile_index,
                            int64_t local_col)
{
    if (k_in <= 0 || p_group <= 0 || tile_k <= 0 || k_in % p_group || tile_k % p_group ||
        k_in % tile_k || tile_index < 0 || tile_index >= k_in / tile_k || local_col < 0)
        return -1;
    const int64_t s_tile = tile_k / p_group;      // slices of the fused group inside the tile
    const int64_t s_row = k_in / p_group;         // ... inside the whole row
    const int64_t qq = local_col / s_tile;
    const int64_t r = local_col % s_tile;
    return qq * s_row + tile_index * s_tile + r;
}

// Column blocks (of 16) per unit of the run-time-shape MFMA kernel for a factor with Q columns: one or
// two for factors that narrow, else the width among 4, 5 and 3 that leaves the fewest padded blocks
// (narrower units would re-read the slices once per 16 or 32 columns).
inline int any_column_blocks(int Q)
{
    const int blocks = (Q + 15) / 16;
    if (blocks <= 2) return blocks < 1 ? 1 : blocks;
    int best = 4, waste = (4 - blocks % 4) % 4 * 1000 / ((blocks + 3) / 4 * 4);
    const int others[2] = {5, 3};
    for (int cb : others) {
        const int w = (cb - blocks % cb) % cb * 1000 / ((blocks + cb - 1) / cb * cb);
        if (w < waste) { waste = w; best = cb; }
    }
    return best;
}

// Units of work of the kernels without compiled shapes: (tile t of `tiles` slice tiles, group c of
// `groups` factor-column groups).  The groups of one tile read the same slices, so they should meet in
// one L2: workgroup b runs on XCD b % 8, hence within each run of 8 tiles the unit number is
// b = (8 * (t / 8) * groups) + c * 8 + t % 8; the last tiles % 8 tiles are numbered plainly.
KM_HOST_DEVICE inline void unit_of(int64_t b, int64_t tiles, int groups, int64_t& t, int& c)
{
    const int64_t full = tiles / 8 * 8 * groups;
    if (b < full) {
        t = b / (8 * groups) * 8 + b % 8;
        c = (int)(b / 8 % groups);
    } else {
        b -= full;
        t = tiles / 8 * 8 + b / groups;
        c = (int)(b % groups);
    }
}

// A compiled instance chosen for one group of factors, with the slices per tile it will run with.
// What the planner needs to know of the generic kernel: a workgroup of `threads` work-items takes
// `tile_slices` slices and `tile_cols` factor columns at a time.
struct GenericKernel {
    int threads, tile_slices, tile_cols, lds_bytes;
    // the whole-row kernel: a workgroup of row_threads_many work-items (row_threads_few when there
    // are at most row_few_rows rows) applies up to row_max_factors factors to one row held, with the
    // factors, in at most row_lds_limit bytes of LDS
    int row_threads_many, row_threads_few, row_few_rows, row_lds_limit, row_max_factors;
    // the run-time-shape MFMA kernel: a workgroup of any_threads work-items takes
    // any_tile_slices slices and 16 * any_column_blocks(Q) factor columns at a time, chunks of
    // any_row_bytes per slice in LDS rows padded by one 16-byte unit; slices of at most half a chunk
    // take the narrow shape: twice the slices, chunks of half the bytes
    int any_threads, any_tile_slices, any_row_bytes;
};

inline bool any_narrow(const GenericKernel& gen, int P, size_t esize) { return (size_t)P * esize * 2 <= (size_t)gen.any_row_bytes; }
inline int any_unit_slices(const GenericKernel& gen, int P, size_t esize)
{
    return any_narrow(gen, P, esize) ? 2 * gen.any_tile_slices : gen.any_tile_slices;
}
inline int any_lds_bytes(const GenericKernel& gen, int P, int Q, size_t esize)
{
    const int row = any_narrow(gen, P, esize) ? gen.any_row_bytes / 2 : gen.any_row_bytes;
    return (any_unit_slices(gen, P, esize) + 16 * any_column_blocks(Q)) * (row + 16);
}

struct Choice {
    bool any_mfma = false;   // with var == nullptr: the run-time-shape MFMA kernel instead of the generic one
    const Variant* var = nullptr;
    int tile_slices = 0;
    int64_t grid = 0;        // tiles (before the persistent-walk division)
    int tiles_per_wg = 0;    // persistent instances: 0 = take the rule of tiles_per_wg()
    int tile_order = -1;     // persistent instances: -1 = take the option
    int tile_rows = 1;       // rows per tile; above 1 the tile holds whole rows (tile_slices = K/prod(P))
};

// Rows a flexible instance puts into one tile when a whole row is shorter than its tile (rows are
// contiguous in memory, so several of them pass through the stages as one long tile): as many as
// fit 48 KB of LDS (three and more workgroups per compute unit, see find_variant), within the
// instance's limit, leaving at least 512 tiles when there are that many rows.
// (the autotuner's finding on 2^6 ... 2^10, 3^5, 4^4, 4^5 and 5^3 with 16 K to 1 M rows: fp32 tiles of
// 24 KB are 5-20 % faster than tiles of 48 KB, fp64 tiles are best at 48 KB: about 6000 elements either way)
inline int64_t whole_rows_lds_budget(size_t esize) { return esize == 4 ? 24 * 1024 : 48 * 1024; }

inline int whole_rows_per_tile(const Variant& c, int64_t s_row, int64_t M, int64_t row_bytes, int64_t row_out_bytes,
                               int64_t lds_budget)
{
    if (!c.flexible || s_row > c.tile_slices / 2 || M < 1024) return 1;   // few rows: one workgroup each
    // rows of 8 KB that do not start on 16-byte boundaries are tiles of their own: the joined rows
    // would be stored element by element (1024 rows of 3^7: one row per tile 0.014 ms, two 0.018 ms)
    if (row_bytes >= 8192 && row_bytes % 16 != 0) return 1;
    int64_t most = c.tile_slices / s_row;
    if (c.lds_per_slice > 0) {
        const int64_t fit = lds_budget / c.lds_per_slice / s_row;
        if (fit < most) most = fit < 1 ? 1 : fit;
    }
    // the output rows are collected in the tile's own LDS: where they are longer than the input rows
    // (Q > P) they set the limit, and the launch asks for their size (build_step)
    if (row_out_bytes > row_bytes) {
        const int64_t room = lds_budget < c.lds_bytes ? lds_budget : c.lds_bytes;
        const int64_t fit = room / row_out_bytes;
        if (fit < most) most = fit < 1 ? 1 : fit;
    }
    if (most > M) most = M;
    while (most > 1 && (M + most - 1) / most < 512) --most;
    return most < 1 ? 1 : (int)most;
}

// Tile order 3 gives each of the 8 XCDs a contiguous eighth of the tiles, walked by grid / 8 workgroups.
inline bool xcd_order_fits(int64_t num_tiles, int64_t grid)
{
    return num_tiles % 8 == 0 && grid % 8 == 0 && grid >= 8;
}

// Workgroups of an instance that one compute unit holds at once (160 KB of LDS, 2048 threads).
inline int64_t resident_per_cu(const Variant& c)
{
    int64_t by_lds = c.lds_bytes > 0 ? (160 * 1024) / c.lds_bytes : 8;
    int64_t by_threads = 2048 / (c.threads > 0 ? c.threads : 256);
    int64_t n = by_lds < by_threads ? by_lds : by_threads;
    return n < 1 ? 1 : (n > 8 ? 8 : n);
}

// The divisors of s_row an instance may run with (fixed instances: their one tile length).
inline void tile_lengths(const Variant& c, int64_t s_row, std::vector<int>& out, int at_most)
{
    out.clear();
    if (!c.flexible) {
        if (s_row % c.tile_slices == 0) out.push_back(c.tile_slices);
        return;
    }
    const int64_t lim = s_row < c.tile_slices ? s_row : c.tile_slices;
    for (int64_t d = lim; d >= 1 && (int)out.size() < at_most; --d)
        if (s_row % d == 0) out.push_back((int)d);
}

// Can factors [f - nf + 1, f] on rows of width k_cur be one tiled launch at all?  Fills prod(P), K/prod(P).
inline bool group_shape(const Problem& pr, int f, int nf, int64_t k_cur, int64_t& pg, int64_t& s_row)
{
    int64_t qg = 1;
    pg = 1;
    for (int i = f - nf + 1; i <= f; ++i) {
        pg *= pr.P[i];
        qg *= pr.Q[i];
        if (pg > ((int64_t)1 << 40) || qg > ((int64_t)1 << 40)) return false;
    }
    if (k_cur % pg) return false;
    s_row = k_cur / pg;
    // the tiled kernels address within a row with 32-bit offsets
    if ((double)s_row * (double)qg * (double)pr.esize >= 2147483648.0) return false;
    if ((double)k_cur * (double)pr.esize >= 2147483648.0) return false;
    return true;
}

// Every (instance, tile length, walk) combination that can run the group: the autotuner's search space.
inline void enumerate_choices(const Variant* table, int count, const Problem& pr, int f, int nf,
                              int64_t k_cur, const Options& opt, std::vector<Choice>& out)
{
    out.clear();
    int64_t pg, s_row;
    if (!group_shape(pr, f, nf, k_cur, pg, s_row)) return;
    int64_t qg_all = 1;
    for (int i = f - nf + 1; i <= f; ++i) qg_all *= pr.Q[i];
    std::vector<int> lens;
    for (int v = 0; v < count; ++v) {
        const Variant& c = table[v];
        if (!(opt.kernels >> c.kernel & 1)) continue;
        if (c.dtype != pr.dtype || !shapes_match(c, pr.P, pr.Q, f, nf)) continue;
        if (c.max_srow > 0 && s_row > c.max_srow) continue;
        if (c.rows_per_tile > 1 && s_row != c.tile_slices) continue;      // tiles of several rows hold whole rows
        tile_lengths(c, s_row, lens, 5);
        const int rows = whole_rows_per_tile(c, s_row, pr.M, s_row * pg * (int64_t)pr.esize, s_row * qg_all * (int64_t)pr.esize, 48 * 1024);
        if (rows > 1) {                                   // whole rows, several per tile, then half and a quarter as many
            for (int r = rows; r >= 2 && r >= rows / 4; r /= 2) {
                Choice ch;
                ch.var = &c;
                ch.tile_slices = (int)s_row;
                ch.tile_rows = r;
                ch.grid = (pr.M + r - 1) / r;
                out.push_back(ch);
            }
        }
        for (int st : lens) {
            Choice ch;
            ch.var = &c;
            ch.tile_slices = st;
            ch.tile_rows = c.rows_per_tile;
            ch.grid = ((pr.M + c.rows_per_tile - 1) / c.rows_per_tile) * (s_row / st);
            if (!c.persistent) { out.push_back(ch); continue; }
            // walks: fixed lengths, and the lengths that make the grid exactly one or two rounds of
            // the workgroups the chip holds at once (every workgroup then gets the same share)
            const int64_t resident = 256 * resident_per_cu(c);
            int64_t walks[6] = {1, 4, 16, 32, (ch.grid + resident - 1) / resident,
                                (ch.grid + 2 * resident - 1) / (2 * resident)};
            for (int i = 0; i < 6; ++i) {
                const int64_t w = walks[i];
                bool seen = w < 1 || w > 4096;
                for (int j = 0; j < i; ++j) seen = seen || walks[j] == w;
                if (seen) continue;
                if (w > 1 && ch.grid / w < 256) continue;      // keep every compute unit busy
                ch.tiles_per_wg = (int)w;
                ch.tile_order = 2;
                out.push_back(ch);
                if (w > 1 && xcd_order_fits(ch.grid, (ch.grid + w - 1) / w)) {
                    ch.tile_order = 3;
                    out.push_back(ch);
                }
            }
        }
    }
}

// Picks the instance for factors [f - nf + 1, f] applied to rows of width k_cur (var == nullptr: none).
// The table is in order of preference (fastest instance on a full machine first).  The first instance
// that fits the shape and still gives the chip enough workgroups wins; failing that, the fitting
// instance with the most workgroups among those whose output runs are at least 32 bytes.  The tuning
// options override both.
inline double launch_cost(const Problem& pr, int64_t k_in, int64_t k_out, const Choice& ch, int generic_P);

inline Choice find_variant(const Variant* table, int count, const Problem& pr, int f, int nf,
                           int64_t k_cur, const Options& opt)
{
    Choice none;
    int64_t pg, s_row;
    if (!group_shape(pr, f, nf, k_cur, pg, s_row)) return none;
    int64_t k_out = s_row;
    for (int i = f - nf + 1; i <= f; ++i) k_out *= pr.Q[i];

    const int64_t enough = 2 * 256;
    Choice first_big, first_tiny, most, wanted, cheapest;
    double cheapest_cost = 0;
    int64_t wanted_score = 0;
    for (int v = 0; v < count; ++v) {
        const Variant& c = table[v];
        if (!(opt.kernels >> c.kernel & 1)) continue;
        if (c.dtype != pr.dtype || !shapes_match(c, pr.P, pr.Q, f, nf)) continue;
        if (c.max_srow > 0 && s_row > c.max_srow) continue;
        if (c.rows_per_tile > 1 && s_row != c.tile_slices) continue;      // tiles of several rows hold whole rows
        if (c.min_tiles > 0 && !c.flexible && pr.M * (s_row / c.tile_slices) < c.min_tiles && opt.prefer_instance != v + 1)
            continue;                                     // too few tiles for this instance (unless it is asked for)
        // slices per tile: fixed, or the best divisor of s_row up to the instance's limit
        int cand[3] = {0, 0, 0};
        int rows = c.rows_per_tile;
        if (!c.flexible) {
            if (s_row % c.tile_slices) continue;
            cand[0] = c.tile_slices;
        } else {
            // Best tile length; best one that still leaves enough workgroups; the tuning wish.
            // "Best" (measured with the autotuner on factors of 3 to 6): output runs that are whole
            // 128-byte lines before anything else (6x6: runs of 1152 bytes are 50 % faster than runs of
            // 1296), then tiles of at most 48 KB of LDS (three and more workgroups per compute unit are
            // 10-30 % faster than two) unless that would cut runs that are not whole lines below 256
            // bytes (6^6: 288-byte runs in 62 KB tiles are 50 % faster than 96-byte runs in 21 KB
            // tiles; rows of odd length, where no run is ever aligned, below 64 bytes: since such tiles
            // are fetched with 16-byte loads and LDS writes, 5^8 with 100-byte runs in 12 KB tiles is
            // 20 % faster than with 500-byte runs in 62 KB tiles), then the longest tile.
            const int64_t lim = s_row < c.tile_slices ? s_row : c.tile_slices;
            const int64_t row_bytes = s_row * (int64_t)pr.esize;
            const bool alignable = (row_bytes & -row_bytes) >= 32;      // some tile length gives 32-byte aligned runs
            // (rows of odd length: 40 KB, four workgroups per compute unit; 1024 x 15^4 fp64 in tiles of 15
            // slices, 27 KB, 0.363 ms, of 25 slices, 45 KB, 0.429)
            const int64_t fit = c.lds_per_slice > 0 ? ((alignable ? 48 : 40) * 1024) / c.lds_per_slice : lim;
            int64_t best_key[2] = {-1, -1};
            int best_tier = 0;
            for (int64_t d = lim; d >= 1; --d) {
                if (s_row % d) continue;
                const int64_t run = d * (int64_t)pr.esize;
                int64_t align = run & -run;                          // largest power of two dividing the run
                if (align > 128) align = 128;
                // (runs of 256 bytes and more that start on 64-byte boundaries count as whole lines: 53 x 10^7
                // in tiles of 80 slices, 320-byte runs, 3.43 ms, of 32 slices, 128-byte runs, 4.07; shorter ones
                // do not: 256 x 12^4 fp64 with 192-byte runs 0.052 ms, with 128-byte runs 0.045)
                if (align == 64 && run >= 256) align = 128;
                const bool small_enough = d <= fit && (align >= 128 || run >= 256 || (!alignable && run >= 64));
                const int64_t key = (align * 2 + (small_enough ? 1 : 0)) * (lim + 1) + d;
                if (key > best_key[0]) { best_key[0] = key; cand[0] = (int)d; }
                // ... that leaves enough workgroups: 512 with at least 16 busy threads, else 96 with at
                // least 4.  A thread takes thread_elems contiguous elements, so short tiles only
                // multiply the wavefronts that run the same instructions for a few lanes (20 rows of
                // 5^6, 125 elements per thread: one-slice tiles 0.037 ms, 5 or 25 slices 0.018 ms).
                const int64_t wgs = pr.M * (s_row / d);
                const int64_t busy = c.thread_elems > 0 ? d * pg / c.thread_elems : d;     // threads with work
                const int tier = (wgs >= enough && (busy >= 16 || d == lim)) ? 2 : (wgs >= 96 && (busy >= 4 || d == lim)) ? 1 : 0;
                if (tier > 0 && (tier > best_tier || (tier == best_tier && key > best_key[1]))) {
                    best_tier = tier; best_key[1] = key; cand[1] = (int)d;
                }
                // ... and the tile length the cost estimate likes best (small problems, see below)
                if ((busy >= 4 || d == lim) && (c.persistent || (double)wgs * (double)c.threads < 4294967296.0)) {
                    Choice t;
                    t.var = &c;
                    t.tile_slices = (int)d;
                    t.grid = wgs;
                    const double tc = launch_cost(pr, k_cur, k_out, t, 0);
                    if (!cheapest.var || tc < cheapest_cost) { cheapest = t; cheapest_cost = tc; }
                }
            }
            if (opt.prefer_tile > 0 && opt.prefer_tile <= c.tile_slices && s_row % opt.prefer_tile == 0) cand[2] = opt.prefer_tile;
            // rows much shorter than the tile: whole rows, several per tile
            rows = whole_rows_per_tile(c, s_row, pr.M, s_row * pg * (int64_t)pr.esize, k_out * (int64_t)pr.esize, whole_rows_lds_budget(pr.esize));
            if (rows > 1) {
                cand[0] = (int)s_row; cand[1] = cand[2] = 0;
                if (cheapest.var == &c) cheapest = Choice();
            }
        }
        for (int k = 0; k < 3; ++k) {
            if (!cand[k]) continue;
            Choice ch;
            ch.var = &c;
            ch.tile_slices = cand[k];
            ch.grid = pr.M * (s_row / cand[k]);
            if (rows > 1) {
                ch.tile_rows = rows;
                ch.grid = (pr.M + rows - 1) / rows;
            }
            // a launch may hold at most 2^32 - 1 work-items (walking instances shrink their grid later)
            if (!c.persistent && (double)ch.grid * (double)c.threads >= 4294967296.0) continue;
            // Tiles under 1 KB leave a workgroup with next to nothing to do (one 8x8 factor on rows of
            // 8 elements: a tile of several whole rows is 10 times faster): they only count when no
            // instance with a decent tile gives the chip enough workgroups.
            const int64_t tile_bytes = (int64_t)ch.tile_slices * ch.tile_rows * pg * (int64_t)pr.esize;
            if (!first_big.var && ch.grid >= enough && tile_bytes >= 1024) first_big = ch;
            if (!first_tiny.var && ch.grid >= enough) first_tiny = ch;
            // among small launches: at least 96 workgroups first (16 rows of 10^4 in 16 tiles of 100
            // slices are twice as slow as in 400 tiles of 4), then output runs of at least 32 bytes,
            // then more workgroups
            auto rank = [&](const Choice& x) {
                return (x.grid >= 96 ? 2 : 0) + ((int64_t)x.tile_slices * (int64_t)pr.esize >= 32 ? 1 : 0);
            };
            if (!most.var || rank(ch) > rank(most) || (rank(ch) == rank(most) && ch.grid > most.grid)) most = ch;
            int64_t sc = 0;
            if (opt.prefer_tile && ch.tile_slices == opt.prefer_tile) sc += 2;
            if (opt.prefer_threads && c.threads == opt.prefer_threads) sc += 1;
            if (opt.prefer_instance && v == opt.prefer_instance - 1) sc += 4;
            if (sc > wanted_score) { wanted = ch; wanted_score = sc; }
        }
    }
    if (wanted.var) return wanted;
    const Choice base = first_big.var ? first_big : (first_tiny.var ? first_tiny : most);
    // The rules above are made for launches that fill the chip.  On small problems they would cut a
    // row into tiles with runs of 16 bytes to reach 512 workgroups, where a hundred workgroups with
    // decent runs finish sooner (16 rows of 6^6: three launches of two factors in 1296 tiles 0.024 ms,
    // two of three factors in 144 tiles of 24 slices 0.013): when the cost estimate rates another
    // tile length of a fitting flexible instance a fifth cheaper than the rules' choice, that one is taken.
    if (base.var && cheapest.var && cheapest_cost < 0.8 * launch_cost(pr, k_cur, k_out, base, 0)) return cheapest;
    return base;
}

// Estimated cost of one launch in "bytes moved at full speed": rows read and written, scaled up for
// short output runs and for the generic kernel, plus a constant per launch.
inline double launch_cost(const Problem& pr, int64_t k_in, int64_t k_out, const Choice& ch, int generic_P)
{
    const double bytes = (double)pr.M * ((double)k_in + (double)k_out) * (double)pr.esize;
    double slow = ch.any_mfma ? 1.5 : 3.0;               // generic kernel; run-time-shape MFMA kernel
    if (ch.var) {
        int64_t run = (int64_t)ch.tile_slices * (int64_t)pr.esize;
        // a tile that holds a whole row writes the whole output row: its runs join up
        if (ch.tile_rows > 1 || ch.grid == pr.M) run = k_out * (int64_t)pr.esize;
        slow = run >= 128 ? 1.0 : (run >= 64 ? 1.25 : (run >= 32 ? 2.5 : 4.0));
        // Rows of odd length: no run ever fills whole lines, so short runs cost less on top (measured
        // with the autotuner: 1024 x 7^6 as 3+3 factors with 28-byte runs is 12 % faster than 2+2+2 with
        // 196-byte runs, 9^5 as 2+3 with 36-byte runs 19 % faster than 2+2+1, 3^11 as 7+4 with 12-byte
        // runs 3 % faster than 4+4+3)
        const int64_t row_bytes = k_out * (int64_t)pr.esize;
        if ((row_bytes & -row_bytes) < 16) slow = run >= 64 ? 1.0 : (run >= 32 ? 1.15 : (run >= 16 ? 1.3 : 1.9));
        slow *= ch.var->slowdown;
    }
    // fewer workgroups than compute units: the launch streams at a matching fraction of the chip's
    // rate (one row of 4^9: seven factors in 16 workgroups take 0.017 ms, four in 256 take 0.005)
    if (ch.var && ch.grid < 256) slow *= 256.0 / (double)(ch.grid < 1 ? 1 : ch.grid);
    double fixed = 2.5e7;                                // ~5 us of launch latency at 5 TB/s
    // the generic kernel walks the slice elements in chunks of 16, a barrier apart: a launch of it
    // takes about 2 us + 0.7 us per chunk even when it moves next to nothing (measured: 5.5 us for
    // P = 65, 4.8 us for P = 52 on ten rows)
    if (!ch.var && !ch.any_mfma) fixed += 1.0e7 + 3.5e6 * (double)((generic_P + 15) / 16);
    // a launch of the run-time-shape MFMA kernel that moves next to nothing takes 6-8 us (measured on the
    // paper's Table 4 sizes: two such launches 12.5 us for 50 x (32x8, 64x128), 15.4 us for 10 x (52x65,
    // 50x20), where the whole-row kernel takes 17 and 13.4)
    if (ch.any_mfma) fixed += 1.25e7;
    return bytes * slow + fixed;
}

// Tile order 1 hands tiles out in groups of 16 workgroups (8 XCDs x 2) that each take every other
// tile of a range of 2 * tiles_per_wg: the grid must be whole groups and the tiles whole ranges.
inline bool pair_order_fits(int64_t num_tiles, int64_t tpw)
{
    const int64_t grid = (num_tiles + tpw - 1) / tpw;
    return grid % 16 == 0 && num_tiles % (2 * tpw) == 0;
}

// One launch of the plan for factors [r - nf, r - 1] with the given choice (var == nullptr: generic).
inline km_plan_step build_step(const Problem& pr, const Options& opt, const Variant* table, int r, int nf,
                               const Choice& ch, const std::vector<int64_t>& width,
                               const GenericKernel& gen)
{
    const int f = r - 1;
    km_plan_step st = {};
    st.first_factor = f - nf + 1;
    st.num_factors = nf;
    st.k_in = width[r];
    st.k_out = width[r - nf];
    if (ch.var) {
        const Variant* var = ch.var;
        int64_t pg = 1;
        for (int i = f - nf + 1; i <= f; ++i) pg *= pr.P[i];
        st.kernel = var->kernel;
        st.variant = (int)(var - table);
        st.tile_slices = ch.tile_slices;
        st.block = var->threads;
        st.tile_rows = ch.tile_rows;
        st.lds_bytes = launch_lds_bytes(*var, ch.tile_slices * ch.tile_rows);
        if (ch.tile_rows > 1) {                           // whole rows: the output rows are collected in LDS too
            const int64_t out_bytes = ((int64_t)ch.tile_rows * st.k_out * (int64_t)pr.esize + 15) / 16 * 16;
            if (out_bytes > st.lds_bytes) st.lds_bytes = (int)out_bytes;
        }
        st.grid = ch.grid;
        if (var->persistent) {
            const int hint = ch.tiles_per_wg > 0 ? ch.tiles_per_wg : opt.tiles_per_wg;
            int64_t tpw = tiles_per_wg(st.grid, hint, (int64_t)nf * var->P * var->Q,
                                       (int64_t)ch.tile_slices * ch.tile_rows * pg, var->lds_bytes, pr.esize, var->walk);
            if (hint <= 0 && var->walk == -1) {
                // every workgroup resident from the start and each with the same share of the tiles
                // (measured with the autotuner: 256 x 80x80^3 walks of 17 instead of 8 tiles 0.809 -> 0.721 ms,
                // 256 x 112x112^3 49 instead of 32 2.68 -> 2.38, 64 x 144x144^3 27 instead of 32 2.07 -> 1.76)
                const int64_t resident = 256 * resident_per_cu(*var);
                tpw = (st.grid + resident - 1) / resident;
                // ... or up to a third longer walks when that lowers the tiles the busiest compute unit
                // gets (workgroups on it times walk; 16 x 80x80^3 fp64, 1600 tiles: walks of 3 in 534
                // workgroups 0.140 ms, walks of 4 in 400 workgroups 0.122)
                auto busiest = [&](int64_t t) { return (((st.grid + t - 1) / t + 255) / 256) * t; };
                // (by 5 % at least: fewer workgroups per unit cost more than a tile: 256 x 96x96^3 in 1272
                // workgroups of 29 tiles 1.59 ms, in 1024 of 36 1.78)
                const int64_t first = tpw;
                for (int64_t t = first + 1, last = first + (first + 2) / 3; t <= last; ++t)
                    if (busiest(t) * 20 <= busiest(tpw) * 19) tpw = t;
                if (tpw > 4096) tpw = 4096;
                while (tpw > 1 && st.grid / tpw < 256) --tpw;
            } else if (hint <= 0 && var->walk == 0 && tpw > 1 && !var->xcd_order) {
                // The other walking instances, by the same measure (17 x 128x128^3 fp64, 8704 tiles: walks of
                // 16 in 544 workgroups, two or three to a compute unit, 0.626 ms; walks of 17 in 512, two to each)
                auto busiest = [&](int64_t t) { return (((st.grid + t - 1) / t + 255) / 256) * t; };
                const int64_t first = tpw;
                for (int64_t t = first + 1, last = first + (first + 2) / 3; t <= last; ++t)
                    if (busiest(t) * 20 <= busiest(tpw) * 19) tpw = t;
            }
            const int64_t num_tiles = st.grid;
            st.tiles_per_wg = (int)tpw;
            st.grid = (num_tiles + tpw - 1) / tpw;
            st.tile_order = ch.tile_order >= 0 ? ch.tile_order : (opt.tile_order >= 0 ? opt.tile_order : (var->xcd_order ? 3 : 2));
            // output runs shorter than a 128-byte line: neighbouring tiles go to a pair of workgroups
            // that run side by side (order 1), when the tiles split evenly that way
            if (ch.tile_order < 0 && var->persistent == 1 && opt.pair_interleave &&
                (int64_t)ch.tile_slices * (int64_t)pr.esize < 128 && pair_order_fits(num_tiles, tpw))
                st.tile_order = 1;
            if (st.tile_order == 1 && (var->persistent != 1 || !pair_order_fits(num_tiles, tpw))) st.tile_order = 0;
            if (st.tile_order == 3 && !xcd_order_fits(num_tiles, st.grid)) st.tile_order = 2;
        }
    } else if (ch.any_mfma) {
        st.kernel = KM_KERNEL_MFMA_ANY;
        st.variant = -1;
        st.tile_rows = 1;
        st.tile_slices = any_unit_slices(gen, pr.P[f], pr.esize);
        st.block = gen.any_threads;
        st.lds_bytes = any_lds_bytes(gen, pr.P[f], pr.Q[f], pr.esize);
        const int64_t S = st.k_in / pr.P[f];
        const int cols = 16 * any_column_blocks(pr.Q[f]);
        st.grid = ((pr.M * S + st.tile_slices - 1) / st.tile_slices) * ((pr.Q[f] + cols - 1) / cols);
        const int64_t most = ((int64_t)1 << 32) / gen.any_threads - 1;     // the kernel strides over its units
        if (st.grid > most) st.grid = most;
        // two rounds of the workgroups the chip holds at once (three per compute unit, two with five column
        // blocks), each striding over its share of the units: 2-11 % faster than one workgroup per unit
        // (512 x 40x40^3 fp64 0.458 -> 0.409 ms, 512 x 20x20^4 0.729 -> 0.691, 64 x 100x100^3 0.822 -> 0.789)
        const int64_t rounds2 = 2 * 256 * (any_column_blocks(pr.Q[f]) >= 5 ? 2 : 3);
        if (st.grid > rounds2) st.grid = rounds2;
    } else {
        st.kernel = KM_KERNEL_GENERIC;
        st.variant = -1;
        st.tile_rows = 1;
        st.tile_slices = gen.tile_slices;
        st.block = gen.threads;
        st.lds_bytes = gen.lds_bytes;
        const int64_t S = st.k_in / pr.P[f];
        // one workgroup per (tile of slices, group of factor columns); tiles may span rows
        st.grid = ((pr.M * S + gen.tile_slices - 1) / gen.tile_slices) * ((pr.Q[f] + gen.tile_cols - 1) / gen.tile_cols);
        // the generic kernel strides over its work, so its grid can stay below the launch limit
        const int64_t most = ((int64_t)1 << 32) / gen.threads - 1;
        if (st.grid > most) st.grid = most;
    }
    return st;
}

// The run-time-shape MFMA kernel takes single factors whose slices start on 16-byte boundaries
// (P a multiple of 4 floats or 2 doubles) or are at most 256 bytes long.  It pads P and Q to multiples of 16 with zeros, so a factor
// is given to it only while the padded product is at most 3 times the real one (measured against the
// generic kernel, 3 factors each: fp32 20x20 4 % faster at 2.56x padding, 36x36 19 % at 1.78x, 40x40
// 18 %, 52x52 10 %, 100x100 level; fp64 20x20 9 % faster, 36x36 31 %, 34x34 26 %, 84x84 14 %, 50x50 and
// 22x22 level, 30x30 4 % slower).
inline bool any_mfma_fits(const Problem& pr, int f, const Options& opt)
{
    const int P = pr.P[f], Q = pr.Q[f];
    if (!(opt.kernels >> KM_KERNEL_MFMA_ANY & 1)) return false;
    const int cols = 16 * any_column_blocks(Q);
    const double padded = (double)((P + 15) / 16 * 16) * (double)((Q + cols - 1) / cols * cols);
    return padded <= 3.0 * (double)P * (double)Q;
}

inline void row_widths(const Problem& pr, std::vector<int64_t>& width)
{
    // width[r]: row width when factors 0..r-1 are still to be applied (the others already were)
    width.assign(pr.N + 1, 0);
    width[pr.N] = pr.k_in;
    for (int r = pr.N; r >= 1; --r) width[r - 1] = width[r] / pr.P[r - 1] * pr.Q[r - 1];
}

// Completes a plan from its groups: take[r] factors are applied when r remain, with pick[r].
inline km_status finish_plan(const Problem& pr, const Options& opt, const Variant* table,
                             const std::vector<int>& take, const std::vector<Choice>& pick,
                             const std::vector<int64_t>& width,
                             const GenericKernel& gen, Plan& plan)
{
    plan = Plan();
    for (int r = pr.N; r >= 1; r -= take[r]) {
        const int nf = take[r];
        const int f = r - 1;
        km_plan_step st = build_step(pr, opt, table, r, nf, pick[r], width, gen);
        // flops of the iterations this launch covers
        int64_t w = st.k_in;
        for (int i = f; i >= f - nf + 1; --i) {
            plan.flops += 2.0 * (double)pr.M * (double)w * pr.Q[i];
            w = w / pr.P[i] * pr.Q[i];
            plan.bytes += (double)pr.P[i] * pr.Q[i] * pr.esize;
        }
        plan.bytes += (double)pr.M * ((double)st.k_in + (double)st.k_out) * pr.esize;
        plan.steps.push_back(st);
    }
    // Buffers, assigned backwards from Y: the last launch writes Y, the one before it writes WS0,
    // the one before that writes "B", and so on alternately.  B is Y itself when every row written
    // there fits in a row of Y, otherwise the second workspace.
    const int n = (int)plan.steps.size();
    bool b_is_y = true;
    for (int i = n - 3; i >= 0; i -= 2)
        if (plan.steps[i].k_out > pr.k_out) b_is_y = false;
    int64_t w0 = 0, w1 = 0;
    for (int i = n - 1; i >= 0; --i) {
        const int back = n - 1 - i;
        int dst = back == 0 ? KM_BUF_Y : (back % 2 == 1 ? KM_BUF_WS0 : (b_is_y ? KM_BUF_Y : KM_BUF_WS1));
        plan.steps[i].dst = dst;
        if (dst == KM_BUF_WS0 && plan.steps[i].k_out > w0) w0 = plan.steps[i].k_out;
        if (dst == KM_BUF_WS1 && plan.steps[i].k_out > w1) w1 = plan.steps[i].k_out;
        if (i + 1 < n) plan.steps[i + 1].src = dst;
    }
    plan.steps[0].src = KM_BUF_X;
    plan.ws0_bytes = round_up((size_t)(pr.M * w0) * pr.esize, 256);
    plan.ws1_bytes = round_up((size_t)(pr.M * w1) * pr.esize, 256);
    return KM_OK;
}

inline km_status make_plan(const Problem& pr, const Options& opt, const Variant* table, int count,
                           const GenericKernel& gen, Plan& plan)
{
    const int N = pr.N;
    std::vector<int64_t> width;
    row_widths(pr, width);
    // Grouping by dynamic programming over r: best[r] = cheapest way to apply factors 0..r-1.
    std::vector<double> best(N + 1, 0.0);
    std::vector<int> take(N + 1, 1);
    std::vector<Choice> pick(N + 1);
    for (int r = 1; r <= N; ++r) {
        best[r] = -1;
        for (int nf = 1; nf <= r && nf <= opt.max_fuse; ++nf) {
            Choice ch = find_variant(table, count, pr, r - 1, nf, width[r], opt);
            if (nf > 1 && !ch.var) continue;             // only single factors fall back to the kernels without compiled shapes
            if (!ch.var) ch.any_mfma = any_mfma_fits(pr, r - 1, opt);
            const double c = launch_cost(pr, width[r], width[r - nf], ch, pr.P[r - 1]) + best[r - nf];
            if (best[r] < 0 || c <= best[r] * (1 + 1e-9)) { best[r] = c; take[r] = nf; pick[r] = ch; }
        }
    }
    km_status st = finish_plan(pr, opt, table, take, pick, width, gen, plan);
    if (st != KM_OK) return st;

    // Every factor in one launch with the row resident in LDS, whatever the factor shapes, when
    // that is cheaper: plain FMA code run by one workgroup per row, so only where the launches saved
    // outweigh it.  Measured time per row of one workgroup: about 2 us plus 0.4 us per factor of
    // fixed cost, plus 35 ns per multiply-add of each of its 256 threads, or 50 ns with the 1024
    // threads taken when rows are few (fp64: 1.5 times that); rows run side by side as far as LDS
    // and 2048 threads per compute unit allow.
    const bool force_rows = opt.prefer_instance == count + 1;      // tuning aid: whenever it fits
    if ((opt.kernels >> KM_KERNEL_ROWS & 1) && N >= 2 && N <= gen.row_max_factors && N <= opt.max_fuse &&
        (plan.steps.size() > 1 || force_rows)) {
        int64_t maxw = 0;
        double macs = 0;
        for (int r = 0; r <= N; ++r) maxw = width[r] > maxw ? width[r] : maxw;
        for (int r = 1; r <= N; ++r) macs += (double)width[r] * (double)pr.Q[r - 1];
        int64_t fel = 0;
        for (int i = 0; i < N; ++i) fel += (int64_t)pr.P[i] * pr.Q[i];
        // two row buffers (one word in 33 skipped, see row_kernel.hpp) and every factor
        const int64_t lds = (2 * (maxw + (maxw >> 5) + 1) + fel) * (int64_t)pr.esize;
        if (lds <= gen.row_lds_limit) {
            const bool few = pr.M <= gen.row_few_rows;
            const int threads = few ? gen.row_threads_few : gen.row_threads_many;
            int64_t per_cu = 160 * 1024 / (lds < 20 * 1024 ? 20 * 1024 : lds);
            if (per_cu > 2048 / threads) per_cu = 2048 / threads;
            const int64_t side_by_side = 256 * per_cu;
            const double rounds = (double)((pr.M + side_by_side - 1) / side_by_side);
            const double per_mac = (few ? 50e-9 : 35e-9) * (pr.esize == 4 ? 1.0 : 1.5);
            // ... and rows that share a compute unit share its LDS bandwidth: about 60 ps per multiply-add
            // and compute unit, whatever the precision (measured with 7 or 8 rows per unit: 103563 x 6^4
            // 14.9 us per round, 116508 x 24x24^2 fp64 13.6, 37282 x (9x3, 32x100) 13.2)
            const int64_t rows_per_cu = per_cu < (pr.M + 255) / 256 ? per_cu : (pr.M + 255) / 256;
            // (long rows: about 0.1 us per trip of the workgroup through the loops that load and store a
            // row, beyond the first trips, which are part of the fixed cost; it was 0.45 us while the row
            // loader kept no loads in flight: 3355 x (10x5)^4, rows of 10000 floats on 256 threads, took 34 us
            // per round where the multiply-adds account for 16, and takes 15.5 now)
            const double trips = (double)(width[N] + width[0]) / threads;
            const double alone = 2.0e-6 + 0.4e-6 * N + macs / threads * per_mac + (trips > 8 ? (trips - 8) * 0.1e-6 : 0.0);
            const double shared = 2.0e-6 + (double)rows_per_cu * macs * 60e-12;
            const double seconds = rounds * (alone > shared ? alone : shared);
            const double bytes = (double)pr.M * ((double)width[N] + (double)width[0]) * (double)pr.esize;
            double c = seconds * 5e12;
            // and its row loads and stores, a short loop without loads in flight ahead, stream at about
            // 1.1 TB/s over the whole chip at best (13107 x (80x5, 64x2), rows of 20 KB: 0.384 ms, the tiled
            // plan 0.090; 116508 x (16x13, 36x4) fp64 0.628 against 0.228)
            if (c < 4.5 * bytes) c = 4.5 * bytes;
            c += 2.5e7;
            if (c < best[N] || force_rows) {
                km_plan_step one{};
                one.kernel = KM_KERNEL_ROWS;
                one.variant = -1;
                one.first_factor = 0;
                one.num_factors = N;
                one.tile_slices = 1;
                one.tile_rows = 1;
                one.k_in = width[N];
                one.k_out = width[0];
                one.src = KM_BUF_X;
                one.dst = KM_BUF_Y;
                one.grid = pr.M < 65536 ? pr.M : 65536;     // the kernel strides over the rows
                one.block = threads;
                one.lds_bytes = (int)lds;
                plan.steps.assign(1, one);
                plan.ws0_bytes = plan.ws1_bytes = 0;
                plan.bytes = bytes;
                for (int i = 0; i < N; ++i) plan.bytes += (double)pr.P[i] * pr.Q[i] * pr.esize;
            }
        }
    }
    return KM_OK;
}

}  // namespace km
