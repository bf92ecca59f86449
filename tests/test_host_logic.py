"""Host-side logic of the HIP library: exported symbols, planner, index maps, argument checks.
Nothing here launches a kernel, so it runs without a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2401_10187_amd as km
from conftest import ROOT, read_golden


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "kronmatmul.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(kronmatmul\w*)\s*\(", header))
    assert declared == set(km.EXPORTS)
    L = km.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 and a C program that calls a host-only entry
    point links against the shared library and runs."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use.c"
    src.write_text('''
#include <stdio.h>
#include "kronmatmul.h"
int main(void)
{
    int P[3] = {8, 8, 8}, Q[3] = {8, 8, 8}, n = 0;
    km_plan_step steps[8];
    km_status s = kronmatmul_plan(16, 3, P, Q, KM_F32, steps, 8, &n);
    if (s != KM_OK || n != 1 || steps[0].num_factors != 3) return 1;
    if (kronmatmul_store_column(64, 2, 8, 3, 5) != 45) return 2;
    printf("%s\\n", kronmatmul_status_string(KM_EUNSUPPORTED));
    return 0;
}
''')
    exe = tmp_path / "use"
    lib_dir = os.path.dirname(km.LIB_PATH)
    subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src),
                    "-o", str(exe), "-L", lib_dir, "-lkronmatmul", "-Wl,-rpath," + lib_dir], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stderr
    assert "not supported" in out.stdout


def test_status_and_kernel_names():
    assert km.status_string(km.KM_OK) == "ok"
    assert "invalid" in km.status_string(km.KM_EINVAL)
    assert km.kernel_name(km.KM_KERNEL_GENERIC) == "generic"
    assert km.kernel_name(km.KM_KERNEL_FUSED) == "fused"
    assert km.kernel_name(km.KM_KERNEL_MFMA) == "mfma"
    assert km.kernel_name(km.KM_KERNEL_SHUFFLE) == "shuffle"


def test_store_column_matches_fused_store_example():
    g = read_golden("fused_store_example.txt")
    k, p, tk, nf = int(g["k"][0]), int(g["p"][0]), int(g["tile_k"][0]), int(g["n_fused"][0])
    assert k // p == g["slices_row"][0] and tk // p == g["slices_tile"][0]
    assert k // p ** nf == g["fused_slices_row"][0] and tk // p ** nf == g["fused_slices_tile"][0]
    assert km.store_column(k, p ** nf, tk, int(g["block"][0]), int(g["element"][0])) == g["column"][0]


def test_store_column_matches_single_factor_example():
    g = read_golden("fig4_store_index.txt")
    k, p, tk = int(g["k"][0]), int(g["p"][0]), int(g["tile_k"][0])
    s = tk // p
    assert km.store_column(k, p, tk, 0, 0 * s) == g["column0_start"][0]
    assert km.store_column(k, p, tk, 0, 1 * s) == g["column1_start"][0]
    # run lengths inside a fused tile: consecutive local elements stay consecutive for exactly T_K/P^i
    tk, p = int(g["fig6_tile_k"][0]), int(g["fig6_p"][0])
    for i, key in ((1, "fig6_run_after_1"), (2, "fig6_run_after_2")):
        cols = [km.store_column(256, p ** i, tk, 1, c) for c in range(tk)]
        runs = np.split(np.array(cols), np.where(np.diff(cols) != 1)[0] + 1)
        assert {len(r) for r in runs} == {int(g[key][0])}
        assert len(runs) == p ** i


def test_store_column_is_the_composition_of_single_steps():
    """A fused group's store equals applying the single-factor output map once per factor to the
    whole row (a6: local tile index -> global column)."""
    K, P, nf, tile_k = 4 ** 4, 4, 3, 4 ** 3 * 2
    cols = np.arange(K)
    # follow every input column's *slice group* through nf single steps with square factors: after one
    # step the element made from slice s and column q sits at q*(K/P)+s.
    # Enumerate outputs: output digit string (q1..qnf, a) <-> a*P^nf + (p-digits) block of inputs.
    s_t = tile_k // P ** nf
    for tile in range(K // tile_k):
        for c in range(tile_k):
            qq, r = divmod(c, s_t)
            a = tile * s_t + r
            assert km.store_column(K, P ** nf, tile_k, tile, c) == qq * (K // P ** nf) + a
    assert km.store_column(K, P ** nf, tile_k, K // tile_k, 0) == -1
    assert km.store_column(K, 3, tile_k, 0, 0) == -1


@pytest.mark.parametrize("M,shapes,dtype", [
    (16, [(8, 8)] * 3, "float32"),
    (1024, [(8, 8)] * 6, "float32"),
    (1024, [(32, 32)] * 4, "float32"),
    (16, [(128, 128)] * 3, "float64"),
    (256, [(16, 32)] * 4, "float32"),
    (7, [(3, 5), (4, 2), (6, 6), (2, 3)], "float64"),
    (3, [(5, 2), (5, 2), (5, 2)], "float32"),
])
def test_plan_is_consistent(M, shapes, dtype):
    P = [s[0] for s in shapes]
    Q = [s[1] for s in shapes]
    steps = km.plan(M, P, Q, dtype)
    es = 4 if dtype == "float32" else 8
    # factors are consumed last to first, each exactly once
    f = len(shapes)
    k = int(np.prod(P, dtype=np.int64))
    widths = {km.KM_BUF_WS0: 0, km.KM_BUF_WS1: 0}
    for i, st in enumerate(steps):
        assert st["first_factor"] + st["num_factors"] == f
        f = st["first_factor"]
        assert st["k_in"] == k
        for j in range(st["num_factors"]):
            k = k // P[f + st["num_factors"] - 1 - j] * Q[f + st["num_factors"] - 1 - j]
        assert st["k_out"] == k
        assert st["src"] == (km.KM_BUF_X if i == 0 else steps[i - 1]["dst"])
        assert st["dst"] != st["src"] and st["dst"] != km.KM_BUF_X
        if st["dst"] == km.KM_BUF_Y:
            assert st["k_out"] <= int(np.prod(Q, dtype=np.int64))
        else:
            widths[st["dst"]] = max(widths[st["dst"]], st["k_out"])
        assert st["grid"] > 0 and st["block"] > 0
        assert st["lds_bytes"] <= 160 * 1024
        # walking workgroups cover every tile: grid = ceil(tiles / tiles_per_wg)
        assert st["tile_order"] in (0, 1, 2, 3) and st["tiles_per_wg"] >= 0
        if st["tiles_per_wg"] > 0:
            pg = int(np.prod(P[st["first_factor"]:st["first_factor"] + st["num_factors"]], dtype=np.int64))
            tiles = M * (st["k_in"] // (st["tile_slices"] * pg))
            assert st["grid"] == -(-tiles // st["tiles_per_wg"])
            if st["tile_order"] == 1:
                assert st["grid"] % 16 == 0 and tiles % (2 * st["tiles_per_wg"]) == 0
    assert f == 0
    assert steps[-1]["dst"] == km.KM_BUF_Y
    need = sum((M * w * es + 255) // 256 * 256 for w in widths.values())
    assert km.workspace_size(M, P, Q, dtype) == need
    # flops: 2 * M * sum_f K_f * Q_f (section 3, counted as multiply-add = 2)
    flops, nbytes = km.cost(M, P, Q, dtype)
    kk, want = int(np.prod(P, dtype=np.int64)), 0
    for p, q in reversed(shapes):
        want += 2 * M * kk * q
        kk = kk // p * q
    assert flops == want
    assert nbytes >= es * M * (steps[0]["k_in"] + steps[-1]["k_out"])


def test_workspace_follows_algorithm_1_buffers():
    """Two swapped intermediates of M x max-width (the pair Algorithm 1 declares) are an upper bound."""
    M, P, Q = 5, [4, 2, 3, 2], [2, 6, 3, 5]
    ws = km.workspace_size(M, P, Q, "float64")
    k, widest = int(np.prod(P)), 0
    for p, q in reversed(list(zip(P, Q))):
        k = k // p * q
        widest = max(widest, k)
    assert ws <= 2 * ((M * widest * 8 + 255) // 256 * 256)
    assert km.workspace_size(M, [4], [7], "float32") == 0


def test_tuning_options_round_trip():
    for opt, good, bad in ((km.KM_OPT_PREFER_TILE, 16, -1), (km.KM_OPT_PREFER_THREADS, 256, 5000),
                           (km.KM_OPT_TILES_PER_WG, 8, -2), (km.KM_OPT_PAIR_INTERLEAVE, 0, 2),
                           (km.KM_OPT_PROFILE, 1, 3), (km.KM_OPT_KEEP_MIB, 0, -1)):
        old = km.get_option(opt)
        try:
            km.set_option(opt, good)
            assert km.get_option(opt) == good
            with pytest.raises(km.KronMatmulError):
                km.set_option(opt, bad)
            assert km.get_option(opt) == good
        finally:
            km.set_option(opt, old)


def test_padded_shapes_go_to_the_run_time_shape_mfma_kernel_within_its_padding_limits():
    """A padded product of at most 3x the real one, whatever the alignment of the slices; everything else
    without a compiled instance stays with the generic kernel.  The narrow shape (slices of up to 128
    bytes) takes 256 slices per unit, the wide one 128."""
    def kernels(dtype, M, shapes):
        return [(s["kernel"], s["tile_slices"]) for s in km.plan(M, [p for p, _ in shapes], [q for _, q in shapes], dtype)]
    any_, gen = km.KM_KERNEL_MFMA_ANY, km.KM_KERNEL_GENERIC
    assert kernels("float32", 4096, [(20, 20)] * 3) == [(any_, 256)] * 3          # 32*32 / 400 = 2.56
    assert kernels("float32", 4096, [(36, 50)] * 3) == [(any_, 128)] * 3
    assert kernels("float32", 4096, [(20, 15)] * 3) == [(any_, 256)] * 3          # Q need not be a whole vector
    assert [k for k, _ in kernels("float32", 4096, [(20, 7)] * 4)] == [gen] * 4    # 32*16 / 140 = 3.7
    assert kernels("float32", 4096, [(22, 22)] * 4) == [(any_, 256)] * 4          # slices not 16-byte aligned, but one chunk
    assert kernels("float32", 1024, [(66, 66)] * 3) == [(any_, 128)] * 3          # ... or longer than a chunk (264 bytes)
    assert kernels("float64", 4096, [(16, 20)] * 4) == [(any_, 256)] * 4          # 16*32 / 320 = 1.6, 128-byte slices
    assert kernels("float64", 4096, [(26, 26)] * 3) == [(any_, 128)] * 3          # 32*32 / 676 = 1.5
    assert kernels("float64", 4096, [(40, 40)] * 3) == [(any_, 128)] * 3          # 48*48 / 1600 = 1.44
    assert kernels("float64", 4096, [(20, 20)] * 3) == [(any_, 128)] * 3          # 32*32 / 400 = 2.56
    assert [k for k, _ in kernels("float64", 4096, [(6, 50)] * 3)] == [gen] * 3    # 16*64 / 300 = 3.4
    assert kernels("float64", 4096, [(15, 16)] * 4) == [(any_, 256)] * 4          # odd P, 120-byte slices
    assert kernels("float64", 4096, [(33, 33)] * 3) == [(any_, 128)] * 3          # odd P, 264-byte slices


def test_neighbouring_runs_of_different_small_shapes_are_one_launch_where_an_instance_is_compiled():
    """The small-factor kernel has a factor shape per stage; the planner matches a group's shapes against
    the stages in order of application (the group's last factors first)."""
    def steps(M, shapes, dtype="float32"):
        return [(s["kernel"], s["num_factors"]) for s in km.plan(M, [p for p, _ in shapes], [q for _, q in shapes], dtype)]
    fused = km.KM_KERNEL_FUSED
    assert steps(1024, [(4, 4)] * 5 + [(2, 2)] * 4) == [(fused, 9)]
    assert steps(1024, [(4, 4)] * 4 + [(2, 2)] * 4, "float64") == [(fused, 8)]
    assert steps(4096, [(5, 5)] * 2 + [(2, 2)]) == [(fused, 3)]
    assert steps(4096, [(2, 2)] + [(5, 5)] * 2) == [(fused, 3)]
    assert steps(1024, [(8, 8)] * 2 + [(4, 4)] * 2) == [(fused, 4)]
    # no instance for this order of the same factors: one launch per run of equal shapes
    assert steps(1024, [(2, 2)] * 4 + [(4, 4)] * 5) == [(fused, 5), (fused, 4)]
    # a run-time check on the launch side too: the plan of one shape sequence is refused for another
    assert len(steps(1024, [(4, 4)] * 5 + [(2, 2)] * 3 + [(3, 3)])) > 1


def test_square_mfma_instances_between_the_powers_of_two_walk_one_round_of_resident_workgroups():
    """80, 112 and 144 (and 96 in fp64): the grid is the number of workgroups the chip holds at once
    (three of 640 threads, four of 448, three of 576, three with 49 KB of LDS each per compute unit), each walking its share."""
    for P, M, dtype, per_cu in ((80, 256, "float32", 3), (112, 256, "float32", 4), (144, 64, "float32", 3),
                                (96, 64, "float64", 3)):
        plan = km.plan(M, [P] * 3, [P] * 3, dtype)
        assert [s["kernel"] for s in plan] == [km.KM_KERNEL_MFMA] * 3
        for s in plan:
            tiles = M * (P * P * P // P // s["tile_slices"])
            assert s["grid"] == -(-tiles // s["tiles_per_wg"])
            assert 256 * per_cu * 0.9 <= s["grid"] <= 256 * per_cu, (P, s["grid"], s["tiles_per_wg"])


def test_planner_prefers_fusion_and_mfma_for_the_measured_workloads():
    import kron_inputs
    want = {"c1_f32_m16_8x8x3": [(km.KM_KERNEL_FUSED, 3)],
            "c2_f32_m1024_8x8x6": [(km.KM_KERNEL_FUSED, 3)] * 2,
            "c3_f32_m1024_32x32x4": [(km.KM_KERNEL_MFMA, 2)] * 2,
            "c4_f64_m16_128x128x3": [(km.KM_KERNEL_MFMA, 1)] * 3,
            "c5_f32_m256_16x32x4": [(km.KM_KERNEL_MFMA, 2)] * 2}
    for name, steps in want.items():
        c = kron_inputs.CONFIGS[name]
        got = km.plan(c["M"], [s[0] for s in c["shapes"]], [s[1] for s in c["shapes"]], c["dtype"])
        assert [(st["kernel"], st["num_factors"]) for st in got] == steps, name
        # 128-byte output runs wherever the row is long enough
        if name != "c1_f32_m16_8x8x3":
            es = 4 if c["dtype"] == "float32" else 8
            assert all(st["tile_slices"] * es >= 128 for st in got), name


def test_walk_lengths_follow_the_measured_rule():
    """Large factors: long walks (factor loads amortised); small factors: one tile per workgroup;
    the grid keeps at least two workgroups per compute unit."""
    big = km.plan(1024, [64] * 3, [64] * 3, "float32")
    assert all(st["tiles_per_wg"] == 32 for st in big)
    small = km.plan(1024, [16] * 5, [16] * 5, "float32")
    assert all(st["tiles_per_wg"] == 1 for st in small)
    few = km.plan(16, [128] * 3, [128] * 3, "float64")
    assert all(st["grid"] >= 512 for st in few)


def test_tile_lengths_for_small_problems_and_odd_rows():
    """Small problems keep several threads of a workgroup busy instead of cutting one-slice tiles to
    reach more workgroups; rows of odd length take tiles whose output runs reach 64 bytes; long
    rows that do not start on 16-byte boundaries are not joined into tiles of several rows."""
    old = km.get_option(km.KM_OPT_KERNELS)
    try:
        km.set_option(km.KM_OPT_KERNELS, 7)              # the tiled families, not the whole-row kernel
        for M, P, n, dtype in ((20, 5, 8, "float32"), (50, 5, 7, "float32"), (100, 5, 7, "float64")):      # 25 or 125 elements per thread
            steps = km.plan(M, [P] * n, [P] * n, dtype)
            assert all(st["tile_slices"] * st["tile_rows"] >= 4 for st in steps if st["num_factors"] >= 2), (M, P, n, steps)
            assert all(st["grid"] >= 96 for st in steps), (M, P, n, steps)
        # ... unless the whole row fits one tile: one launch, one workgroup per row (20 x 5^6: 0.013 ms, two launches 0.016)
        for M, P, n, dtype in ((20, 5, 6, "float32"), (100, 5, 5, "float64")):
            steps = km.plan(M, [P] * n, [P] * n, dtype)
            assert len(steps) == 1 and steps[0]["grid"] == M, (M, P, n, steps)
    finally:
        km.set_option(km.KM_OPT_KERNELS, old)
    first = km.plan(1024, [5] * 8, [5] * 8, "float32")[0]
    assert first["num_factors"] == 4 and first["tile_slices"] == 25       # 100-byte runs, 62 KB tiles, two launches of four factors
    first = km.plan(1024, [5] * 7, [5] * 7, "float64")[0]
    assert first["num_factors"] == 3 and first["tile_slices"] == 25       # 200-byte runs, 25 KB tiles
    assert all(st["tile_rows"] == 1 for st in km.plan(1024, [3] * 7, [3] * 7, "float32"))
    assert all(st["tile_rows"] == 1 for st in km.plan(1526, [4] * 6, [4] * 6, "float32"))   # 16 KB rows: fp32 tiles hold 24 KB
    assert all(24 < st["tile_rows"] * 8 <= 48 for st in km.plan(4096, [4] * 5, [4] * 5, "float64"))   # ... fp64 tiles 48 KB (rows of 8 KB)
    assert all(st["tile_rows"] == 4 for st in km.plan(4096, [4] * 5, [4] * 5, "float32"))
    assert km.plan(1 << 20, [4] * 4, [4] * 4, "float32")[0]["tile_rows"] > 8


def test_generic_launches_cover_slices_times_column_groups():
    """The generic kernel's units of work are 128 slices by 32 factor columns."""
    st = km.plan(300, [5], [40], "float32")[0]
    assert st["kernel"] == km.KM_KERNEL_GENERIC
    assert st["grid"] == -(-300 // 128) * -(-40 // 32)
    old = km.get_option(km.KM_OPT_KERNELS)
    try:
        km.set_option(km.KM_OPT_KERNELS, 1)              # generic kernel only
        st = km.plan(50, [64], [128], "float32")[0]
    finally:
        km.set_option(km.KM_OPT_KERNELS, old)
    assert st["kernel"] == km.KM_KERNEL_GENERIC and st["grid"] == -(-50 // 128) * (128 // 32)


def test_host_entry_points_are_thread_safe():
    """Planning from several threads at once (the plan cache and the options are shared state) gives
    what planning serially gives."""
    import threading
    rng = np.random.default_rng(5)
    problems = []
    for _ in range(40):
        p = int(rng.choice([2, 3, 4, 5, 6, 8, 16, 32, 64, 7]))
        n = int(rng.integers(1, 7))
        while p ** n > 2 ** 24:                      # keep to sizes a device could hold
            n -= 1
        problems.append((int(rng.integers(1, 2000)), [p] * n, [p] * n, "float32" if rng.random() < 0.5 else "float64"))
    serial = [(km.plan(*pr), km.workspace_size(*pr), km.cost(*pr)) for pr in problems]
    results, errors = {}, []

    def work(t):
        try:
            for rep in range(5):
                for i in range(t, len(problems), 4):
                    results[(t, rep, i)] = (km.plan(*problems[i]), km.workspace_size(*problems[i]), km.cost(*problems[i]))
        except Exception as e:          # noqa: BLE001 - reported below
            errors.append(e)

    threads = [threading.Thread(target=work, args=(t,)) for t in range(4)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors
    assert all(v == serial[i] for (_, _, i), v in results.items())


def test_launches_stay_below_the_work_item_limit():
    """A launch may hold fewer than 2^32 work-items: instances whose grid would exceed that are not
    chosen; the generic kernel strides over its tiles with a capped grid, so size alone never makes a
    problem unsupported."""
    for M, P, n in [(1 << 20, 4, 4), (1 << 24, 8, 3), (1 << 22, 2, 6), (1 << 24, 2, 8), (1 << 26, 7, 2)]:
        for st in km.plan(M, [P] * n, [P] * n, "float32"):
            assert 0 < st["grid"] * st["block"] < 2 ** 32


def test_tile_instances_are_skipped_for_rows_beyond_32_bit_offsets():
    # 2^31 bytes per row and more: only the generic kernel addresses such rows
    steps = km.plan(1, [8] * 10, [8] * 10, "float32")
    assert all(st["kernel"] == km.KM_KERNEL_GENERIC for st in steps)


def test_options_round_trip():
    old = km.get_option(km.KM_OPT_MAX_FUSE)
    try:
        km.set_option(km.KM_OPT_MAX_FUSE, 1)
        assert km.get_option(km.KM_OPT_MAX_FUSE) == 1
        assert all(st["num_factors"] == 1 for st in km.plan(16, [8] * 3, [8] * 3, "float32"))
        with pytest.raises(km.KronMatmulError):
            km.set_option(km.KM_OPT_MAX_FUSE, 0)
        with pytest.raises(km.KronMatmulError):
            km.set_option(99, 0)
    finally:
        km.set_option(km.KM_OPT_MAX_FUSE, old)
    old = km.get_option(km.KM_OPT_KERNELS)
    try:
        km.set_option(km.KM_OPT_KERNELS, 0)
        assert km.get_option(km.KM_OPT_KERNELS) & 1
        assert all(st["kernel"] == km.KM_KERNEL_GENERIC for st in km.plan(1024, [8] * 6, [8] * 6, "float32"))
    finally:
        km.set_option(km.KM_OPT_KERNELS, old)


def _raw(M, P, Q, X, F, Y, dtype=0, with_ws=False):
    L = km.lib()
    n = len(P)
    p = (ctypes.c_int * max(n, 1))(*P)
    q = (ctypes.c_int * max(n, 1))(*Q)
    f = None if F is None else ctypes.cast((ctypes.c_void_p * max(n, 1))(*F), ctypes.c_void_p)
    if with_ws:
        return L.kronmatmul_ws(M, n, p, q, X, f, Y, dtype, None, 0, None)
    return L.kronmatmul(M, n, p, q, X, f, Y, dtype, None)


def test_argument_errors_are_status_codes():
    """Validation happens before any HIP call, so these never touch a device."""
    bad = 0x1000   # never dereferenced: the calls below must fail before any launch
    assert _raw(-1, [2], [2], bad, [bad], bad) == km.KM_EINVAL
    assert _raw(4, [], [], bad, [], bad) == km.KM_EINVAL
    assert _raw(4, [0], [2], bad, [bad], bad) == km.KM_EINVAL
    assert _raw(4, [2], [-3], bad, [bad], bad) == km.KM_EINVAL
    assert _raw(4, [2], [2], None, [bad], bad) == km.KM_EINVAL
    assert _raw(4, [2], [2], bad, [bad], None) == km.KM_EINVAL
    assert _raw(4, [2], [2], bad, [None], bad) == km.KM_EINVAL
    assert _raw(4, [2], [2], bad, None, bad) == km.KM_EINVAL
    assert _raw(4, [2], [2], bad, [bad], bad, dtype=7) == km.KM_EINVAL
    assert _raw(4, [2 ** 20] * 3, [2] * 3, bad, [bad] * 3, bad) == km.KM_EINVAL      # width overflow
    assert _raw(2 ** 31 - 1, [2 ** 15] * 2, [2 ** 15] * 2, bad, [bad] * 2, bad) == km.KM_EINVAL
    assert _raw(4, [2], [2], bad + 4, [bad], bad) == km.KM_EINVAL            # X not 16-byte aligned
    assert _raw(4, [2], [2], bad, [bad], bad + 8) == km.KM_EINVAL            # Y not 16-byte aligned
    assert _raw(4, [2], [2], bad, [bad + 2], bad) == km.KM_EINVAL            # factor not element aligned
    # M == 0 is a successful no-op, with or without buffers
    assert _raw(0, [2, 3], [2, 3], None, [bad, bad], None) == km.KM_OK
    assert _raw(0, [2, 3], [2, 3], None, [bad, bad], None, with_ws=True) == km.KM_OK
    # a workspace that is too small is refused before any launch
    # (two factors of different shapes, rows too long for the one-launch kernel: two launches, hence an intermediate)
    assert km.workspace_size(4, [70, 110], [30, 50], "float32") > 0
    assert _raw(4, [70, 110], [30, 50], bad, [bad, bad], bad + (1 << 30), with_ws=True) == km.KM_ENOMEM


def test_overlapping_buffers_are_refused():
    """X, Y and the workspace must be apart: checked on the host, before any launch."""
    L = km.lib()
    base = 0x10000000
    P, Q = [70, 110], [30, 50]                       # two launches, hence an intermediate in the workspace
    n = len(P)
    p, q = (ctypes.c_int * n)(*P), (ctypes.c_int * n)(*Q)
    f = ctypes.cast((ctypes.c_void_p * n)(0x1000, 0x2000), ctypes.c_void_p)
    x_bytes, y_bytes = 4 * 7700 * 4, 4 * 1500 * 4
    need = km.workspace_size(4, P, Q, "float32")
    far = base + (1 << 30)
    call = lambda X, Y, ws: L.kronmatmul_ws(4, n, p, q, X, f, Y, 0, ws, need, None)
    assert call(base, base, far) == km.KM_EINVAL                              # Y is X
    assert call(base, base + x_bytes - 16, far) == km.KM_EINVAL               # Y starts inside X
    assert call(base + y_bytes - 16, base, far) == km.KM_EINVAL               # X starts inside Y
    assert call(base, far, base + x_bytes - 256) == km.KM_EINVAL              # workspace reaches into X ... from inside
    assert call(base + need - 16, far, base) == km.KM_EINVAL                  # ... from below
    assert call(base, far, far + y_bytes - 16) == km.KM_EINVAL                # workspace starts inside Y
    # the library-managed form checks X against Y too
    assert L.kronmatmul(4, n, p, q, base, f, base + 64, 0, None) == km.KM_EINVAL


def test_static_entry_point_refuses_what_does_not_fit():
    """kronmatmul_static takes its workspace from an array of KM_STATIC_SCRATCH_BYTES: a problem whose
    intermediates need more (1024 x 8^6: 1 GiB) is refused with KM_ENOMEM before anything touches a device;
    its other argument checks are those of kronmatmul_ws."""
    L = km.lib()
    base, n = 0x10000000, 6
    p = (ctypes.c_int * n)(*[8] * n)
    f = ctypes.cast((ctypes.c_void_p * n)(*[0x1000] * n), ctypes.c_void_p)
    assert km.workspace_size(1024, [8] * n, [8] * n, "float32") > km.KM_STATIC_SCRATCH_BYTES
    assert L.kronmatmul_static(1024, n, p, p, base, f, base + (1 << 40), km.KM_F32, None) == km.KM_ENOMEM
    assert L.kronmatmul_static(1024, n, p, p, base, f, base, km.KM_F32, None) == km.KM_EINVAL          # Y is X
    assert L.kronmatmul_static(1024, n, p, p, None, f, base, km.KM_F32, None) == km.KM_EINVAL
    assert L.kronmatmul_static(0, n, p, p, None, f, None, km.KM_F32, None) == km.KM_OK


def test_empty_problems_plan_to_nothing():
    """M == 0 is a successful no-op for every entry point, the planning ones included."""
    assert km.plan(0, [8, 8], [8, 8], "float32") == []
    assert km.cost(0, [8, 8], [8, 8], "float64") == (0.0, 0.0)
    assert km.workspace_size(0, [70, 110], [30, 50], "float32") == 0
    km.prepare(0, [8, 8], [8, 8], "float32")
    with pytest.raises(km.KronMatmulError):
        km.prepare(4, [0], [8], "float32")


def test_unaligned_tiles_are_moved_without_leaving_the_buffer(tmp_path):
    """Rows of odd length (3^7 fp32 and the like) start off 16-byte boundaries; their tiles are moved in
    16-byte vectors counted from the boundary below.  The two counts the kernels take from plan.hpp
    must cover the run exactly, with every whole vector inside [-mis, valid): checked for every
    (run length, misalignment, vector width) by a host program that includes that header."""
    src = tmp_path / "span.cpp"
    src.write_text(r"""
#include "paper_2401_10187_amd/csrc/plan.hpp"
#include <stdio.h>
int main() {
    for (int vn = 2; vn <= 4; vn += 2)
        for (int mis = 0; mis < vn; ++mis)
            for (int valid = 1; valid <= 3 * 3 * 3 * 3 * 3 * 3 * 3 + 5; ++valid) {
                const int nv = km::unaligned_vectors(valid, mis, vn), nfull = km::unaligned_whole_vectors(valid, mis, vn);
                if (nfull > nv || nv - nfull > 1) return 1;
                if (nv * vn - mis < valid) return 2;                      // the vectors cover the run
                if ((nv - 1) * vn - mis >= valid) return 3;               // and none lies wholly outside it
                for (int v = 0; v < nfull; ++v)                           // whole vectors stay inside [-mis, valid)
                    if (v * vn - mis < -mis || (v + 1) * vn - mis > valid) return 4;
                if (nfull < nv && nfull * vn - mis + vn <= valid) return 5;   // the partial one really is partial
            }
    puts("ok");
    return 0;
}
""")
    exe = tmp_path / "span"
    import subprocess
    subprocess.run(["g++", "-std=c++17", "-I", ROOT, "-o", str(exe), str(src)], check=True)
    assert subprocess.run([str(exe)], capture_output=True, text=True).stdout.strip() == "ok"


def test_clock_probe_argument_errors():
    """The probe checks its arguments before launching anything."""
    probe = km.lib().kronmatmul_clock_probe
    bad = 0x1000
    assert probe(None, 100, None) == km.KM_EINVAL
    assert probe(ctypes.c_void_p(bad + 4), 100, None) == km.KM_EINVAL        # not 8-byte aligned
    assert probe(ctypes.c_void_p(bad), 0, None) == km.KM_EINVAL
    assert probe(ctypes.c_void_p(bad), 1000001, None) == km.KM_EINVAL


def test_transposed_form_needs_room_for_the_factor_copies():
    """The transposed-factor entry points copy the factors behind the plan's workspace: each copy on a
    256-byte boundary.  Their argument checks are those of the plain form."""
    for M, P, Q, dtype, es in [(4, [7, 11], [3, 5], "float32", 4), (16, [8] * 3, [8] * 3, "float32", 4),
                               (2, [128] * 2, [128] * 2, "float64", 8)]:
        plain = km.workspace_size(M, P, Q, dtype)
        copies = sum((p * q * es + 255) // 256 * 256 for p, q in zip(P, Q))
        assert km.workspace_size(M, P, Q, dtype, transposed=True) == (plain + 255) // 256 * 256 + copies
    assert km.workspace_size(0, [8], [8], "float32", transposed=True) == 0
    L = km.lib()
    bad = 0x1000
    p, q = (ctypes.c_int * 1)(2), (ctypes.c_int * 1)(2)
    f = ctypes.cast((ctypes.c_void_p * 1)(bad), ctypes.c_void_p)
    assert L.kronmatmul_transposed(4, 1, p, q, None, f, bad, 0, None) == km.KM_EINVAL
    assert L.kronmatmul_transposed(-1, 1, p, q, bad, f, bad, 0, None) == km.KM_EINVAL
    assert L.kronmatmul_transposed_ws(4, 1, p, q, bad, f, bad + 4096, 0, None, 0, None) == km.KM_ENOMEM   # copies need room
    assert L.kronmatmul_transposed_ws(0, 1, p, q, None, f, None, 0, None, 0, None) == km.KM_OK


def test_workspace_size_errors():
    L = km.lib()
    p = (ctypes.c_int * 1)(2)
    assert L.kronmatmul_workspace_size(1, 1, p, p, 0, None) == km.KM_EINVAL
    out = ctypes.c_size_t(123)
    assert L.kronmatmul_workspace_size(1, 0, p, p, 0, ctypes.byref(out)) == km.KM_EINVAL
    assert L.kronmatmul_workspace_size(0, 1, p, p, 1, ctypes.byref(out)) == km.KM_OK and out.value == 0


def test_last_profile_without_a_call_is_an_error_or_needs_device():
    L = km.lib()
    cnt = ctypes.c_int(0)
    assert L.kronmatmul_last_profile(None, 0, None) == km.KM_EINVAL


def test_missing_library_is_a_loud_error(monkeypatch):
    """There is no CPU fallback: without the built HIP library the binding refuses to work."""
    import paper_2401_10187_amd.binding as B
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", os.path.join(ROOT, "paper_2401_10187_amd", "no_such_library.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.lib()
    with pytest.raises(RuntimeError):
        B.plan(4, [2], [2], "float32")


def test_oracle_and_product_do_not_import_each_other():
    """The oracle is test infrastructure: the package never imports it, and it never imports the
    package; only the input generators are shared, and they hold none of the method's arithmetic."""
    def sources(folder, exts):
        for base, _, files in os.walk(os.path.join(ROOT, folder)):
            for f in files:
                if f.endswith(exts):
                    yield os.path.join(base, f)
    for path in sources("paper_2401_10187_amd", (".py", ".hip", ".hpp", ".h")):
        text = open(path).read()
        assert "oracle" not in text.lower(), path
    for path in sources("oracle", (".py", ".c", ".h")):
        text = open(path).read()
        assert "paper_2401_10187_amd" not in text and "kronmatmul.h" not in text, path
        assert "#include <hip" not in text and "libkronmatmul" not in text and "import torch" not in text, path
    gen = open(os.path.join(ROOT, "kron_inputs.py")).read()
    assert "import oracle" not in gen and "paper_2401_10187_amd" not in gen
    for needle in ("kron_matmul(", "sliced_multiply(", " @ ", "np.kron", "matmul"):
        assert needle not in gen


def test_unit_numbering_is_a_bijection_that_keeps_a_tile_on_one_xcd(tmp_path):
    """The kernels without compiled shapes number their units (slice tile, column group) so that the
    groups of a tile run on the same XCD (workgroup b runs on XCD b % 8): every unit must occur exactly
    once, and inside the whole runs of 8 tiles all groups of a tile must share b % 8."""
    src = tmp_path / "units.cpp"
    src.write_text(r"""
#include "paper_2401_10187_amd/csrc/plan.hpp"
#include <stdio.h>
#include <vector>
int main() {
    for (int64_t tiles = 1; tiles <= 70; ++tiles)
        for (int groups = 1; groups <= 9; ++groups) {
            std::vector<int> seen(tiles * groups, 0), xcd(tiles, -1);
            for (int64_t b = 0; b < tiles * groups; ++b) {
                int64_t t; int c;
                km::unit_of(b, tiles, groups, t, c);
                if (t < 0 || t >= tiles || c < 0 || c >= groups) return 1;
                if (seen[t * groups + c]++) return 2;
                if (t < tiles / 8 * 8) {
                    if (xcd[t] >= 0 && xcd[t] != b % 8) return 3;
                    xcd[t] = (int)(b % 8);
                }
            }
        }
    puts("ok");
    return 0;
}
""")
    exe = tmp_path / "units"
    import subprocess
    subprocess.run(["g++", "-std=c++17", "-I", ROOT, "-o", str(exe), str(src)], check=True)
    assert subprocess.run([str(exe)], capture_output=True, text=True).stdout.strip() == "ok"
