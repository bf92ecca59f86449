#!/usr/bin/env python3
"""Benchmark of the Kron-Matmul hot path on one MI355X.

A step is one whole Kron-Matmul Y = X (F_1 (x) ... (x) F_N) through the C-ABI library (all planned
launches) on a synthetic workload that already sits in HBM.  Prints ONE JSON line:
whole-job GFLOP/s (flops = 2*M*sum_f K_f*Q_f, one multiply-add = 2), the roofline of the dominant
kernel from HIP-event durations taken inside the timed region, and the CPU oracle timed on the host.
The line is about the headline workload (--workload); unless --only-headline is given, the other
measured workloads are run the same way in the same process and reported, in short, under
config.other_workloads.
"""
import argparse
import glob
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
PEAKS_TFLOPS = {"float32": 157.3, "float64": 78.6}   # dense MFMA / vector peaks, published

# The paper's own time for the same shape on one V100 (Table 1), as GFLOP/s with the same flop count.
# Other hardware: reported as context under config.paper_context, never as vs_baseline.
PAPER_GFLOPS = {"c2_f32_m1024_8x8x6": 25769803776 / 5.76e-3 / 1e9,
                "c3_f32_m1024_32x32x4": 274877906944 / 38.8e-3 / 1e9}

HEADLINE = "c2_f32_m1024_8x8x6"
OTHERS = ["c1_f32_m16_8x8x3", "c3_f32_m1024_32x32x4", "c4_f64_m16_128x128x3", "c5_f32_m256_16x32x4"]

SETTLE_TOLERANCE = 0.01          # two consecutive batches of `steps` steps must agree this closely ...
SETTLE_MAX_BATCHES = 40          # ... within this many batches
SETTLE_MAX_MS = 2000.0           # ... and this much GPU time


def profile_traffic(workload):
    """HBM bytes per launch of the workload's dominant kernel as measured with rocprofv3 --pmc
    (FETCH_SIZE and WRITE_SIZE, each scaled by a copy kernel of known size): read from the summary
    under profiles/ whose header names the workload.  (value or None, file name or None)."""
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        head = open(path).read(4000)
        m = re.search(r"^workload: (\S+)$", head, re.M)
        if not m or m.group(1) != workload:
            continue
        t = re.search(r"^hbm_traffic_bytes_per_launch: (\d+)$", head, re.M)
        return (int(t.group(1)) if t else None), os.path.relpath(path, ROOT)
    return None, None


def parse_shape(text):
    """M:PxQ^N[,PxQ^N...]:f32|f64 -> (M, [(P, Q), ...], dtype name)."""
    m_s, f_s, d_s = text.split(":")
    shapes = []
    for part in f_s.split(","):
        pq, _, n = part.partition("^")
        p_, q_ = pq.split("x")
        shapes += [(int(p_), int(q_))] * int(n or 1)
    return int(m_s), shapes, {"f32": "float32", "f64": "float64"}[d_s]


def make_workload(name, seed):
    """(dtype name, X, factor list) of a named workload, a Table 4 size or an ad-hoc shape."""
    import kron_inputs
    if name.startswith("shape_"):
        M, shapes, dtype = parse_shape(name[len("shape_"):])
        return (dtype,) + kron_inputs.make_problem(M, shapes, dtype, "uniform", "uniform", seed)
    if name.startswith("table4_id"):
        # table4_id<k>[_f64]: problem size k of the paper's Table 4 with synthetic values
        parts = name.split("_")
        case = {c[0]: c for c in kron_inputs.TABLE4}[int(parts[1][2:])]
        dtype = "float64" if parts[-1] == "f64" else "float32"
        return (dtype,) + kron_inputs.make_problem(case[1], case[2], dtype, "uniform", "uniform", seed)
    return (kron_inputs.CONFIGS[name]["dtype"],) + kron_inputs.make_config(name, seed=seed)


def shape_runs(P, Q):
    """Factor shapes as runs of equal ones: "3x(8x8)", "5x(4x4)+4x(2x2)"."""
    runs = []
    for pq in zip(P, Q):
        if runs and runs[-1][0] == pq:
            runs[-1][1] += 1
        else:
            runs.append([pq, 1])
    return "+".join("%dx(%dx%d)" % (n, p, q) for (p, q), n in runs)


def measure(name, args, headline):
    """Runs one workload: warm-up, settling, the timed steps, per-launch durations, the clock probe,
    and the comparison with the CPU oracle.  Returns the full result dictionary."""
    import numpy as np
    import torch
    import paper_2401_10187_amd as km

    dtype, X, Fs = make_workload(name, args.seed)
    M = X.shape[0]
    P = [F.shape[0] for F in Fs]
    Q = [F.shape[1] for F in Fs]
    dev = torch.device("cuda:0")
    Xd = torch.from_numpy(X).to(dev)
    Fd = [torch.from_numpy(F).to(dev) for F in Fs]
    Yd = torch.empty((M, int(np.prod(Q, dtype=np.int64))), dtype=Xd.dtype, device=dev)
    tuned = km.tune(M, P, Q, dtype) if args.tune else None
    ws_bytes = km.workspace_size(M, P, Q, dtype)
    ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device=dev)
    steps = km.plan(M, P, Q, dtype)
    flops, planned_bytes = km.cost(M, P, Q, dtype)
    es = Xd.element_size()
    separate_profile = args.separate_profile or args.graph

    stream = torch.cuda.current_stream(dev)
    if args.calibrate_copy and headline:
        # a plain elementwise kernel that reads X once and writes the same number of bytes once
        cal = torch.empty_like(Xd)
        torch.mul(Xd, 1.0, out=cal)
        torch.cuda.synchronize()
        del cal
    # arguments are marshalled once; a step is then exactly one call through the C-ABI
    step = km.Prepared(Xd, Fd, Y=Yd, workspace=ws)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = torch.cuda.Event(enable_timing=True)
    t1 = torch.cuda.Event(enable_timing=True)

    def batch():
        t0.record(stream)
        for _ in range(args.steps):
            step()
        t1.record(stream)
        torch.cuda.synchronize()
        return t0.elapsed_time(t1)

    # Settling: the chip raises its clocks over tens of milliseconds of load, longer than a short
    # warm-up lasts.  Untimed batches of `steps` steps are run until two in a row agree within 1 %.
    settle, spent, prev = 0, 0.0, None
    if not args.no_settle:
        while settle < SETTLE_MAX_BATCHES and spent < SETTLE_MAX_MS:
            cur = batch()
            settle += 1
            spent += cur
            if prev is not None and abs(cur - prev) <= SETTLE_TOLERANCE * max(cur, prev):
                break
            prev = cur

    if not separate_profile:
        km.set_option(km.KM_OPT_PROFILE, 1)     # HIP events around every launch, on the launch stream
    graph = None
    if args.graph:
        # the steps become one graph (kronmatmul_ws allocates nothing and synchronises nothing); one
        # replay warms it up, the next is timed
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for _ in range(args.steps):
                    step()
        stream.wait_stream(side)
        graph.replay()
    torch.cuda.synchronize()
    wall0 = time.perf_counter()
    t0.record(stream)
    if graph is not None:
        graph.replay()
    else:
        for _ in range(args.steps):
            step()
    t1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    ms_total = t0.elapsed_time(t1)
    if separate_profile:
        km.set_option(km.KM_OPT_PROFILE, 1)
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
    per_launch_ms, _ncalls = km.mean_profile()
    km.set_option(km.KM_OPT_PROFILE, 0)
    # a further, untimed pass with the clock probe on a second stream: the shader clock the chip
    # sustains under this load (the matrix cores' published peak is quoted at the maximum clock)
    ticks = torch.zeros(2, dtype=torch.int64, device=dev)
    probe_stream = torch.cuda.Stream()
    probe_us = int(min(max(0.8 * ms_total * 1e3, 50.0), 1e6))
    torch.cuda.synchronize()
    km.clock_probe(ticks, probe_us, probe_stream)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    tk = ticks.tolist()
    shader_mhz = round(100.0 * tk[0] / tk[1], 1) if tk[1] > 0 else None
    ms_per_step = ms_total / args.steps
    gflops = flops / (ms_per_step * 1e-3) / 1e9

    # dominant kernel = the launch kind with the largest share of the step
    keep_mib = km.get_option(km.KM_OPT_KEEP_MIB)
    launches = []
    for st, ms in zip(steps, per_launch_ms):
        nb = es * M * (st["k_in"] + st["k_out"])
        f0, nf = st["first_factor"], st["num_factors"]
        nb += es * sum(P[i] * Q[i] for i in range(f0, f0 + nf))
        k, fl = st["k_in"], 0
        for i in range(f0 + nf - 1, f0 - 1, -1):
            fl += 2 * M * k * Q[i]
            k = k // P[i] * Q[i]
        key = (st["kernel"], st["variant"], st["k_in"], st["k_out"])
        # did the launch before this one leave its output (this one's input) in the last-level cache?
        # (the library's rule: not a call's last launch, 48 MiB to KM_OPT_KEEP_MIB, four times as much
        # for the small-factor family)
        prev = steps[len(launches) - 1] if launches else None
        in_mib = es * M * st["k_in"] / 2.0 ** 20
        kept_in = bool(prev and 48.0 <= in_mib <= keep_mib * (4 if prev["kernel"] == km.KM_KERNEL_FUSED else 1))
        launches.append(dict(key=key, ms=ms, bytes=nb, flops=fl, kept_in=kept_in,
                             name="%s[%s]" % (km.kernel_name(st["kernel"]), shape_runs(P[f0:f0 + nf], Q[f0:f0 + nf]))))
    groups = {}
    for l in launches:
        g = groups.setdefault(l["key"], dict(ms=0.0, n=0, bytes=l["bytes"], flops=l["flops"], name=l["name"],
                                             kept_in=l["kept_in"]))
        g["ms"] += l["ms"]
        g["n"] += 1
    dom = max(groups.values(), key=lambda g: g["ms"])
    dom_ms = dom["ms"] / dom["n"]
    gbs = dom["bytes"] / (dom_ms * 1e-3) / 1e9
    tfl = dom["flops"] / (dom_ms * 1e-3) / 1e12
    peak_tf = PEAKS_TFLOPS[dtype]
    if gbs / HBM_PEAK_GBS >= tfl / peak_tf:
        roofline = dict(bound="hbm", achieved=round(gbs, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=round(gbs / HBM_PEAK_GBS, 4))
    else:
        roofline = dict(bound="mfma", achieved=round(tfl, 2), peak=peak_tf, unit="TFLOP/s",
                        frac=round(tfl / peak_tf, 4))
    traffic, traffic_file = profile_traffic(name)
    roofline.update(traffic=traffic, traffic_source=traffic_file, kernel=dom["name"],
                    kernel_ms=round(dom_ms, 4), launches_per_step=dom["n"],
                    algorithmic_bytes_per_launch=dom["bytes"], flops_per_launch=dom["flops"],
                    alt_frac_hbm=round(gbs / HBM_PEAK_GBS, 4), alt_frac_flops=round(tfl / peak_tf, 4),
                    # True: the kernel's input is an intermediate that the launch before it wrote with
                    # cacheable stores, so part of the algorithmic bytes come from the last-level cache
                    input_partly_cache_resident=dom["kept_in"])

    out = {
        "metric": "kron_matmul_gflops", "value": round(gflops, 1), "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,      # the paper's numbers are another machine's (one V100): context, below
        "dtype": "f32" if dtype == "float32" else "f64", "data": "synthetic",
        "config": {"workload": name, "M": M,
                   "factors": ",".join("%dx%d" % pq for pq in zip(P, Q)) if len(set(zip(P, Q))) > 1
                   else "%dx(%dx%d)" % (len(P), P[0], Q[0]),
                   "launches": [l["name"] for l in launches],
                   "per_launch_ms": [round(l["ms"], 4) for l in launches],
                   "planned_bytes": planned_bytes, "flops": flops,
                   "end_to_end_gbs": round(planned_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                   "wall_ms_per_step": round(wall * 1e3 / args.steps, 4),
                   "settle_steps": settle * args.steps,
                   "shader_clock_mhz_under_load": shader_mhz,
                   "launch_events_in_timed_region": not separate_profile,
                   "steps_replayed_from_one_graph": bool(args.graph),
                   "planner_options": {"kernels": km.get_option(km.KM_OPT_KERNELS),
                                       "max_fuse": km.get_option(km.KM_OPT_MAX_FUSE)},
                   "autotuned": ({"kept_ms": round(tuned[0], 4), "cost_model_ms": round(tuned[1], 4)}
                                 if tuned else False),
                   "paper_context": ({"hardware": "one V100, the paper's Table 1",
                                      "gflops": round(PAPER_GFLOPS[name], 1),
                                      "ratio_to_it": round(gflops / PAPER_GFLOPS[name], 2)}
                                     if name in PAPER_GFLOPS else None)},
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        import oracle
        # bounded sample: rows of the same workload worth at most 1e12 multiply-adds (10-30 s of CPU work;
        # the five measured workloads are smaller than that and are run whole)
        macs_per_row = flops / 2 / M
        rows = int(max(1, min(M, 1e12 // macs_per_row)))
        c0 = time.perf_counter()
        ref = oracle.kron_matmul(X[:rows], Fs)
        cpu_s = time.perf_counter() - c0
        diff = 0.0
        for r0 in range(0, rows, 64):                    # in slabs, to keep host memory small
            got = Yd[r0:min(r0 + 64, rows)].cpu().numpy().astype(np.float64)
            diff = max(diff, float(np.abs(got - ref[r0:r0 + 64]).max()))
        err = diff / float(np.abs(ref).max())
        out["cpu_baseline"] = {"value": round(flops * rows / M / cpu_s / 1e9, 2), "unit": "GFLOP/s",
                               "cores": oracle.threads(), "kind": "oracle",
                               "sample": "%d of %d rows of the same X, %.2f s wall" % (rows, M, cpu_s),
                               "max_rel_err_gpu_vs_oracle": err}
    del step, Xd, Yd, ws, Fd
    torch.cuda.empty_cache()
    return out


def brief(res):
    """What config.other_workloads keeps of a full result."""
    r, c = res["roofline"], res["config"]
    return {"workload": c["workload"], "dtype": res["dtype"], "ms_per_step": res["ms_per_step"],
            "gflops": res["value"], "launches": c["launches"], "kernel": r["kernel"], "kernel_ms": r["kernel_ms"],
            "bound": r["bound"], "frac": r["frac"], "frac_hbm": r["alt_frac_hbm"], "frac_flops": r["alt_frac_flops"],
            "input_partly_cache_resident": r["input_partly_cache_resident"],
            "traffic": r["traffic"], "algorithmic_bytes_per_launch": r["algorithmic_bytes_per_launch"],
            "settle_steps": c["settle_steps"], "shader_clock_mhz_under_load": c["shader_clock_mhz_under_load"],
            "max_rel_err": res.get("cpu_baseline", {}).get("max_rel_err_gpu_vs_oracle"),
            "oracle_gflops": res.get("cpu_baseline", {}).get("value")}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--shape", default=None,
                    help="ad-hoc workload instead of a named one: M:PxQ^N[,PxQ^N...]:f32|f64, "
                         "e.g. 1024:3x3^7:f32 or 10:52x50^1,65x20^1:f32 (uniform X and factors)")
    ap.add_argument("--only-headline", action="store_true",
                    help="measure the headline workload only (default: when it is the default workload, the "
                         "other four measured workloads are run as well and listed in config.other_workloads)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-settle", action="store_true",
                    help="time the steps right after the warm-up steps, without waiting for the clocks to settle")
    ap.add_argument("--separate-profile", action="store_true",
                    help="time the steps without per-launch events and take the per-launch durations from a "
                         "second, untimed pass (for launch-bound problems, where the events cost as much as "
                         "the kernels); default: events inside the timed region")
    ap.add_argument("--graph", action="store_true",
                    help="capture the timed steps in one HIP graph and time its replay (the repeated small-M "
                         "calls of an iterative solver; implies --separate-profile)")
    ap.add_argument("--tune", action="store_true",
                    help="run the library's autotuner for the workload before the warm-up (set-up, not timed)")
    ap.add_argument("--kernels", type=int, default=None,
                    help="bit mask of kernel families the planner may use (the library's KM_OPT_KERNELS), to measure a "
                         "family that is not planned by default, e.g. 9 = generic + the lane-exchange 8x8 kernel")
    ap.add_argument("--max-fuse", type=int, default=None, help="upper limit on factors per launch (KM_OPT_MAX_FUSE)")
    ap.add_argument("--instance", type=int, default=None,
                    help="make the planner take compiled instance number N (a plan step's `variant`) wherever it fits "
                         "(KM_OPT_PREFER_INSTANCE), to measure an instance that is not the planner's choice")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain elementwise copy of X's size (for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build measures one GPU only (rows of X are independent, so they would "
                 "shard across GPUs without communication); run with --gpus 1")

    import torch
    import paper_2401_10187_amd as km

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    km.lib()
    if args.kernels is not None:
        km.set_option(km.KM_OPT_KERNELS, args.kernels)
    if args.max_fuse is not None:
        km.set_option(km.KM_OPT_MAX_FUSE, args.max_fuse)
    if args.instance is not None:
        km.set_option(km.KM_OPT_PREFER_INSTANCE, args.instance + 1)
    if args.shape:
        parse_shape(args.shape)
        args.workload = "shape_" + args.shape
    out = measure(args.workload, args, True)
    if args.workload == HEADLINE and not args.only_headline and not args.shape:
        out["config"]["other_workloads"] = [brief(measure(w, args, False)) for w in OTHERS]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
