"""The benchmark's command-line contract: one JSON line with the agreed keys; more than one GPU is
refused with a message (this build measures one GPU)."""
import glob
import json
import os
import re
import subprocess
import sys

import pytest

from conftest import ROOT

BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    proc = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=300)
    assert proc.returncode != 0
    assert "one GPU" in (proc.stdout + proc.stderr)
    assert not any(line.startswith("{") for line in proc.stdout.splitlines())


@pytest.mark.gpu
@pytest.mark.parametrize("workload,extra", [("c1_f32_m16_8x8x3", []), ("table4_id21_f64", []),
                                            ("c1_f32_m16_8x8x3", ["--graph"])])
def test_one_json_line_with_the_agreed_keys(workload, extra):
    proc = subprocess.run([sys.executable, BENCH, "--workload", workload, "--steps", "7", "--warmup", "3"] + extra,
                          capture_output=True, text=True, timeout=600)
    assert proc.returncode == 0, proc.stderr[-2000:]
    lines = [line for line in proc.stdout.splitlines() if line.strip()]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 7 and out["warmup"] == 3
    assert out["metric"] == "kron_matmul_gflops" and out["unit"] == "GFLOP/s" and out["higher_is_better"] is True
    assert out["data"] == "synthetic" and out["config"]["workload"] == workload
    assert out["value"] > 0 and out["ms_per_step"] > 0
    roof = out["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert roof["bound"] in ("hbm", "mfma", "alu") and abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    assert 300.0 < out["config"]["shader_clock_mhz_under_load"] < 3000.0
    cpu = out["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in cpu, key
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1
    assert cpu["max_rel_err_gpu_vs_oracle"] <= (1e-5 if out["dtype"] == "f32" else 1e-12)


def test_measured_traffic_comes_from_the_profile_summaries():
    """roofline.traffic is not a constant in bench.py: it is read from the rocprofv3 summary under
    profiles/ whose header names the workload.  Every summary's header figure must be the one its own
    counter table gives, bench.py must find it, and the five measured workloads must each have one."""
    import bench
    files = sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md")))
    assert files
    for path in files:
        text = open(path).read()
        workload = re.search(r"^workload: (.+)$", text, re.M)
        traffic = re.search(r"^hbm_traffic_bytes_per_launch: (\d+)$", text, re.M)
        algorithmic = re.search(r"^algorithmic_bytes_per_launch: (\d+)$", text, re.M)
        table = re.search(r"^Dominant kernel: ([\d,]+) B measured against ([\d,]+) B algorithmic", text, re.M)
        assert workload and traffic and algorithmic and table, path
        t, a = int(traffic.group(1)), int(algorithmic.group(1))
        assert t == int(table.group(1).replace(",", "")) and a == int(table.group(2).replace(",", "")), path
        # measured traffic well above the algorithmic bytes would mean wasted re-reads
        assert 0.95 * a <= t <= (1.1 * a if a > 1 << 24 else 2 * a), (path, t, a)
        if " " not in workload.group(1):          # summaries of non-default planner options carry a tag after the name
            assert bench.profile_traffic(workload.group(1)) == (t, os.path.relpath(path, ROOT)), path
    for w in [bench.HEADLINE] + bench.OTHERS:
        assert bench.profile_traffic(w)[0] is not None, w


def test_profiler_commands_keep_to_what_the_profiler_can_collect():
    """Every rocprofv3 command of the harness runs `python3 bench.py ...` directly after `--`, collects
    counters in runs of their own (never together with a trace), and asks for no more counters of one
    hardware block than a single run can hold (8 SQ, 4 TCC, 4 TCP, 2 TA, 2 GRBM)."""
    from paper_2401_10187_amd import profile
    limits = {"SQ_": 8, "TCC_": 4, "TCP_": 4, "TA_": 2, "TD_": 2, "GRBM_": 2}
    for name in profile.PASSES:
        cmd = profile.pass_command("c2_f32_m1024_8x8x6", name, "/tmp/out")
        assert cmd[:3] == ["timeout", "-s", "KILL"] and cmd[4] == "rocprofv3"
        split = cmd.index("--")
        assert cmd[split + 1] == "python3" and cmd[split + 2].endswith("bench.py")
        opts = cmd[5:split]
        if "--pmc" in opts:
            assert not any(o in opts for o in ("--kernel-trace", "--stats", "--sys-trace", "--hip-trace", "--hsa-trace"))
            counters = opts[opts.index("--pmc") + 1:opts.index("--output-format")]
            for block, most in limits.items():
                stems = {re.sub(r"_(sum|avr|min|max)$", "", c) for c in counters if c.startswith(block)}
                cost = sum(3 if c == "FETCH_SIZE" else 2 if c == "WRITE_SIZE" else 1 for c in stems)
                assert cost <= most, (name, block, sorted(stems))
        else:
            assert "--kernel-trace" in opts
