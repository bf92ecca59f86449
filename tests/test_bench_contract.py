"""The benchmark's command-line contract: one JSON line with the agreed keys; more than one GPU is
refused with a message (this build measures one GPU)."""
import json
import os
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
