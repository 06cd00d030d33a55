"""bench.py's one JSON line: the fields a reader of the measurement relies on, on the small workloads.

The benchmark runs as a child process (its own GPU context), exactly as a user starts it."""
import json
import math
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*flags):
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *flags], cwd=ROOT, capture_output=True,
                          text=True, timeout=300)
    assert proc.returncode == 0, proc.stderr[-2000:]
    lines = [l for l in proc.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, f"expected one line on stdout, got {len(lines)}"
    return json.loads(lines[0])


def test_line_of_the_tiny_workload_with_the_oracle_beside_it():
    j = _bench("--workload", "C1", "--steps", "5", "--warmup", "2")
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 5 and j["warmup"] == 2
    assert j["unit"] == "TFLOP/s" and j["higher_is_better"] is True and j["dtype"] == "bf16" and j["data"] == "synthetic"
    assert j["vs_baseline"] is None                      # the paper quotes no number for this metric
    assert "workload" in j["config"] and "model" not in j["config"]
    assert j["value"] > 0 and j["ms_per_step"] > 0
    # useful flops: forward 2 sum L(L+1) d Hq, backward counted 2.5 x
    cfg = j["config"]
    fwd = 2 * cfg["sum_L_Lplus1"] * cfg["head_dim"] * cfg["q_heads"]
    assert cfg["fwd_useful_flops"] == fwd
    assert math.isclose(j["value"], 3.5 * fwd / (j["ms_per_step"] * 1e-3) / 1e12, rel_tol=5e-2)
    cpu = j["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["unit"] == "TFLOP/s" and cpu["value"] > 0 and cpu["cores"] >= 1 and cpu["sample"]


def test_roofline_object_of_a_mid_sized_workload():
    j = _bench("--workload", "C2", "--steps", "5", "--warmup", "2", "--no-cpu-baseline")
    r = j["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert r["kernel"] == "bwd_dkv_kernel"
    assert math.isclose(r["frac"], r["achieved"] / r["peak"], rel_tol=1e-3, abs_tol=1e-4)
    assert 0.05 < r["frac"] < 1.0
    # achieved = the pass's 4 GEMMs over the visible pairs / its average launch time
    assert math.isclose(r["achieved"], r["flops_per_launch"] / (j["kernel_ms"]["bwd_dkv_kernel"] * 1e-3) / 1e12, rel_tol=1e-3)
    assert r["flops_per_launch"] == 2 * j["config"]["fwd_useful_flops"]   # 4 GEMMs against the forward's 2
    # the step cannot be shorter than its kernels
    assert j["ms_per_step"] >= sum(j["kernel_ms"].values()) * 0.98
    assert r["measured_mfma_peak"] > r["measured_mfma_peak_varied_operands"] > 500.0
