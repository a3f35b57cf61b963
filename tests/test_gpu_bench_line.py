"""The benchmark's one JSON line on a real GPU: a short run of bench.py (few steps, no CPU baseline) must print the
contract's keys with consistent values.  The run also exercises bench.py's own checks (the flop counts the library
reports per launch add up to 18 T d f)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_short_run_prints_the_contract_line():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "5", "--warmup", "2", "--no-cpu-baseline"],
                       capture_output=True, text=True, timeout=500, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-3000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1, r.stdout[-2000:]
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["higher_is_better"] is True
    assert d["unit"] == "TFLOP/s" and d["vs_baseline"] is None and "workload" in d["config"]
    T, dm, f = 4096, 4096, 11008
    assert abs(d["value"] * 1e12 * d["ms_per_step"] * 1e-3 / (18.0 * T * dm * f) - 1.0) < 1e-9
    rf = d["roofline"]
    assert rf["bound"] == "mfma" and rf["peak"] == 5000.0 and rf["unit"] == "TFLOP/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-12 and 0.0 < rf["frac"] < 1.0
    assert abs(rf["achieved"] * 1e12 * rf["avg_launch_ms"] * 1e-3 / rf["flops_per_launch"] - 1.0) < 1e-9
    assert rf["kernel"] in rf["kernels"]
    assert rf["traffic"] is None or rf["traffic"] > 0
    assert sum(v["flops_per_launch"] * v["launches_per_step"] for v in rf["kernels"].values()) == 18.0 * T * dm * f
    for v in rf["elementwise"].values():
        assert 0.0 < v["frac_of_hbm_peak"] < 1.0 or v["algorithmic_MB_per_step"] < 1.0
    plan = rf["backward_plan"]
    assert 0 <= plan["dw3_sets_in_first_launch"] <= plan["dw3_sets"] == 86
    for k in ("weights_cached", "delayed_scaling", "delayed_scaling_weights_cached", "plain_fp8", "bf16_last_layer",
              "training_forward_only", "inference_forward"):
        assert d[k]["value"] > 0.0, k
    # the ordering of the paper's Table 3: plain FP8 >= Smooth-SwiGLU (within noise) > last layer in bf16
    assert d["bf16_last_layer"]["value"] < d["value"]
