"""Host-side contract of bench.py that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_flop_accounting_adds_up_to_18_T_d_f():
    sys.path.insert(0, ROOT)
    import bench
    T, d, f = 4096, 4096, 11008
    per_tag = bench.gemm_flops_by_tag(T, d, f)
    assert sum(v[0] for v in per_tag.values()) == 18.0 * T * d * f
    assert sum(v[1] for v in per_tag.values()) == 8          # GEMM launches per step
    assert set(per_tag) == set(bench.TAG_NAMES)
