"""The single-product GEMMs have two kernels: 4 waves with 128 x 128 wave tiles (the default) and
8 waves with 128 x 64 wave tiles (SSG_GEMM_VARIANT=0; the form the two-product GEMM always uses).
The choice is read once per process, so the 8-wave form is exercised by running the GEMM and MLP
parity tests again in a child process."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.gpu
def test_eight_wave_kernels_pass_the_parity_tests():
    env = dict(os.environ, SSG_GEMM_VARIANT="0")
    cmd = [sys.executable, "-u", "-m", "pytest", "-x", "-q", "-m", "gpu", "--timeout", "120", "--timeout-method",
           "thread", "-p", "no:cacheprovider", os.path.join(ROOT, "tests", "test_gpu_gemm.py"),
           os.path.join(ROOT, "tests", "test_gpu_mlp.py")]
    r = subprocess.run(cmd, env=env, cwd=ROOT, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-4000:] + r.stderr[-2000:]
