"""The grouped launches (several GEMMs in one grid, dW3 shared out between the two backward launches, the range
pass over W3 inside the gate/up GEMM's grid, the casts of h and w3 in one launch) are a scheduling matter: every
output must have exactly the bits the single launches give.  The switch (SSG_GEMM_GROUPING=0) is read once per
process, so the single-launch run happens in a child process on the same seeded inputs."""
import os
import subprocess
import sys

import pytest
import torch

import synth

pytestmark = pytest.mark.gpu

import paper_2409_12517_amd as ssg  # noqa: E402
import gpu_util as gu  # noqa: E402
import test_gpu_mlp as tm  # noqa: E402

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
# 176 tiles each for dH, dW3, dW1, dW2 and 64 for dX: the first backward launch does not fit one round of 256
# compute units, so the library moves part of dW3 into the second
SHAPE = (2048, 2048, 5632)
SEED = 77

CHILD = r"""
import sys, torch
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
import synth, test_gpu_grouping as tg
out = tg.run_block()
torch.save({{k: v.cpu() for k, v in out.items()}}, {path!r})
print("child done", flush=True)
"""


def run_block():
    T, d, f = SHAPE
    blk = tm.Block(synth.make_inputs(T, d, f, seed=SEED))
    blk.fwd()
    blk.bwd()
    out = {"y": blk.y, "dx": blk.dx, "dW1": blk.dW1, "dW2": blk.dW2, "dW3": blk.dW3,
           "h_q": blk.sv("h_q", (T, f), torch.uint8), "w3_q": blk.sv("w3_q", (d, f), torch.uint8),
           "w3_camax": blk.sv("w3_camax", (f,), torch.float32), "scales": blk.sv("scales", (16,), torch.float32),
           "du_q": blk.wv("du_q", (T, f), torch.uint8), "dg_q": blk.wv("dg_q", (T, f), torch.uint8)}
    return {k: v.clone() for k, v in out.items()}


def test_single_launches_give_the_same_bits_as_grouped_launches(tmp_path):
    assert os.environ.get("SSG_GEMM_GROUPING", "1") != "0", "this process must run the grouped launches"
    first, total = ssg.ssg_mlp_bwd_plan(ssg.make_desc(*SHAPE), torch.cuda.get_device_properties(0).multi_processor_count)
    assert 0 <= first < total, "the shape was chosen so that dW3 is split between the two launches"
    grouped = run_block()
    path = str(tmp_path / "single.pt")
    env = dict(os.environ, SSG_GEMM_GROUPING="0")
    code = CHILD.format(root=ROOT, tests=os.path.join(ROOT, "tests"), path=path)
    r = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "child done" in r.stdout, r.stderr[-2000:]
    single = torch.load(path, weights_only=True)
    for k, v in grouped.items():
        a, b = v.cpu(), single[k]
        # bit patterns, so that -0.0 / NaN payloads count too
        assert torch.equal(a.view(torch.uint8) if a.dtype != torch.uint8 else a,
                           b.view(torch.uint8) if b.dtype != torch.uint8 else b), k
