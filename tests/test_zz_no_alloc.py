"""The allocation-free inference forward (ssg_infer_fwd_noalloc, workspace in a static device array of the
library) against ssg_infer_fwd with a caller-allocated workspace: same kernels, so the same bytes -- on two
calls in a row, the second with a smaller input (the array keeps the first call's contents)."""
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu

import paper_2409_12517_amd as ssg  # noqa: E402
import gpu_util as gu  # noqa: E402


def _calibrate(inp):
    """The per-channel factors of a calibration call of the training block and the prepared weights."""
    T, d = inp["x"].shape
    f = inp["W1"].shape[0]
    desc = ssg.make_desc(T, d, f)
    x, W1, W2, W3 = (gu.dev(inp[k]) for k in ("x", "W1", "W2", "W3"))
    saved = torch.empty(ssg.ssg_mlp_saved_bytes(desc), dtype=torch.uint8, device=gu.DEV)
    y = torch.empty(T, d, dtype=torch.bfloat16, device=gu.DEV)
    ssg.ssg_mlp_fwd(desc, x, W1, W2, W3, y, saved)
    v = ssg.ssg_mlp_view_saved(desc, saved)
    s = ssg.view_tensor(saved, saved.data_ptr(), v.s, (f,), torch.float32).clone()
    sinv = ssg.view_tensor(saved, saved.data_ptr(), v.sinv, (f,), torch.float32).clone()
    prep = torch.empty(ssg.ssg_infer_prepared_bytes(desc), dtype=torch.uint8, device=gu.DEV)
    ssg.ssg_infer_prepare(desc, W1, W2, W3, s, sinv, prep)
    torch.cuda.synchronize()
    return prep


def test_noalloc_forward_matches_the_workspace_form_on_two_calls():
    d, f = 512, 1376
    big = synth.make_inputs(528, d, f, seed=81)
    prep = _calibrate(big)
    small_x = synth.make_inputs(144, d, f, seed=82)["x"]
    for x_host in (big["x"], small_x):                      # the second call is smaller than the first
        T = x_host.shape[0]
        x = gu.dev(x_host)
        desc = ssg.make_desc(T, d, f)
        assert ssg.ssg_infer_workspace_bytes(desc) <= ssg.ssg_infer_noalloc_max_bytes()
        work = torch.empty(ssg.ssg_infer_workspace_bytes(desc), dtype=torch.uint8, device=gu.DEV)
        y_ref = torch.empty(T, d, dtype=torch.bfloat16, device=gu.DEV)
        y = torch.full((T, d), float("nan"), dtype=torch.bfloat16, device=gu.DEV)
        ssg.ssg_infer_fwd(desc, x, prep, y_ref, work)
        before = torch.cuda.memory_allocated()
        ssg.ssg_infer_fwd_noalloc(desc, x, prep, y)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16))
        assert bool(torch.isfinite(y.float()).all())
    # a shape beyond the static array is refused before anything is launched
    with pytest.raises(ssg.SsgError) as e:
        ssg.ssg_infer_fwd_noalloc(ssg.make_desc(4096, 4096, 11008), gu.dev(big["x"]), prep, y, prepared_bytes=1 << 40)
    assert e.value.status == ssg.SSG_ERR_WORKSPACE
