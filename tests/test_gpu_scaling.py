"""Delayed scaling with an amax history (Sections 2, 6.2) on the GPU: a sequence of calls whose inputs
change magnitude (so that remembered ranges are too small, too large and eventually forgotten), every
call checked against the oracle driven by the same history rule."""
import numpy as np
import pytest
import torch

import synth
from oracle import scaling

pytestmark = pytest.mark.gpu

import paper_2409_12517_amd as ssg  # noqa: E402
import gpu_util as gu  # noqa: E402
import test_gpu_mlp as tm  # noqa: E402

NAMES = ("x", "w1", "w2", "dy", "du", "dg")


def _state_words(state):
    return state[: 6 * 32 * 4].view(torch.float32).cpu().numpy().reshape(6, 32)


def _scaled_inputs(base, fx, fw, fdy):
    inp = dict(base)
    inp["x"] = (base["x"].float() * fx).to(torch.bfloat16)
    inp["W1"] = (base["W1"].float() * fw).to(torch.bfloat16)
    inp["W2"] = (base["W2"].float() * fw).to(torch.bfloat16)
    inp["dY"] = (base["dY"].float() * fdy).to(torch.bfloat16)
    return inp


def test_sequence_of_calls_follows_the_oracle_history():
    base = synth.make_inputs(272, 256, 400, seed=41)
    state = torch.empty(ssg.ssg_mlp_scaling_state_bytes(), dtype=torch.uint8, device=gu.DEV)
    ssg.ssg_mlp_scaling_init(state)
    torch.cuda.synchronize()
    w = _state_words(state)
    assert np.all(w[:, 0] == 1.0) and not w[:, 1:].any()
    ds = scaling.DelayedScaling()
    # call 0 under current scaling fills the history; then ranges shrink, grow fourfold (saturation), return
    plan = [(ssg.SSG_SCALE_CURRENT, 1.0, 1.0, 1.0), (ssg.SSG_SCALE_DELAYED, 0.5, 1.0, 2.0),
            (ssg.SSG_SCALE_DELAYED, 4.0, 1.5, 0.25), (ssg.SSG_SCALE_DELAYED, 1.0, 1.0, 8.0)]
    for call, (mode, fx, fw, fdy) in enumerate(plan):
        inp = _scaled_inputs(base, fx, fw, fdy)
        npi = tm._np_inputs(inp)
        blk = tm.Block(inp)
        blk.desc = ssg.make_desc(blk.T, blk.d, blk.f, scale_mode=mode, scaling_state=state, keep_bf16_grads=1)
        fwd_scales = ds.scales(("x", "w1", "w2")) if mode == ssg.SSG_SCALE_DELAYED else None
        bwd_scales = ds.scales(("dy", "du", "dg")) if mode == ssg.SSG_SCALE_DELAYED else None
        blk.fwd()
        ref_fw, fw_gpu = tm.check_forward(blk, npi, scales=fwd_scales)
        blk.bwd()
        ref_bw, cont = tm.check_backward(blk, npi, ref_fw, fw_gpu, scales=bwd_scales)
        # the history: ranges of the GPU's own tensors.  x, w1, w2, dy are inputs; dU, dG are the stored bf16
        # tensors (kept under delayed scaling too: keep_bf16_grads), whose ranges `cont` holds: all exact.
        w = _state_words(state)
        ds.record_all(ref_fw.amax)
        ds.record_all({"dy": cont.amax["dy"], "du": cont.amax["du"], "dg": cont.amax["dg"]})
        for k, n in enumerate(NAMES):
            assert w[k, 0] == ds.scale(n), (call, n, w[k, 0], ds.scale(n))
            assert np.array_equal(w[k, 8:24], ds.hist[n]), (call, n)
            assert w[k, 2] == ds.hist[n][(ds.pos[n] - 1) % scaling.HISTORY]
        if call == 2:
            # x grew fourfold against a remembered range: the excess saturates, on both sides alike
            x_q = gu.u8(blk.sv("x_q", (blk.T, blk.d), torch.uint8))
            assert int(((x_q & 0x7F) == 0x7E).sum()) > 100
    # the record slots are left clean for the next call
    assert not state[256 * 4:].any()


def test_delayed_mode_needs_a_state_and_cached_weights_keep_their_history():
    base = synth.make_inputs(64, 64, 96, seed=43)
    blk = tm.Block(base)
    blk.desc = ssg.make_desc(blk.T, blk.d, blk.f, scale_mode=ssg.SSG_SCALE_DELAYED)
    with pytest.raises(ssg.SsgError):
        blk.fwd()
    state = torch.empty(ssg.ssg_mlp_scaling_state_bytes(), dtype=torch.uint8, device=gu.DEV)
    ssg.ssg_mlp_scaling_init(state)
    blk.desc = ssg.make_desc(blk.T, blk.d, blk.f, scaling_state=state)
    blk.fwd(); blk.bwd()
    before = _state_words(state).copy()
    blk.desc = ssg.make_desc(blk.T, blk.d, blk.f, scale_mode=ssg.SSG_SCALE_DELAYED, scaling_state=state,
                             weights_cached=1)
    y0 = blk.y.clone()
    blk.fwd(); blk.bwd()
    after = _state_words(state)
    assert np.array_equal(before[1:3], after[1:3])            # w1, w2 entries untouched
    pos = lambda w: int(w[0, 1:2].view(np.int32)[0])          # the ring position is an integer word
    assert pos(after) == pos(before) + 1                      # x advanced
    assert torch.equal(y0, blk.y)                             # same inputs, history = their own ranges


def test_recorded_range_ignores_nan_and_keeps_infinity():
    """The cast that records the range for the history takes it on the raw bf16 patterns: NaN must not
    enter it (as in the stand-alone range pass), infinity must."""
    base = synth.make_inputs(64, 64, 96, seed=47)
    state = torch.empty(ssg.ssg_mlp_scaling_state_bytes(), dtype=torch.uint8, device=gu.DEV)
    ssg.ssg_mlp_scaling_init(state)
    blk = tm.Block(base)
    blk.desc = ssg.make_desc(blk.T, blk.d, blk.f, scale_mode=ssg.SSG_SCALE_DELAYED, scaling_state=state)
    x = base["x"].clone()
    x[3, 5] = float("nan")
    x[7, 9] = -float("nan")
    big = float(x[torch.isfinite(x.float())].float().abs().max())
    blk.x = gu.dev(x)
    blk.fwd()
    assert _state_words(state)[0, 2] == np.float32(big)
    x[11, 1] = -float("inf")
    blk.x = gu.dev(x)
    blk.fwd()
    assert _state_words(state)[0, 2] == np.inf
