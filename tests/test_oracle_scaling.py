"""Pins of the delayed-scaling oracle: it must reduce to the (pinned) current-scaling path when the
tensor does not change, saturate exactly what exceeds the remembered range, and forget after H calls."""
import numpy as np

import synth
from oracle import fp8, mlp, quant, scaling


def _np(inp):
    return {k: synth.bf16_to_f32_numpy(v) for k, v in inp.items() if hasattr(v, "dtype") and k != "aligned"}


def test_stationary_tensors_reduce_to_current_scaling():
    """Same inputs every call: from the second call on the remembered range of x, W1, W2, dY is the
    tensor's own, so the forward equals the current-scaling block byte for byte; dU and dG of the first
    call were formed from a badly scaled dY, so the backward follows one call later."""
    npi = _np(synth.make_inputs(64, 64, 96, seed=5))
    cur_f = mlp.forward(npi["x"], npi["W1"], npi["W2"], npi["W3"])
    cur_b = mlp.backward(cur_f, npi["dY"])
    ds = scaling.DelayedScaling(history=1)       # only the previous call counts: no older, larger range lingers
    for call in range(3):
        fw = mlp.forward(npi["x"], npi["W1"], npi["W2"], npi["W3"], scales=ds.scales(("x", "w1", "w2")))
        bw = mlp.backward(fw, npi["dY"], scales=ds.scales(("dy", "du", "dg")))
        ds.record_all(fw.amax)
        ds.record_all(bw.amax)
        if call == 0:
            assert fw.sx == 1.0 and bw.sdy == 1.0              # empty history: scale 1
        else:
            assert np.array_equal(fw.x_q, cur_f.x_q) and np.array_equal(fw.h_q, cur_f.h_q)
            assert np.array_equal(fw.Y, cur_f.Y)
            assert np.array_equal(bw.dy_q, cur_b.dy_q) and np.array_equal(bw.dU, cur_b.dU)
        if call == 2:
            for n in ("dX", "dW1", "dW2", "dW3"):
                assert np.array_equal(getattr(bw, n), getattr(cur_b, n))


def test_growth_saturates_exactly_the_excess():
    """A tensor that grows fourfold between calls: elements whose magnitude exceeds the remembered
    maximum land on the largest code, all others are encoded as under a scale that fits."""
    rng = np.random.default_rng(0)
    v = rng.standard_normal(4096).astype(np.float32)
    ds = scaling.DelayedScaling(names=("x",))
    ds.record("x", quant.amax(v))
    big = (v * np.float32(4.0)).astype(np.float32)
    codes, s, a = quant.quantize_per_tensor(big, fp8.E4M3, scale=ds.scale("x"))
    assert s == quant.scale_from_amax(quant.amax(v), fp8.E4M3)
    over = np.abs(big) * s > 448 * (1 + 2.0 ** -4)
    assert over.sum() > 100
    assert np.all((codes[over] & 0x7F) == 0x7E)
    assert quant.count_saturated(big, s, fp8.E4M3) == int((np.abs(big).astype(np.float64) * float(s) > 448 + 16).sum())
    assert a == quant.amax(big)


def test_history_window():
    """A spike governs the scale for exactly H calls."""
    ds = scaling.DelayedScaling(names=("dy",), history=4)
    ds.record("dy", 100.0)
    for k in range(3):
        ds.record("dy", 1.0)
        assert ds.scale("dy") == np.float32(57344.0) / np.float32(100.0)
    ds.record("dy", 1.0)
    assert ds.scale("dy") == np.float32(57344.0)
    assert scaling.FORMATS["x"] is fp8.E4M3 and scaling.FORMATS["dg"] is fp8.E5M2
