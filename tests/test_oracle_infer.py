"""Pins of the inference oracle (factors folded into w1 and w3, last paragraph of Section 4.4)."""
import numpy as np

import synth
from oracle import fp8, infer, mlp


def _np(inp):
    return {k: synth.bf16_to_f32_numpy(v) for k, v in inp.items() if hasattr(v, "dtype") and k != "aligned"}


def test_folding_does_not_change_the_function():
    """Q := identity: for ANY positive factors (s_i, 1/s_i) the folded block is the plain SwiGLU block --
    the claim that the modification preserves the function (Section 4.4)."""
    npi = _np(synth.make_inputs(48, 64, 80, seed=3))
    plain = mlp.forward(npi["x"], npi["W1"], npi["W2"], npi["W3"], quantized=False, smooth=False).Y
    rng = np.random.default_rng(0)
    s = np.exp(rng.standard_normal(80) * 3.0)
    y = infer.forward_unquantized(npi["x"], npi["W1"], npi["W2"], npi["W3"], s, 1.0 / s)
    assert np.max(np.abs(y - plain)) <= 1e-12 * np.max(np.abs(plain))


def test_calibrated_inference_tracks_the_training_forward():
    """Factors calibrated on a batch, inference on the same batch: the output agrees with the training
    block's at the FP8 noise level, and the folded first layer really carries the factor."""
    npi = _np(synth.make_inputs(128, 64, 96, seed=7, aligned_channels=4))
    tr = mlp.forward(npi["x"], npi["W1"], npi["W2"], npi["W3"])
    p = infer.prepare(npi["W1"], npi["W2"], npi["W3"], tr.s, tr.sinv)
    inf = infer.forward(npi["x"], p)
    assert np.array_equal(inf.x_q, tr.x_q) and np.array_equal(p.w3_q, tr.w3_q) and p.s3 == tr.sw3
    rel = np.linalg.norm(inf.Y - tr.Y) / np.linalg.norm(tr.Y)
    assert rel < 6e-2, rel          # two more E4M3 roundings than the training path (w1 after folding, h without bf16)
    # every channel of the product fills the format: its largest code sits in the top binade of E4M3
    top = (inf.h_q & 0x7F).max(axis=0)
    assert np.all(top[tr.a > 0] >= 0x78) and np.all(top <= 0x7E)
    # largest code of each prepared matrix is the format maximum (a per-tensor Q of a non-zero matrix)
    for q in (p.w1_q, p.w2_q, p.w3_q):
        assert int((q & 0x7F).max()) == 0x7E


def test_row_scaling_of_w1_is_what_is_quantized():
    """prepare() must scale row i of w1 (channel i), not column i: decode and compare with s_i * w1_i."""
    npi = _np(synth.make_inputs(16, 32, 48, seed=9))
    rng = np.random.default_rng(1)
    s = (2.0 ** rng.integers(-3, 4, size=48)).astype(np.float32)        # powers of two: products are exact
    p = infer.prepare(npi["W1"], npi["W2"], npi["W3"], s, (1.0 / s).astype(np.float32))
    back = fp8.decode(p.w1_q, fp8.E4M3).astype(np.float64) / float(p.s1)
    want = npi["W1"].astype(np.float64) * s[:, None]
    scale = np.abs(want).max()
    assert np.max(np.abs(back - want)) <= 2.0 ** -4 * scale            # half an ulp of E4M3 at the top binade
    back3 = fp8.decode(p.w3_q, fp8.E4M3).astype(np.float64) / float(p.s3)
    want3 = npi["W3"].astype(np.float64) / s[None, :]
    assert np.max(np.abs(back3 - want3)) <= 2.0 ** -4 * np.abs(want3).max()
