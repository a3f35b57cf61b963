"""Pins of the FP8-moment Adam oracle (Section 5) against things other than itself: the library's
AdamW in binary64, closed forms of the first step and of the memoryless case, exact power-of-two
covariance, format limits, and the half-ulp bound of each moment format."""
import numpy as np
import pytest
import torch

from oracle import adam, fp8


def _problem(n=4096, seed=0, gstd=1e-3):
    rng = np.random.default_rng(seed)
    w = rng.standard_normal(n).astype(np.float32) * np.float32(0.02)
    gs = [(rng.standard_normal(n) * gstd * (1.0 + 0.3 * k)).astype(np.float32) for k in range(6)]
    return w, gs


@pytest.mark.parametrize("wd", [0.0, 0.1])
def test_unquantized_oracle_is_the_library_adamw(wd):
    """quantize=False must be the textbook optimizer: torch.optim.AdamW run in binary64 on the same data."""
    w, gs = _problem()
    p = torch.tensor(w.astype(np.float64), requires_grad=True)
    opt = torch.optim.AdamW([p], lr=3e-4, betas=(0.9, 0.95), eps=1e-8, weight_decay=wd)
    st = adam.init(w.size, quantize=False)
    wo = w.copy()
    for g in gs:
        p.grad = torch.tensor(g.astype(np.float64))
        opt.step()
        wo, st = adam.step(wo, g, st, lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=wd, quantize=False)
        ref = p.detach().numpy()
        # binary32 steps against binary64: a few ulps of the weights per step
        assert np.max(np.abs(wo - ref)) <= 8 * np.finfo(np.float32).eps * np.max(np.abs(ref))
    # the moments themselves
    state = opt.state[p]
    # (sums of terms of either sign: the binary32 error is relative to the largest moment)
    em, ev = state["exp_avg"].numpy(), state["exp_avg_sq"].numpy()
    np.testing.assert_allclose(st.m, em, rtol=0, atol=1e-6 * np.abs(em).max())
    np.testing.assert_allclose(st.v, ev, rtol=1e-5, atol=0)


def test_first_step_closed_form():
    """After one step from zero moments: m = (1-b1) g, v = (1-b2) g^2, and the bias-corrected update is
    g / (|g| + eps), i.e. every weight moves by lr against the sign of its gradient."""
    w, gs = _problem()
    g = gs[0]
    wn, st = adam.step(w, g, adam.init(w.size, quantize=False), lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-12,
                       quantize=False)
    np.testing.assert_allclose(st.m, 0.1 * g.astype(np.float64), rtol=1e-6)
    np.testing.assert_allclose(st.v, 0.05 * g.astype(np.float64) ** 2, rtol=1e-6)
    big = np.abs(g) > 1e-5                      # eps / |g| < 1e-7 there; binary32 weights: 1 ulp(0.03) = 4e-9
    assert big.mean() > 0.98
    np.testing.assert_allclose(wn[big], (w.astype(np.float64) - 1e-3 * np.sign(g))[big], rtol=0, atol=8e-9)


def test_memoryless_case_is_a_sign_step_every_time():
    """beta1 = beta2 = 0: m = g and v = g^2 whatever the stored state, with or without FP8 storage."""
    w, gs = _problem()
    for q in (False, True):
        wo, st = w.copy(), adam.init(w.size, quantize=q)
        for g in gs[:3]:
            before = wo.astype(np.float64)
            wo, st = adam.step(wo, g, st, lr=1e-3, beta1=0.0, beta2=0.0, eps=1e-12, quantize=q)
            big = np.abs(g) > 1e-5
            np.testing.assert_allclose(wo[big], (before - 1e-3 * np.sign(g))[big], rtol=0, atol=8e-9)


def test_formats_first_moment_e4m3_second_moment_e5m2():
    """The largest stored magnitude is the format's largest finite code: 0x7E for the first moment
    (E4M3), 0x7B for the second (E5M2), whose codes never carry a sign."""
    w, gs = _problem()
    st = adam.init(w.size)
    for g in gs[:3]:
        w, st = adam.step(w, g, st, lr=3e-4)
        assert st.m.dtype == np.uint8 and st.v.dtype == np.uint8
        assert int((st.m & 0x7F).max()) == 0x7E
        assert int(st.v.max()) == 0x7B
        assert not np.any(st.v & 0x80)
        m, v = adam.moments_from_state(st)
        assert np.all(v >= 0)


def test_power_of_two_covariance_is_exact():
    """Gradients scaled by 2^k (eps = 0, no decay): every binary32 step scales exactly, so the codes and
    the weights are unchanged, the first-moment scale moves by 2^-k and the second-moment scale by 2^-2k."""
    w, gs = _problem(seed=3)
    k = 5
    wa, sa = w.copy(), adam.init(w.size)
    wb, sb = w.copy(), adam.init(w.size)
    for g in gs[:4]:
        wa, sa = adam.step(wa, g, sa, lr=3e-4, eps=0.0)
        wb, sb = adam.step(wb, g * np.float32(2.0 ** k), sb, lr=3e-4, eps=0.0)
        assert np.array_equal(sa.m, sb.m) and np.array_equal(sa.v, sb.v)
        assert np.array_equal(wa, wb)
        assert sb.scale_m == sa.scale_m * np.float32(2.0 ** -k)
        assert sb.scale_v == sa.scale_v * np.float32(2.0 ** (-2 * k))


def test_stored_moments_are_within_half_an_ulp_of_the_exact_ones():
    """Reading the state back gives each moment to within half a unit in the last place of its format
    (2^-4 relative for E4M3's 3 mantissa bits, 2^-3 for E5M2's 2) wherever the scaled value is normal."""
    w, gs = _problem(seed=5)
    g = gs[0]
    _, exact = adam.step(w, g, adam.init(w.size, quantize=False), lr=3e-4, quantize=False)
    _, st = adam.step(w, g, adam.init(w.size), lr=3e-4)
    m, v = adam.moments_from_state(st)
    normal_m = np.abs(exact.m) * st.scale_m >= 2.0 ** -6
    normal_v = exact.v * st.scale_v >= 2.0 ** -14
    assert normal_m.mean() > 0.9 and normal_v.mean() > 0.99
    rel_m = np.abs(m[normal_m] - exact.m[normal_m]) / np.abs(exact.m[normal_m])
    rel_v = np.abs(v[normal_v] - exact.v[normal_v]) / exact.v[normal_v]
    assert rel_m.max() <= 2.0 ** -4 * (1 + 1e-5)
    assert rel_v.max() <= 2.0 ** -3 * (1 + 1e-5)
    # and the errors are really of that size: a float32 or fp16 state would pass a looser test vacuously
    assert rel_m.max() > 2.0 ** -6 and rel_v.max() > 2.0 ** -5


def test_zero_gradient_and_weight_decay_only():
    """All-zero gradients: moments stay zero (codes 0, scales 1); the weights only decay."""
    w, _ = _problem()
    st = adam.init(w.size)
    wn, st = adam.step(w, np.zeros_like(w), st, lr=1e-2, weight_decay=0.1)
    assert not st.m.any() and not st.v.any()
    assert st.scale_m == 1.0 and st.scale_v == 1.0
    np.testing.assert_allclose(wn, w.astype(np.float64) * (1 - 1e-2 * 0.1), rtol=1e-6)


def test_fp8_trajectory_tracks_the_binary32_one():
    """Ten steps with FP8 moments stay close to ten steps with binary32 moments (the claim of Section 5):
    the total displacement of the weights differs by a few percent."""
    w, gs = _problem(n=8192, seed=7)
    rng = np.random.default_rng(11)
    base = rng.standard_normal(w.size).astype(np.float32) * np.float32(1e-3)      # a persistent gradient direction
    wq, sq = w.copy(), adam.init(w.size)
    wf, sf = w.copy(), adam.init(w.size, quantize=False)
    for k in range(10):
        g = base + rng.standard_normal(w.size).astype(np.float32) * np.float32(5e-4)
        wq, sq = adam.step(wq, g, sq, lr=3e-4)
        wf, sf = adam.step(wf, g, sf, lr=3e-4, quantize=False)
    dq, df = wq - w, wf - w
    assert np.linalg.norm(dq - df) / np.linalg.norm(df) < 0.08
    assert sq.step == 10


def test_bias_corrections_closed_form():
    c1, c2 = adam.bias_corrections(0.9, 0.95, 1)
    assert abs(float(c1) - 10.0) < 1e-5 and abs(float(c2) - 20.0) < 1e-4
    c1, c2 = adam.bias_corrections(0.9, 0.95, 10 ** 6)
    assert c1 == 1.0 and c2 == 1.0
