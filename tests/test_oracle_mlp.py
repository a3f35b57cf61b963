"""Pins for the oracle's SwiGLU, GEMM and MLP forward/backward (CPU only).

Independent references used here: PyTorch's float64 CPU ops and autograd (for
the unquantized function and its gradients), exact integer brute force (for
the FP8 contractions), closed forms and invariances that the paper states.
"""
import os

import numpy as np
import pytest
import torch

import synth
from oracle import fp8, gemm, mlp, quant, swiglu


def _inputs(T=48, d=32, f=80, seed=0, **kw):
    t = synth.make_inputs(T, d, f, seed, **kw)
    return {k: (synth.bf16_to_f32_numpy(v) if isinstance(v, torch.Tensor) and v.dtype == torch.bfloat16 else v)
            for k, v in t.items()}


# ------------------------------------------------------------------ SwiGLU

def test_swiglu_closed_form_against_torch():
    rng = np.random.default_rng(0)
    u, g = rng.standard_normal(1000) * 5, rng.standard_normal(1000) * 5
    ref = (torch.from_numpy(u) * torch.nn.functional.silu(torch.from_numpy(g))).numpy()
    assert np.allclose(swiglu.swiglu(u, g), ref, rtol=1e-14, atol=0)
    assert swiglu.swiglu(np.array([2.0]), np.array([0.0]))[0] == 0.0
    assert swiglu.sigmoid(np.array([0.0]))[0] == 0.5


def test_swiglu_quadratic_limit(golden_dir):
    # Section 4.1: w1 = w2, w1.x = 1  =>  SwiGLU(c x) / c^2 -> 1
    rows = [l.split() for l in open(os.path.join(golden_dir, "swiglu_limit.txt")) if l.strip() and l[0] != "#"]
    rng = np.random.default_rng(1)
    w = rng.standard_normal(16)
    x = w / (w @ w)                                   # w.x = 1
    for c_s, tol_s in rows:
        c = float(c_s)
        val = swiglu.swiglu(np.array([(c * x) @ w]), np.array([(c * x) @ w]))[0]
        assert abs(val / c ** 2 - 1.0) <= float(tol_s) + 1e-12
    # and a linear-growth neuron for contrast: Swish alone is at most linear
    assert abs(swiglu.swish(np.array([1000.0]))[0] / 1000.0) <= 1.0


def test_swiglu_grads_against_finite_differences_and_autograd():
    rng = np.random.default_rng(2)
    u, g, dh = (rng.standard_normal(200) * 3 for _ in range(3))
    du, dg = swiglu.swiglu_grads(u, g, dh)
    eps = 1e-6
    fd_u = (swiglu.swiglu(u + eps, g) - swiglu.swiglu(u - eps, g)) / (2 * eps) * dh
    fd_g = (swiglu.swiglu(u, g + eps) - swiglu.swiglu(u, g - eps)) / (2 * eps) * dh
    assert np.allclose(du, fd_u, rtol=1e-6, atol=1e-8)
    assert np.allclose(dg, fd_g, rtol=1e-6, atol=1e-8)
    ut = torch.tensor(u, requires_grad=True); gt = torch.tensor(g, requires_grad=True)
    (ut * torch.nn.functional.silu(gt) * torch.tensor(dh)).sum().backward()
    assert np.allclose(du, ut.grad.numpy(), rtol=1e-12, atol=1e-14)
    assert np.allclose(dg, gt.grad.numpy(), rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ GEMM

@pytest.mark.parametrize("fa,fb", [(fp8.E4M3, fp8.E4M3), (fp8.E5M2, fp8.E4M3)], ids=["e4m3xe4m3", "e5m2xe4m3"])
def test_fp64_gemm_equals_exact_integer_brute_force(fa, fb):
    rng = np.random.default_rng(4)
    M, N, K = 9, 7, 33
    def codes(fmt, shape):
        c = rng.integers(0, fmt.max_code + 1, size=shape).astype(np.uint8)
        return c | (rng.integers(0, 2, size=shape).astype(np.uint8) << 7)
    a, b = codes(fa, (M, K)), codes(fb, (N, K))
    a[0, :] = fa.max_code; b[0, :] = fb.max_code            # worst-case magnitude row
    got = gemm.matmul_nt(a, fa, b, fb)
    ref = gemm.matmul_nt_exact(a, fa, b, fb)
    for m in range(M):
        for n in range(N):
            exact = ref[m][n]
            assert abs(got[m, n] - float(exact)) <= 2.0 ** -52 * K * abs(float(exact)) + 1e-300
    assert float(ref[0][0]) == K * fp8.max_finite(fa) * fp8.max_finite(fb)
    # a transposed operand gives the transposed result
    assert np.array_equal(gemm.matmul_nt(b, fb, a, fa), got.T)


# ------------------------------------------------------------------ helpers of mlp

def test_round_bf16_matches_torch():
    rng = np.random.default_rng(6)
    v = np.concatenate([rng.standard_normal(100000) * rng.choice([1e-30, 1e-3, 1, 1e4, 1e30], 100000),
                        [0.0, -0.0, 1.00390625, 1.01171875, 3.3895313892515355e38, 1e-40, 2.0 ** -133, 2.0 ** -134]])
    v32 = v.astype(np.float32)                       # bf16 rounding of a binary32 value: compare with torch
    ref = torch.from_numpy(v32).to(torch.bfloat16).to(torch.float64).numpy()
    got = mlp.round_bf16(v32.astype(np.float64))
    assert np.array_equal(ref, got)
    # ties to even on a float64 value that binary32 cannot hold exactly
    assert mlp.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert mlp.round_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40]))[0] == 1.0 + 2.0 ** -7


# ------------------------------------------------------------------ unquantized function

def _torch_mlp(inp):
    x, W1, W2, W3 = (torch.tensor(inp[k], dtype=torch.float64, requires_grad=True) for k in ("x", "W1", "W2", "W3"))
    y = ((x @ W1.T) * torch.nn.functional.silu(x @ W2.T)) @ W3.T
    return x, W1, W2, W3, y


@pytest.mark.parametrize("smooth", [False, True])
def test_unquantized_block_and_gradients_match_torch_autograd(smooth):
    inp = _inputs()
    x, W1, W2, W3, y = _torch_mlp(inp)
    (y * torch.tensor(inp["dY"], dtype=torch.float64)).sum().backward()
    fw = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"], quantized=False, smooth=smooth)
    bw = mlp.backward(fw, inp["dY"])
    def close(a, b):
        return np.abs(a - b).max() <= 1e-12 * np.abs(b).max()
    assert close(fw.Y, y.detach().numpy())
    assert close(bw.dX, x.grad.numpy())
    assert close(bw.dW1, W1.grad.numpy())
    assert close(bw.dW2, W2.grad.numpy())
    assert close(bw.dW3, W3.grad.numpy())


def test_smooth_swiglu_leaves_the_function_unchanged():
    # Section 4.4: scaling by s_i before Q and by 1/s_i in w3 is the identity when Q is.
    inp = _inputs(seed=3, aligned_channels=4)
    plain = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"], quantized=False, smooth=False)
    smooth = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"], quantized=False, smooth=True)
    assert np.abs(plain.Y - smooth.Y).max() <= 1e-13 * np.abs(plain.Y).max()
    assert np.allclose(smooth.s * smooth.sinv, 1.0, rtol=1e-15)
    # binary32 factors of the quantized path: s_i * sinv_i = 1 up to two roundings
    q = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"])
    assert np.abs(q.s.astype(np.float64) * q.sinv.astype(np.float64) - 1.0).max() <= 2.0 ** -22


# ------------------------------------------------------------------ quantized block

def test_quantized_forward_structure_and_closeness():
    inp = _inputs(T=64, d=64, f=96, seed=5)
    ref = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"], quantized=False, smooth=False)
    for smooth in (False, True):
        q = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"], smooth=smooth)
        assert q.x_q.dtype == np.uint8 and q.x_q.shape == (64, 64) and q.h_q.shape == (64, 96) and q.w3_q.shape == (64, 96)
        assert (q.x_q & 0x7F).max() == 0x7E and (q.w1_q & 0x7F).max() == 0x7E and (q.w3_q & 0x7F).max() == 0x7E
        # U, G hold bf16 values
        assert np.array_equal(mlp.round_bf16(q.U), q.U) and np.array_equal(mlp.round_bf16(q.G), q.G)
        # FP8 noise level, nothing worse
        rel = np.abs(q.Y - ref.Y).max() / np.abs(ref.Y).max()
        assert rel < 0.12, rel
    q = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"], smooth=True)
    # every channel fills the format (Section 4.4: per-channel maxima set the factors)
    assert np.all((q.h_q & 0x7F).max(axis=0) == 0x7E)
    assert np.array_equal(q.a, np.abs(q.h).max(axis=0))


def test_w3_fold_amax_shortcut():
    # max_ij fl32(|w_ji| * sinv_i) equals max_i fl32(max_j |w_ji| * sinv_i): rounding is monotone.
    inp = _inputs(T=64, d=48, f=80, seed=8)
    q = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"])
    W3 = inp["W3"].astype(np.float32)
    full = np.abs((W3 * q.sinv[None, :]).astype(np.float32)).max()
    short = (np.abs(W3).max(axis=0) * q.sinv).astype(np.float32).max()
    assert full == short
    assert q.sw3 == quant.scale_from_amax(np.float32(short), fp8.E4M3)


def test_channel_permutation_equivariance():
    inp = _inputs(T=32, d=32, f=48, seed=9)
    perm = np.random.default_rng(0).permutation(48)
    a = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"])
    b = mlp.forward(inp["x"], inp["W1"][perm], inp["W2"][perm], inp["W3"][:, perm])
    # W1 and W2 are quantized per tensor, so permuting rows permutes codes
    assert np.array_equal(a.w1_q[perm], b.w1_q)
    assert np.array_equal(a.s[perm], b.s)
    assert np.array_equal(a.h_q[:, perm], b.h_q)
    assert np.array_equal(a.w3_q[:, perm], b.w3_q)
    assert np.abs(a.Y - b.Y).max() <= 2.0 ** -7 * np.abs(a.Y).max()   # at most bf16 rounding of a reassociated sum


def test_scaling_one_channel_only_moves_its_factor():
    # Multiply row i of W1 by 2^k.  U's column i doubles exactly only if the per-tensor code of W1 is
    # unchanged, so drive the check at the level the paper states it: scale column i of h.
    inp = _inputs(T=32, d=32, f=48, seed=10)
    q = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"])
    h2 = q.h.copy(); h2[:, 5] *= np.float32(2.0 ** 6)
    a2, s2, sinv2 = mlp.channel_scales(h2)
    assert s2[5] == q.s[5] * np.float32(2.0 ** -6) and sinv2[5] == q.sinv[5] * np.float32(2.0 ** 6)
    keep = np.arange(48) != 5
    assert np.array_equal(s2[keep], q.s[keep])
    assert np.array_equal(quant.cast_with_scale(h2, s2[None, :], fp8.E4M3), q.h_q)   # codes unchanged


def test_equal_channel_maxima_reduce_to_per_tensor_quantization():
    rng = np.random.default_rng(12)
    h = rng.standard_normal((64, 16)).astype(np.float32)
    h = (h / np.abs(h).max(axis=0, keepdims=True)).astype(np.float32)
    h[np.abs(h).argmax(axis=0), np.arange(16)] = 1.0          # every channel max is exactly 1
    a, s, sinv = mlp.channel_scales(h)
    assert np.all(a == 1.0)
    per_channel = quant.cast_with_scale(h, s[None, :], fp8.E4M3)
    per_tensor, st, _ = quant.quantize_per_tensor(h, fp8.E4M3)
    assert np.array_equal(per_channel, per_tensor) and np.all(s == st)


def test_outlier_channels_saturate_plain_stale_but_not_smooth():
    # Section 3 / 4.4: a stale per-tensor scale overflows when aligned channels spike; per-channel factors do not.
    calm = _inputs(T=128, d=64, f=96, seed=13)
    spiky = _inputs(T=128, d=64, f=96, seed=13, aligned_channels=4)
    stale = mlp.forward(calm["x"], calm["W1"], calm["W2"], calm["W3"], smooth=False).sh
    q_plain = mlp.forward(spiky["x"], spiky["W1"], spiky["W2"], spiky["W3"], smooth=False, h_scale=stale)
    assert quant.count_saturated(q_plain.h, stale, fp8.E4M3) > 0
    q_smooth = mlp.forward(spiky["x"], spiky["W1"], spiky["W2"], spiky["W3"], smooth=True)
    assert quant.count_saturated(q_smooth.h, q_smooth.s[None, :], fp8.E4M3) == 0
    # with a current per-tensor scale nothing saturates but small channels are flushed to zero more often
    q_cur = mlp.forward(spiky["x"], spiky["W1"], spiky["W2"], spiky["W3"], smooth=False)
    assert quant.count_flushed(q_cur.h, q_cur.h_q) > quant.count_flushed(q_smooth.h, q_smooth.h_q)


@pytest.mark.parametrize("smooth", [False, True])
def test_quantized_backward_is_the_unquantized_one_plus_fp8_noise(smooth):
    inp = _inputs(T=64, d=64, f=96, seed=14)
    ref_f = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"], quantized=False, smooth=False)
    ref_b = mlp.backward(ref_f, inp["dY"])
    q_f = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"], smooth=smooth)
    q_b = mlp.backward(q_f, inp["dY"])
    assert (q_b.dy_q & 0x7F).max() == 0x7B and (q_b.du_q & 0x7F).max() == 0x7B and (q_b.dg_q & 0x7F).max() == 0x7B
    assert q_b.sdu != q_b.sdg
    for name in ("dX", "dW1", "dW2", "dW3"):
        a, b = getattr(q_b, name), getattr(ref_b, name)
        assert a.shape == b.shape
        rel = np.linalg.norm(a - b) / np.linalg.norm(b)
        assert rel < 0.12, (name, rel)
    assert np.array_equal(mlp.round_bf16(q_b.dX), q_b.dX)
    assert np.array_equal(q_b.dW1.astype(np.float32).astype(np.float64), q_b.dW1)


def test_planted_mistakes_are_caught_by_the_autograd_pin():
    # A wrong sign or a dropped term in the SwiGLU derivative must fail the pin above; check the pin has teeth.
    u, g, dh = np.array([0.7]), np.array([-1.3]), np.array([1.0])
    du, dg = swiglu.swiglu_grads(u, g, dh)
    sg = swiglu.sigmoid(g)
    wrong = dh * u * sg * (1.0 - g * (1.0 - sg))
    assert abs(wrong - dg) > 0.1


# ------------------------------------------------------------------ last layer left in bf16 (Section 4.3)

def test_bf16_last_layer_against_torch_bf16_matmul_and_autograd():
    """The comparison variant of Table 3 ("SwiGLU output in BF16"): pins that do not restate the oracle.
    (i) y against PyTorch's CPU bf16 matmul of the same bf16 operands (an independent library: it accumulates in
    binary32 and rounds once, the oracle in binary64 and rounds once; they may differ by one bf16 step);
    (ii) dH, dW3 against float64 autograd of the bilinear form sum(dY * (h W3^T)) at the oracle's own bf16 h;
    (iii) the FP8 part upstream (x^, w1^, w2^, U, G) is the one of the fully quantized block, bit for bit;
    (iv) leaving h in bf16 brings y closer to the unquantized block than either FP8 form of h."""
    inp = _inputs(T=64, d=64, f=96, seed=17)
    v = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"], w3_layer_fp8=False)
    q = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"], smooth=True)
    # (iii)
    assert np.array_equal(v.x_q, q.x_q) and np.array_equal(v.w1_q, q.w1_q) and np.array_equal(v.w2_q, q.w2_q)
    assert np.array_equal(v.U, q.U) and np.array_equal(v.G, q.G) and np.array_equal(v.h, q.h)
    assert v.h_q is None and v.w3_q is None
    # the stored SwiGLU output holds bf16 values, one rounding away from the binary32 product
    assert np.array_equal(mlp.round_bf16(v.h_b), v.h_b)
    assert np.abs(v.h_b - v.h).max() <= 2.0 ** -8 * np.abs(v.h).max()
    # (i)
    hb_t = torch.from_numpy(v.h_b).to(torch.bfloat16)
    assert np.array_equal(hb_t.to(torch.float64).numpy(), v.h_b)          # exactly representable
    w3_t = torch.from_numpy(inp["W3"]).to(torch.bfloat16)
    y_t = (hb_t @ w3_t.T).to(torch.float64).numpy()
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(v.Y), 1e-30))) - 7)
    assert np.all(np.abs(y_t - v.Y) <= ulp + 1e-6 * np.abs(v.Y).max())
    assert np.mean(y_t == v.Y) > 0.9
    # (ii)
    b = mlp.backward(v, inp["dY"])
    h_t = torch.tensor(v.h_b, dtype=torch.float64, requires_grad=True)
    W3_t = torch.tensor(inp["W3"], dtype=torch.float64, requires_grad=True)
    ((h_t @ W3_t.T) * torch.tensor(inp["dY"], dtype=torch.float64)).sum().backward()
    assert np.abs(b.dH - h_t.grad.numpy()).max() <= 1e-12 * np.abs(b.dH).max()
    assert np.abs(b.dW3 - W3_t.grad.numpy()).max() <= 2.0 ** -23 * np.abs(b.dW3).max()      # one binary32 rounding
    assert b.dy_q is None and (b.du_q & 0x7F).max() == 0x7B
    # the gradients that stay in FP8 are those of the quantized block fed with this dH
    ref_f = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"], quantized=False, smooth=False)
    ref_b = mlp.backward(ref_f, inp["dY"])
    for name in ("dX", "dW1", "dW2", "dW3"):
        rel = np.linalg.norm(getattr(b, name) - getattr(ref_b, name)) / np.linalg.norm(getattr(ref_b, name))
        assert rel < 0.12, (name, rel)
    # (iv)
    err = lambda f: np.linalg.norm(f.Y - ref_f.Y)
    plain = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"], smooth=False)
    assert err(v) < err(q) and err(v) < err(plain)


def test_bf16_last_layer_planted_mistakes_fail():
    """A transposed W3 or a dW3 taken from the unrounded h must trip the pins above."""
    inp = _inputs(T=32, d=32, f=32, seed=19)
    v = mlp.forward(inp["x"], inp["W1"], inp["W2"], inp["W3"], w3_layer_fp8=False)
    b = mlp.backward(v, inp["dY"])
    wrong_dH = np.asarray(inp["dY"], np.float64) @ np.asarray(inp["W3"], np.float64).T       # square shapes: runs, but wrong
    assert np.abs(wrong_dH - b.dH).max() > 0.1 * np.abs(b.dH).max()
    dW3_unrounded = np.asarray(inp["dY"], np.float64).T @ v.h.astype(np.float64)
    assert np.abs(dW3_unrounded - b.dW3).max() > 2.0 ** -20 * np.abs(b.dW3).max()
