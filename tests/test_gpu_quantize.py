"""GPU parity: amax, per-tensor Q, Smooth-SwiGLU quantization and the w3 fold,
bit-exact against the oracle on identical input bytes (through the C ABI)."""
import numpy as np
import pytest
import torch

import synth
from oracle import fp8, mlp, quant

pytestmark = pytest.mark.gpu

import paper_2409_12517_amd as ssg  # noqa: E402  (no fallback: a missing library is an error)
import gpu_util as gu  # noqa: E402

FMT = {ssg.SSG_E4M3: fp8.E4M3, ssg.SSG_E5M2: fp8.E5M2}


def _quantize(src, fmt, mode=None, rnd=None, scale=None, transposed=True):
    mode = ssg.SSG_SCALE_CURRENT if mode is None else mode
    rnd = ssg.SSG_ROUND_EXACT_DIV if rnd is None else rnd
    rows, cols = src.shape
    dt = ssg.SSG_BF16 if src.dtype == torch.bfloat16 else ssg.SSG_F32
    dst, dst_t = gu.empty_u8(rows, cols), (gu.empty_u8(cols, rows) if transposed else None)
    sc = gu.empty_f32(1) if scale is None else torch.tensor([scale], dtype=torch.float32, device=gu.DEV)
    am = gu.empty_f32(1)
    ssg.ssg_quantize(src, dt, rows, cols, fmt, mode, rnd, dst, dst_t, sc, am)
    torch.cuda.synchronize()
    return gu.u8(dst), (gu.u8(dst_t) if transposed else None), gu.scalar(sc), gu.scalar(am)


@pytest.mark.parametrize("fmt", [ssg.SSG_E4M3, ssg.SSG_E5M2])
def test_cast_exhaustive_vectors(fmt):
    """Every code value, every midpoint and its two binary32 neighbours, saturation, underflow,
    specials -- with a given scale of 1 so that the cast alone is tested."""
    f = FMT[fmt]
    tab = fp8.decode_table(f)[: f.max_code + 1]
    mids = (tab[:-1] + tab[1:]) / 2
    fmax = np.float32(tab[-1])
    vals = np.concatenate([
        tab, mids, np.nextafter(mids.astype(np.float32), np.float32(0)), np.nextafter(mids.astype(np.float32), np.float32(1e30)),
        [np.nextafter(fmax, np.float32(np.inf)), fmax * 1.03, fmax * 1.04, fmax * 2, 1e30, np.inf, 3.4e38],
        [tab[1] / 2, tab[1] / 4, 1e-30, 1e-45, 0.0],
    ]).astype(np.float32)
    vals = np.concatenate([vals, -vals, [np.nan]]).astype(np.float32)
    n = ((len(vals) + 255) // 256) * 256
    vals = np.concatenate([vals, np.zeros(n - len(vals), np.float32)]).reshape(16, n // 16)
    got, got_t, _, am = _quantize(gu.dev(torch.from_numpy(vals)), fmt, mode=ssg.SSG_SCALE_GIVEN, scale=1.0)
    ref = fp8.satcast(vals, f)
    assert np.array_equal(got, ref)
    assert np.array_equal(got_t, ref.T)
    assert am == np.inf                      # amax ignores the NaN and reports the Inf


@pytest.mark.parametrize("fmt", [ssg.SSG_E4M3, ssg.SSG_E5M2])
@pytest.mark.parametrize("shape", [(256, 256), (688, 256), (256, 688), (16, 16), (144, 1040), (2048, 4096)])
def test_per_tensor_quantize_bit_exact(fmt, shape):
    gen = torch.Generator().manual_seed(shape[0] * 7 + shape[1] + fmt)
    std = 1e-3 if fmt == ssg.SSG_E5M2 else 0.02
    src = (torch.randn(*shape, generator=gen) * std).to(torch.bfloat16)
    got, got_t, sc, am = _quantize(gu.dev(src), fmt)
    ref, ref_sc, ref_am = quant.quantize_per_tensor(synth.bf16_to_f32_numpy(src), FMT[fmt])
    assert am == ref_am and sc == ref_sc
    assert np.array_equal(got, ref)
    assert np.array_equal(got_t, ref.T)
    assert (got & 0x7F).max() == FMT[fmt].max_code


def test_quantize_f32_source_pow2_and_given_scale():
    gen = torch.Generator().manual_seed(5)
    src = torch.randn(128, 384, generator=gen) * 3.7
    v = src.numpy()
    got, _, sc, am = _quantize(gu.dev(src), ssg.SSG_E4M3, rnd=ssg.SSG_ROUND_POW2, transposed=False)
    ref, ref_sc, ref_am = quant.quantize_per_tensor(v, fp8.E4M3, pow2=True)
    assert sc == ref_sc and am == ref_am and np.array_equal(got, ref)
    got, got_t, sc, _ = _quantize(gu.dev(src), ssg.SSG_E5M2, mode=ssg.SSG_SCALE_GIVEN, scale=12345.0)
    ref, _, _ = quant.quantize_per_tensor(v, fp8.E5M2, scale=np.float32(12345.0))
    assert sc == np.float32(12345.0) and np.array_equal(got, ref) and np.array_equal(got_t, ref.T)


def test_quantize_degenerate_inputs():
    z = torch.zeros(32, 48, dtype=torch.bfloat16)
    got, got_t, sc, am = _quantize(gu.dev(z), ssg.SSG_E4M3)
    assert sc == 1.0 and am == 0.0 and not got.any() and not got_t.any()
    tiny = torch.full((16, 16), 1e-38, dtype=torch.bfloat16)       # fmax/amax overflows binary32
    got, _, sc, am = _quantize(gu.dev(tiny), ssg.SSG_E4M3)
    ref, ref_sc, _ = quant.quantize_per_tensor(synth.bf16_to_f32_numpy(tiny), fp8.E4M3)
    assert sc == ref_sc == np.finfo(np.float32).max and np.array_equal(got, ref)
    # empty tensor: nothing to do, scale 1, amax 0
    sc_t, am_t = gu.empty_f32(1), gu.empty_f32(1)
    ssg.ssg_quantize(None, ssg.SSG_BF16, 0, 64, ssg.SSG_E4M3, ssg.SSG_SCALE_CURRENT, ssg.SSG_ROUND_EXACT_DIV,
                     None, None, sc_t, am_t)
    torch.cuda.synchronize()
    assert gu.scalar(sc_t) == 1.0 and gu.scalar(am_t) == 0.0


def test_amax_entry_point():
    gen = torch.Generator().manual_seed(9)
    src = (torch.randn(4096 * 33, generator=gen) * 5).to(torch.bfloat16)
    src[12345] = float("nan")
    out = gu.empty_f32(1)
    ssg.ssg_amax(gu.dev(src), ssg.SSG_BF16, src.numel(), out)
    torch.cuda.synchronize()
    assert gu.scalar(out) == quant.amax(synth.bf16_to_f32_numpy(src))


def _ug(T, f, seed, spiky=False):
    gen = torch.Generator().manual_seed(seed)
    U = (torch.randn(T, f, generator=gen) * 1.3).to(torch.bfloat16)
    G = (torch.randn(T, f, generator=gen) * 1.3).to(torch.bfloat16)
    if spiky:
        U[:, 3] *= 60; G[:, 3] *= 60            # one aligned-looking channel with a huge product
        G[:, 5] = -100.0                        # sigma underflows: h is (almost) zero in this channel
        U[:, 7] = 0.0                           # an all-zero channel: s = sinv = 1
    return U, G


@pytest.mark.parametrize("T,f,spiky", [(256, 688, False), (528, 144, True), (1024, 1024, True)])
@pytest.mark.parametrize("smooth", [1, 0])
def test_smooth_swiglu_quantize_bit_exact_given_gpu_h(T, f, spiky, smooth):
    """The per-channel maxima, factors and codes must be exactly what the oracle derives from the
    GPU's own fp32 SwiGLU product (the product itself is compared with a tolerance below)."""
    U, G = _ug(T, f, seed=T + f, spiky=spiky)
    Ud, Gd = gu.dev(U), gu.dev(G)
    h = gu.empty_f32(T, f)
    ssg.ssg_swiglu(Ud, Gd, T, f, h)
    h_q, h_qT = gu.empty_u8(T, f), gu.empty_u8(f, T)
    s, sinv, camax = gu.empty_f32(f), gu.empty_f32(f), gu.empty_f32(f)
    ssg.ssg_smooth_swiglu_quantize(Ud, Gd, T, f, smooth, h_q, h_qT, s, sinv, camax)
    torch.cuda.synchronize()
    h_np = gu.f32(h)
    if smooth:
        a, s_ref, sinv_ref = mlp.channel_scales(h_np)
        ref_q = quant.cast_with_scale(h_np, s_ref[None, :], fp8.E4M3)
    else:
        a = np.abs(h_np).max(axis=0)
        ref_q, sh, _ = quant.quantize_per_tensor(h_np, fp8.E4M3)
        s_ref, sinv_ref = np.full(f, sh, np.float32), np.ones(f, np.float32)
    assert np.array_equal(gu.f32(camax), a)
    assert np.array_equal(gu.f32(s), s_ref) and np.array_equal(gu.f32(sinv), sinv_ref)
    assert np.array_equal(gu.u8(h_q), ref_q)
    assert np.array_equal(gu.u8(h_qT), ref_q.T)
    if smooth:
        live = a > 1e-30          # below ~1.3e-36 the factor clamps at the largest float and the channel cannot fill
        assert np.all((gu.u8(h_q) & 0x7F).max(axis=0)[live] == 0x7E)      # every live channel fills the format


def test_gpu_swiglu_product_close_to_oracle():
    T, f = 512, 256
    U, G = _ug(T, f, seed=77, spiky=True)
    h = gu.empty_f32(T, f)
    ssg.ssg_swiglu(gu.dev(U), gu.dev(G), T, f, h)
    torch.cuda.synchronize()
    from oracle import swiglu
    ref = swiglu.swiglu(synth.bf16_to_f32_numpy(U), synth.bf16_to_f32_numpy(G))
    got = gu.f32(h).astype(np.float64)
    # fp32 evaluation: exp (1 ulp), add, divide, two multiplies -> a few ulps of the result
    assert np.all(np.abs(got - ref) <= 6 * 2.0 ** -23 * np.abs(ref) + 1e-30)


@pytest.mark.parametrize("d,f", [(256, 688), (1024, 2048)])
def test_fold_w3_bit_exact(d, f):
    gen = torch.Generator().manual_seed(d + f)
    W3 = (torch.randn(d, f, generator=gen) * 0.02).to(torch.bfloat16)
    sinv_np = np.exp(np.random.default_rng(1).uniform(-8, 3, f)).astype(np.float32)
    sinv_np[7] = 1.0
    w3_q, w3_qT = gu.empty_u8(d, f), gu.empty_u8(f, d)
    camax, sc, am = gu.empty_f32(f), gu.empty_f32(1), gu.empty_f32(1)
    ssg.ssg_fold_w3(gu.dev(W3), gu.dev(torch.from_numpy(sinv_np)), d, f, w3_q, w3_qT, camax, sc, am)
    torch.cuda.synchronize()
    w = synth.bf16_to_f32_numpy(W3)
    ref_q, ref_sc, ref_am = mlp.fold_w3(w, sinv_np)
    assert np.array_equal(gu.f32(camax), np.abs(w).max(axis=0))
    assert gu.scalar(am) == ref_am and gu.scalar(sc) == ref_sc
    assert np.array_equal(gu.u8(w3_q), ref_q) and np.array_equal(gu.u8(w3_qT), ref_q.T)
