"""GPU parity: the FP8 MFMA GEMM against the oracle's fp64 contraction (through the C ABI)."""
import numpy as np
import pytest
import torch

from oracle import fp8, gemm

pytestmark = pytest.mark.gpu

import paper_2409_12517_amd as ssg  # noqa: E402
import gpu_util as gu  # noqa: E402

FMT = {ssg.SSG_E4M3: fp8.E4M3, ssg.SSG_E5M2: fp8.E5M2}


def _codes(rng, fmt, shape, gaussian=True):
    """Codes with the value distribution of a per-tensor-scaled Gaussian tensor (or uniform over all finite codes)."""
    f = FMT[fmt]
    if gaussian:
        v = rng.standard_normal(shape).astype(np.float32)
        v = v * np.float32(fp8.max_finite(f) / np.abs(v).max())
        return fp8.satcast(v, f)
    c = rng.integers(0, f.max_code + 1, size=shape).astype(np.uint8)
    return c | (rng.integers(0, 2, size=shape).astype(np.uint8) << 7)


def _run(a, a_fmt, b, sa, sb, c_dtype):
    M, K = a.shape
    N = b.shape[0]
    A, B = gu.dev(torch.from_numpy(a)), gu.dev(torch.from_numpy(b))
    sa_t = None if sa is None else torch.tensor([sa], dtype=torch.float32, device=gu.DEV)
    sb_t = None if sb is None else torch.tensor([sb], dtype=torch.float32, device=gu.DEV)
    C = torch.empty(M, N, dtype=torch.float32 if c_dtype == ssg.SSG_F32 else torch.bfloat16, device=gu.DEV)
    ssg.ssg_gemm_fp8(A, a_fmt, B, ssg.SSG_E4M3, M, N, K, sa_t, sb_t, C, c_dtype)
    torch.cuda.synchronize()
    return gu.f32(C)


@pytest.mark.parametrize("a_fmt", [ssg.SSG_E4M3, ssg.SSG_E5M2])
def test_tiny_gemm_against_exact_integer_sum(a_fmt):
    """Operands confined to one binade (plus sign and zeros): every product has the same few
    fractional bits, so neither the matrix core's product alignment nor the fp32 sums round, and
    the result must equal the integer brute force bit for bit (checks operand layouts, indexing
    and the ragged-tile handling)."""
    rng = np.random.default_rng(1)
    M, N, K = 48, 32, 80
    fa = FMT[a_fmt]
    ea = np.full((M, K), fa.bias)
    a = ((ea << fa.man_bits) | rng.integers(0, 1 << fa.man_bits, size=(M, K)) | (rng.integers(0, 2, size=(M, K)) << 7)).astype(np.uint8)
    eb = np.full((N, K), 7)
    b = ((eb << 3) | rng.integers(0, 8, size=(N, K)) | (rng.integers(0, 2, size=(N, K)) << 7)).astype(np.uint8)
    a[rng.random((M, K)) < 0.1] = 0
    b[rng.random((N, K)) < 0.1] = 0x80
    got = _run(a, a_fmt, b, None, None, ssg.SSG_F32)
    exact = gemm.matmul_nt_exact(a, fa, b, fp8.E4M3)
    ref = np.array([[float(v) for v in row] for row in exact])
    assert np.array_equal(got.astype(np.float64), ref)


@pytest.mark.parametrize("a_fmt", [ssg.SSG_E4M3, ssg.SSG_E5M2])
@pytest.mark.parametrize("M,N,K", [(256, 256, 128), (256, 688, 256), (688, 256, 256), (256, 256, 688),
                                   (16, 16, 16), (272, 528, 400), (1024, 768, 2048)])
@pytest.mark.parametrize("c_dtype", [ssg.SSG_F32, ssg.SSG_BF16])
def test_gemm_against_fp64_oracle(a_fmt, M, N, K, c_dtype):
    rng = np.random.default_rng(M + 3 * N + 7 * K + a_fmt)
    a, b = _codes(rng, a_fmt, (M, K)), _codes(rng, ssg.SSG_E4M3, (N, K))
    sa, sb = np.float32(37.5), np.float32(0.8125)
    got = _run(a, a_fmt, b, sa, sb, c_dtype)
    ref = gemm.matmul_nt(a, FMT[a_fmt], b, fp8.E4M3) / (float(sa) * float(sb))
    gu.assert_close_gemm(got, ref, c_dtype == ssg.SSG_BF16, f"gemm {M}x{N}x{K}")


def test_gemm_uniform_codes_full_dynamic_range():
    """Codes uniform over the whole format (11+ binades in one dot product): the matrix core aligns
    products before adding, so this is the hardest case for the stated tolerance."""
    rng = np.random.default_rng(3)
    M, N, K = 256, 256, 512
    a, b = _codes(rng, ssg.SSG_E5M2, (M, K), gaussian=False), _codes(rng, ssg.SSG_E4M3, (N, K), gaussian=False)
    got = _run(a, ssg.SSG_E5M2, b, None, None, ssg.SSG_F32)
    ref = gemm.matmul_nt(a, fp8.E5M2, b, fp8.E4M3)
    gu.assert_close_gemm(got, ref, False, "uniform codes")


@pytest.mark.gpu
def test_mfma_rate_probe_runs_and_checks_its_arguments():
    """The register-only MFMA loop: flop count as documented, checksum written, small workspace refused."""
    import ctypes
    import os
    probe = ctypes.CDLL(os.path.join(os.path.dirname(ssg.LIB_PATH), "libssg_probe.so"))   # the benchmark's helper library
    probe.ssg_probe_mfma_rate.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                                          ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    ws = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
    ws[:65536].fill_(0x38)                       # E4M3 1.0 everywhere: every accumulator ends at iters * 64
    flops = ctypes.c_double(0.0)
    st = torch.cuda.current_stream().cuda_stream
    assert probe.ssg_probe_mfma_rate(ws.data_ptr(), ws.numel(), 3, ctypes.byref(flops), st) == 0
    torch.cuda.synchronize()
    assert flops.value == 256 * 4 * 3 * 16 * 2.0 * 32 * 32 * 64
    sink = ws[65536:65536 + 256 * 256 * 4].view(torch.float32)
    assert torch.all(sink == 16 * 16 * 3 * 64.0)
    assert probe.ssg_probe_mfma_rate(ws.data_ptr(), 4096, 3, ctypes.byref(flops), st) == -1


@pytest.mark.parametrize("c_dtype", [ssg.SSG_F32, ssg.SSG_BF16])
def test_nan_and_inf_codes_propagate_to_their_rows_only(c_dtype):
    """One NaN code in a row of A (E4M3 0x7F) and one infinity in another (E5M2 0x7C): those output rows are
    NaN / non-finite, every other row is untouched (also through the bf16 packing of the epilogue)."""
    rng = np.random.default_rng(5)
    M, N, K = 272, 320, 256
    a = _codes(rng, ssg.SSG_E5M2, (M, K))
    b = _codes(rng, ssg.SSG_E4M3, (N, K))
    clean = _run(a, ssg.SSG_E5M2, b, 2.0, 0.5, c_dtype)
    a2 = a.copy()
    a2[37, 100] = 0x7F          # E5M2 NaN
    a2[200, 3] = 0x7C           # E5M2 +inf
    got = _run(a2, ssg.SSG_E5M2, b, 2.0, 0.5, c_dtype)
    assert np.all(np.isnan(got[37]))
    assert not np.any(np.isfinite(got[200][fp8.decode(b[:, 3], fp8.E4M3) != 0]))
    keep = np.ones(M, bool)
    keep[[37, 200]] = False
    assert np.array_equal(got[keep], clean[keep])


@pytest.mark.parametrize("M,N,K", [(256, 256, 128), (256, 512, 384), (272, 336, 208), (48, 32, 80), (1024, 768, 1040)])
@pytest.mark.parametrize("layout", [(0, 1), (1, 1)])
@pytest.mark.parametrize("a_fmt", [ssg.SSG_E4M3, ssg.SSG_E5M2])
def test_kmajor_operands_match_the_contiguous_form(M, N, K, layout, a_fmt):
    """K-major operands (stored [K,M] / [K,N], read through the transposing LDS load) must give the bytes of
    the K-contiguous form on the same logical operands, for whole tiles, ragged tiles and ragged K -- and the
    K-contiguous form is the one checked against the oracle above."""
    rng = np.random.default_rng(M + N + K)
    a = _codes(rng, a_fmt, (M, K))
    b = _codes(rng, ssg.SSG_E4M3, (N, K))
    want = _run(a, a_fmt, b, 3.0, 0.25, ssg.SSG_F32)
    ak, bk = layout
    A = gu.dev(torch.from_numpy(np.ascontiguousarray(a.T) if ak else a))
    B = gu.dev(torch.from_numpy(np.ascontiguousarray(b.T) if bk else b))
    sa = torch.tensor([3.0], dtype=torch.float32, device=gu.DEV)
    sb = torch.tensor([0.25], dtype=torch.float32, device=gu.DEV)
    for c_dtype, tdt in ((ssg.SSG_F32, torch.float32), (ssg.SSG_BF16, torch.bfloat16)):
        C = torch.empty(M, N, dtype=tdt, device=gu.DEV)
        ssg.ssg_gemm_fp8_layout(A, a_fmt, ak, B, ssg.SSG_E4M3, bk, M, N, K, sa, sb, C, c_dtype)
        torch.cuda.synchronize()
        ref = want if c_dtype == ssg.SSG_F32 else torch.from_numpy(want).to(torch.bfloat16).float().numpy()
        assert np.array_equal(gu.f32(C), ref)


def test_kmajor_unsupported_combination_is_refused():
    t = torch.zeros(256 * 256, dtype=torch.uint8, device=gu.DEV)
    c = torch.zeros(256, 256, device=gu.DEV)
    with pytest.raises(ssg.SsgError) as e:
        ssg.ssg_gemm_fp8_layout(t, ssg.SSG_E4M3, 1, t, ssg.SSG_E4M3, 0, 256, 256, 256, None, None, c, ssg.SSG_F32)
    assert e.value.status == ssg.SSG_ERR_UNSUPPORTED


@pytest.mark.gpu
@pytest.mark.parametrize("c_dtype", [ssg.SSG_F32, ssg.SSG_BF16])
def test_extreme_scales_do_not_zero_the_product(c_dtype):
    """A gradient tensor with a tiny range has a scale near 1e35; times a weight scale the product of the two
    scales leaves the binary32 range although the dequantized result does not.  The oracle divides in float64."""
    rng = np.random.default_rng(11)
    M, N, K = 64, 48, 256
    a, b = _codes(rng, ssg.SSG_E5M2, (M, K)), _codes(rng, ssg.SSG_E4M3, (N, K))
    sa, sb = np.float32(57344.0) / np.float32(1e-30), np.float32(448.0) / np.float32(1e-3)
    with np.errstate(over="ignore"):
        assert not np.isfinite(sa * sb)                   # the binary32 product of the scales overflows
    got = _run(a, ssg.SSG_E5M2, b, float(sa), float(sb), c_dtype)
    ref = gemm.matmul_nt(a, fp8.E5M2, b, fp8.E4M3) / (np.float64(sa) * np.float64(sb))
    assert np.abs(ref).max() > 1e-36 and np.isfinite(ref).all()
    gu.assert_close_gemm(got, ref, c_dtype == ssg.SSG_BF16, "extreme scales")
