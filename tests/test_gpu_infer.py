"""GPU parity of the inference form (factors folded into w1 and w3, end of Section 4.4)."""
import numpy as np
import pytest
import torch

import synth
from oracle import fp8, infer, mlp
from oracle import gemm as fp8_gemm
from oracle import swiglu as oswiglu

pytestmark = pytest.mark.gpu

import paper_2409_12517_amd as ssg  # noqa: E402
import gpu_util as gu  # noqa: E402
import test_gpu_mlp as tm  # noqa: E402


def _rank_table():
    """Position of every finite E4M3 code in the order of its value (so adjacent codes differ by 1)."""
    vals = fp8.decode_table(fp8.E4M3).astype(np.float64)
    finite = np.array([c for c in range(256) if (c & 0x7F) != 0x7F and c != 0x80])     # drop NaN and -0
    order = finite[np.argsort(vals[finite], kind="stable")]
    rank = np.full(256, -10 ** 6, np.int64)
    rank[order] = np.arange(order.size)
    rank[0x80] = rank[0x00]
    return rank


class Infer:
    def __init__(self, inp_cal, T_inf=None, seed_inf=None, y_dtype=ssg.SSG_BF16):
        """Calibrate the factors with the training block on inp_cal, prepare, run inference on x_inf."""
        self.cal = tm.Block(inp_cal)
        self.cal.fwd()
        d, f = self.cal.d, self.cal.f
        self.s = self.cal.sv("s", (f,), torch.float32).clone()
        self.sinv = self.cal.sv("sinv", (f,), torch.float32).clone()
        if T_inf is None:
            self.x = self.cal.x
        else:
            g = torch.Generator().manual_seed(seed_inf)
            self.x = gu.dev(torch.randn(T_inf, d, generator=g).to(torch.bfloat16))
        self.T = self.x.shape[0]
        self.d, self.f = d, f
        self.desc = ssg.make_desc(self.T, d, f, y_dtype=y_dtype)
        self.prep = torch.empty(ssg.ssg_infer_prepared_bytes(self.desc), dtype=torch.uint8, device=gu.DEV)
        self.work = torch.empty(ssg.ssg_infer_workspace_bytes(self.desc), dtype=torch.uint8, device=gu.DEV)
        self.y = torch.empty(self.T, d, dtype=torch.bfloat16 if y_dtype == ssg.SSG_BF16 else torch.float32, device=gu.DEV)
        ssg.ssg_infer_prepare(self.desc, self.cal.W1, self.cal.W2, self.cal.W3, self.s, self.sinv, self.prep)
        ssg.ssg_infer_fwd(self.desc, self.x, self.prep, self.y, self.work)
        torch.cuda.synchronize()
        self.v = ssg.ssg_infer_view(self.desc, self.prep, self.work)

    def pv(self, name, shape, dtype):
        return ssg.view_tensor(self.prep, self.prep.data_ptr(), getattr(self.v, name), shape, dtype)

    def wv(self, name, shape, dtype):
        return ssg.view_tensor(self.work, self.work.data_ptr(), getattr(self.v, name), shape, dtype)


def check(inf: Infer, npi, rows=None):
    T, d, f = inf.T, inf.d, inf.f
    s, sinv = gu.f32(inf.s), gu.f32(inf.sinv)
    # 1. prepared weights and their scales: bit for bit
    p = infer.prepare(npi["W1"], npi["W2"], npi["W3"], s, sinv)
    wsc = gu.f32(inf.pv("weight_scales", (8,), torch.float32))
    assert wsc[0] == p.s1 and wsc[1] == p.s2 and wsc[2] == p.s3
    assert np.array_equal(gu.u8(inf.pv("w1_q", (f, d), torch.uint8)), p.w1_q)
    assert np.array_equal(gu.u8(inf.pv("w2_q", (f, d), torch.uint8)), p.w2_q)
    assert np.array_equal(gu.u8(inf.pv("w3_q", (d, f), torch.uint8)), p.w3_q)
    # 2. Q(x): bit for bit
    x_np = synth.bf16_to_f32_numpy(inf.x.cpu())
    sel = slice(None) if rows is None else rows
    ref = infer.forward(x_np if rows is None else x_np, p) if rows is None else None
    xs = gu.f32(inf.wv("x_scale", (2,), torch.float32))
    x_q = gu.u8(inf.wv("x_q", (T, d), torch.uint8))
    from oracle import quant
    xq_ref, sx_ref, ax_ref = quant.quantize_per_tensor(x_np, fp8.E4M3)
    assert xs[0] == sx_ref and xs[1] == ax_ref and np.array_equal(x_q, xq_ref)
    # 3. the fused product and cast: fp32 accumulation decides a few codes differently from the fp64 oracle, never by
    #    more than one step
    xq_s = x_q[sel]
    u = mlp.round_f32(fp8_gemm.matmul_nt(xq_s, fp8.E4M3, p.w1_q, fp8.E4M3) / (np.float64(sx_ref) * np.float64(p.s1)))
    g = mlp.round_f32(fp8_gemm.matmul_nt(xq_s, fp8.E4M3, p.w2_q, fp8.E4M3) / (np.float64(sx_ref) * np.float64(p.s2)))
    h_ref = mlp.round_f32(oswiglu.swiglu(u.astype(np.float64), g.astype(np.float64)))
    hq_ref = fp8.satcast(h_ref, fp8.E4M3)
    h_q = gu.u8(inf.wv("h_q", (T, f), torch.uint8))[sel]
    # The kernel decides the code from fp32 inner products accumulated in the matrix core's order, which no
    # CPU program reproduces; what is unique is the value: the stored code must be a correct rounding of some
    # product within the propagated GEMM tolerance of the oracle's.  Tolerance of each inner product: 1e-4 of
    # its largest magnitude (20 times tighter than the 2e-3 bar of the GEMM tests); first-order propagation
    # through h = u * Swish(g).
    u64, g64 = u.astype(np.float64), g.astype(np.float64)
    sg = 1.0 / (1.0 + np.exp(-g64))
    tol_h = np.abs(g64 * sg) * (1e-4 * np.abs(u64).max()) + np.abs(u64 * sg * (1.0 + g64 * (1.0 - sg))) * (1e-4 * np.abs(g64).max())
    table = fp8.decode_table(fp8.E4M3).astype(np.float64)
    got = table[h_q]
    mag = np.maximum(np.abs(got), 2.0 ** -6)                       # spacing of E4M3 at `got` (subnormal floor)
    half_spacing = 2.0 ** (np.floor(np.log2(mag)) - 3) / 2
    over = np.abs(h_ref.astype(np.float64)) > 448                   # saturated: any excess maps to +-448
    err = np.abs(got - np.clip(h_ref.astype(np.float64), -448, 448))
    assert np.all(err <= half_spacing * (1 + 1e-6) + tol_h), float((err - half_spacing - tol_h).max())
    assert np.all(np.abs(got[over]) == 448)
    # and in the bulk the decisions agree outright
    rank = _rank_table()
    step = np.abs(rank[h_q] - rank[hq_ref])
    assert (step != 0).mean() < 5e-3, (step != 0).mean()
    assert (step > 1).mean() < 1e-4, (step > 1).mean()
    # 4. the last GEMM on the GPU's own h^
    y_cont = fp8_gemm.matmul_nt(h_q, fp8.E4M3, p.w3_q, fp8.E4M3) / np.float64(p.s3)
    bf = inf.y.dtype == torch.bfloat16
    gu.assert_close_gemm(gu.f32(inf.y)[sel], mlp.round_bf16(y_cont) if bf else y_cont, bf, "y (continued)")
    return p, h_ref


def test_calibrate_prepare_infer_on_the_calibration_batch():
    inp = synth.make_inputs(272, 256, 400, seed=51, aligned_channels=4)
    npi = tm._np_inputs(inp)
    inf = Infer(inp)
    p, _ = check(inf, npi)
    # end to end: the folded block tracks the training block it was calibrated on
    y_train = gu.f32(inf.cal.y)
    rel = np.linalg.norm(gu.f32(inf.y) - y_train) / np.linalg.norm(y_train)
    assert rel < 6e-2, rel
    ref = infer.forward(synth.bf16_to_f32_numpy(inf.x.cpu()), p)
    rel = np.linalg.norm(gu.f32(inf.y) - ref.Y) / np.linalg.norm(ref.Y)
    assert rel < 1e-2, rel


@pytest.mark.parametrize("T_inf,y_dtype", [(16, ssg.SSG_BF16), (528, ssg.SSG_F32)])
def test_other_batches_and_output_types(T_inf, y_dtype):
    """The prepared weights serve any number of tokens; activations beyond the calibrated range saturate."""
    inp = synth.make_inputs(256, 208, 336, seed=53)
    npi = tm._np_inputs(inp)
    inf = Infer(inp, T_inf=T_inf, seed_inf=7, y_dtype=y_dtype)
    check(inf, npi)


def test_7b_shape_on_sampled_rows():
    """Full size in the launch configuration the benchmark times; the oracle follows 24 sampled token rows."""
    cfg = synth.CONFIGS["7b_fwd"]
    inp = synth.make_inputs(cfg.T, cfg.d, cfg.f, cfg.seed, cfg.w_std, backward=False)
    npi = tm._np_inputs(inp)
    inf = Infer(inp)
    rows = np.random.default_rng(0).choice(cfg.T, 24, replace=False)
    rows.sort()
    check(inf, npi, rows=rows)
    y_train = inf.cal.y.float()
    rel = (torch.linalg.norm(inf.y.float() - y_train) / torch.linalg.norm(y_train)).item()
    assert rel < 6e-2, rel


def test_bad_arguments():
    d = ssg.make_desc(64, 64, 96, smooth=0)
    assert ssg.ssg_infer_prepared_bytes(d) == 0
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device=gu.DEV)
    with pytest.raises(ssg.SsgError):
        ssg.ssg_infer_fwd(d, buf, buf, buf, buf)
    with pytest.raises(ssg.SsgError):
        ssg.ssg_infer_prepare(ssg.make_desc(64, 64, 96), buf, buf, buf, None, buf, buf)
