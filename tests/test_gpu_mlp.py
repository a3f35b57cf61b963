"""GPU parity: the whole block, forward and backward, against the oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

import synth
from oracle import fp8, mlp, quant
from oracle import gemm as fp8_gemm

pytestmark = pytest.mark.gpu

import paper_2409_12517_amd as ssg  # noqa: E402
import gpu_util as gu  # noqa: E402


class Block:
    """Device buffers of one forward+backward call and typed views into saved/workspace."""

    def __init__(self, inp, smooth=1, y_dtype=None, dw_dtype=None, rnd=None):
        self.T, self.d = inp["x"].shape
        self.f = inp["W1"].shape[0]
        self.desc = ssg.make_desc(self.T, self.d, self.f, smooth=smooth,
                                  rnd=ssg.SSG_ROUND_EXACT_DIV if rnd is None else rnd,
                                  y_dtype=ssg.SSG_BF16 if y_dtype is None else y_dtype,
                                  dw_dtype=ssg.SSG_F32 if dw_dtype is None else dw_dtype)
        self.x, self.W1, self.W2, self.W3 = (gu.dev(inp[k]) for k in ("x", "W1", "W2", "W3"))
        self.dY = gu.dev(inp["dY"]) if inp.get("dY") is not None else None
        ydt = torch.bfloat16 if self.desc.y_dtype == ssg.SSG_BF16 else torch.float32
        wdt = torch.bfloat16 if self.desc.dw_dtype == ssg.SSG_BF16 else torch.float32
        self.y = torch.empty(self.T, self.d, dtype=ydt, device=gu.DEV)
        self.saved = torch.empty(ssg.ssg_mlp_saved_bytes(self.desc), dtype=torch.uint8, device=gu.DEV)
        self.work = torch.empty(ssg.ssg_mlp_workspace_bytes(self.desc), dtype=torch.uint8, device=gu.DEV)
        self.dx = torch.empty(self.T, self.d, dtype=ydt, device=gu.DEV)
        self.dW1 = torch.empty(self.f, self.d, dtype=wdt, device=gu.DEV)
        self.dW2 = torch.empty(self.f, self.d, dtype=wdt, device=gu.DEV)
        self.dW3 = torch.empty(self.d, self.f, dtype=wdt, device=gu.DEV)

    def fwd(self):
        ssg.ssg_mlp_fwd(self.desc, self.x, self.W1, self.W2, self.W3, self.y, self.saved)
        torch.cuda.synchronize()

    def bwd(self):
        ssg.ssg_mlp_bwd(self.desc, self.dY, self.saved, self.dx, self.dW1, self.dW2, self.dW3, self.work)
        torch.cuda.synchronize()

    def sv(self, name, shape, dtype):
        v = ssg.ssg_mlp_view_saved(self.desc, self.saved)
        return ssg.view_tensor(self.saved, self.saved.data_ptr(), getattr(v, name), shape, dtype)

    def wv(self, name, shape, dtype):
        v = ssg.ssg_mlp_view_workspace(self.desc, self.work)
        return ssg.view_tensor(self.work, self.work.data_ptr(), getattr(v, name), shape, dtype)


def _np_inputs(inp):
    return {k: synth.bf16_to_f32_numpy(v) for k, v in inp.items() if isinstance(v, torch.Tensor) and v.dtype == torch.bfloat16}


def check_forward(blk: Block, npi, smooth=1, scales=None):
    """Tiered comparison of one forward call with the oracle.  ``scales``: the per-tensor scales the call
    was given (delayed scaling); None = current scaling."""
    T, d, f = blk.T, blk.d, blk.f
    ref = mlp.forward(npi["x"], npi["W1"], npi["W2"], npi["W3"], smooth=bool(smooth), scales=scales)
    sc = gu.f32(blk.sv("scales", (8,), torch.float32))
    # tier 1: quantized inputs and their scales are bit-exact
    assert sc[0] == ref.sx and sc[1] == ref.sw1 and sc[2] == ref.sw2
    x_q = gu.u8(blk.sv("x_q", (T, d), torch.uint8))
    assert np.array_equal(x_q, ref.x_q)
    for n, r in (("w1_q", ref.w1_q), ("w2_q", ref.w2_q)):
        assert np.array_equal(gu.u8(blk.sv(n, (f, d), torch.uint8)), r)
    # tier 2: U, G (fp32 accumulation vs fp64) within the GEMM bar
    U = gu.f32(blk.sv("U", (T, f), torch.bfloat16)); G = gu.f32(blk.sv("G", (T, f), torch.bfloat16))
    gu.assert_close_gemm(U, ref.U, True, "U"); gu.assert_close_gemm(G, ref.G, True, "G")
    # tier 3: everything downstream of the GPU's own U, G is bit-exact given the GPU's fp32 h
    h = gu.empty_f32(T, f)
    ssg.ssg_swiglu(blk.sv("U", (T, f), torch.bfloat16), blk.sv("G", (T, f), torch.bfloat16), T, f, h)
    torch.cuda.synchronize()
    h_np = gu.f32(h)
    from oracle import swiglu
    h_ref = swiglu.swiglu(U, G)
    assert np.all(np.abs(h_np - h_ref) <= 6 * 2.0 ** -23 * np.abs(h_ref) + 1e-30)
    if smooth:
        a, s_ref, sinv_ref = mlp.channel_scales(h_np)
        hq_ref = quant.cast_with_scale(h_np, s_ref[None, :], fp8.E4M3)
        w3q_ref, sw3_ref, amax_w3s = mlp.fold_w3(npi["W3"], sinv_ref)
    else:
        a = np.abs(h_np).max(axis=0)
        hq_ref, sh, _ = quant.quantize_per_tensor(h_np, fp8.E4M3)
        s_ref, sinv_ref = np.full(f, sh, np.float32), np.ones(f, np.float32)
        w3q_ref, sw3_ref, amax_w3s = quant.quantize_per_tensor(npi["W3"], fp8.E4M3)
    assert np.array_equal(gu.f32(blk.sv("h_camax", (f,), torch.float32)), a)
    assert np.array_equal(gu.f32(blk.sv("s", (f,), torch.float32)), s_ref)
    assert np.array_equal(gu.f32(blk.sv("sinv", (f,), torch.float32)), sinv_ref)
    h_q = gu.u8(blk.sv("h_q", (T, f), torch.uint8))
    assert np.array_equal(h_q, hq_ref)
    assert sc[7] == amax_w3s and sc[3] == sw3_ref
    w3_q = gu.u8(blk.sv("w3_q", (d, f), torch.uint8))
    assert np.array_equal(w3_q, w3q_ref)
    # tier 4: the last GEMM on identical inputs -- the oracle continued from the GPU's own (verified) operands
    y_cont = fp8_gemm.matmul_nt(h_q, fp8.E4M3, w3_q, fp8.E4M3) / (float(sw3_ref) * (1.0 if smooth else float(s_ref[0])))
    bf_y = blk.desc.y_dtype == ssg.SSG_BF16
    gu.assert_close_gemm(gu.f32(blk.y), mlp.round_bf16(y_cont) if bf_y else y_cont, bf_y, "Y (continued)")
    # tier 5: end to end against the oracle.  A bf16 rounding of U or G that differs (fp32 vs fp64
    # accumulation) can move a channel's maximum, hence its factor and many of its FP8 codes, so the
    # two outputs differ by FP8 decision noise, not by the GEMM bar; bound it normwise.
    rel = np.linalg.norm(gu.f32(blk.y) - ref.Y) / np.linalg.norm(ref.Y)
    assert rel < 1e-2, rel
    if smooth:
        assert np.all(np.abs(s_ref / ref.s - 1) < 2.0 ** -5)
    # the oracle's forward state rebuilt from the GPU's stored tensors, for the backward checks
    fw_gpu = mlp.Forward(quantized=True, smooth=bool(smooth), x_q=x_q, sx=np.float32(sc[0]),
                         w1_q=gu.u8(blk.sv("w1_q", (f, d), torch.uint8)), sw1=np.float32(sc[1]),
                         w2_q=gu.u8(blk.sv("w2_q", (f, d), torch.uint8)), sw2=np.float32(sc[2]),
                         w3_q=w3_q, sw3=np.float32(sw3_ref), h_q=h_q, sh=np.float32(s_ref[0]),
                         U=U.astype(np.float64), G=G.astype(np.float64), h=h_np, a=a, s=s_ref, sinv=sinv_ref)
    return ref, fw_gpu


def check_backward(blk: Block, npi, ref_fw, fw_gpu, smooth=1, scales=None):
    T, d, f = blk.T, blk.d, blk.f
    delayed = scales is not None
    bf_y = blk.desc.y_dtype == ssg.SSG_BF16
    bf_w = blk.desc.dw_dtype == ssg.SSG_BF16
    ydt, wdt = ("bf16" if bf_y else "f32"), ("bf16" if bf_w else "f32")
    # stage 1: upstream gradient, bit-exact
    cont = mlp.backward(fw_gpu, npi["dY"], dx_dtype=ydt, dw_dtype=wdt, scales=scales)
    wsc = gu.f32(blk.wv("scales", (8,), torch.float32))
    dy_q = gu.u8(blk.wv("dy_q", (T, d), torch.uint8))
    assert wsc[0] == cont.sdy and np.array_equal(dy_q, cont.dy_q)
    assert delayed or wsc[3] == quant.amax(npi["dY"])
    if delayed:
        # Under delayed scaling the dH epilogue emits the E5M2 codes of dU, dG directly (no bf16 tensors exist).
        # The code is decided from fp32 values accumulated in the matrix core's order, so what is checked is the
        # value: decode(code) / scale must be a correct E5M2 rounding (half an ulp = 2^-3 relative; half the
        # smallest subnormal absolute; clipped at the format maximum) of a value within the GEMM bar of the
        # oracle's bf16 dU, dG -- and the outright decisions must agree almost everywhere.
        table = fp8.decode_table(fp8.E5M2).astype(np.float64)
        codes = {}
        for nm, ref_v, ref_q, sc_given in (("du_q", cont.dU, cont.du_q, float(scales["du"])), ("dg_q", cont.dG, cont.dg_q, float(scales["dg"]))):
            q = gu.u8(blk.wv(nm, (T, f), torch.uint8))
            codes[nm] = q
            got = table[q] / sc_given
            lim = 57344.0 / sc_given
            want = np.clip(ref_v, -lim, lim)
            tol = 2e-3 * np.abs(ref_v).max() + gu.bf16_ulp(ref_v) + 2.0 ** -3 * np.abs(want) * (1 + 1e-6) + 2.0 ** -17 / sc_given
            assert np.all(np.abs(got - want) <= tol), nm
            assert (q != ref_q).mean() < 2e-2, (nm, (q != ref_q).mean())
        assert wsc[1] == np.float32(scales["du"]) and wsc[2] == np.float32(scales["dg"])
        cont2 = mlp.backward(fw_gpu, npi["dY"], dx_dtype=ydt, dw_dtype=wdt, scales=scales,
                             stored_codes=(codes["du_q"], codes["dg_q"]))
    else:
        # stage 2: dU, dG on identical inputs (one GEMM plus the SwiGLU derivative)
        dU = gu.f32(blk.wv("dU", (T, f), torch.bfloat16)); dG = gu.f32(blk.wv("dG", (T, f), torch.bfloat16))
        gu.assert_close_gemm(dU, cont.dU, True, "dU"); gu.assert_close_gemm(dG, cont.dG, True, "dG")
        # stage 3: quantization of the GPU's own dU, dG, bit-exact
        cont2 = mlp.backward(fw_gpu, npi["dY"], dx_dtype=ydt, dw_dtype=wdt, stored_dU_dG=(dU, dG), scales=scales)
        assert wsc[1] == cont2.sdu and wsc[2] == cont2.sdg
        assert wsc[4] == quant.amax(dU) and wsc[5] == quant.amax(dG)
        assert np.array_equal(gu.u8(blk.wv("du_q", (T, f), torch.uint8)), cont2.du_q)
        assert np.array_equal(gu.u8(blk.wv("dg_q", (T, f), torch.uint8)), cont2.dg_q)
    # stage 4: the four gradient GEMMs on identical inputs
    gu.assert_close_gemm(gu.f32(blk.dx), cont2.dX, bf_y, "dX")
    gu.assert_close_gemm(gu.f32(blk.dW1), cont2.dW1, bf_w, "dW1")
    gu.assert_close_gemm(gu.f32(blk.dW2), cont2.dW2, bf_w, "dW2")
    gu.assert_close_gemm(gu.f32(blk.dW3), cont2.dW3, bf_w, "dW3")
    # stage 5: end to end against the oracle, normwise (FP8 decision noise, see check_forward)
    ref = mlp.backward(ref_fw, npi["dY"], dx_dtype=ydt, dw_dtype=wdt, scales=scales)
    for name, got in (("dX", blk.dx), ("dW1", blk.dW1), ("dW2", blk.dW2), ("dW3", blk.dW3)):
        r = getattr(ref, name)
        rel = np.linalg.norm(gu.f32(got) - r) / np.linalg.norm(r)
        assert rel < 2e-2, (name, rel)
    return ref, cont2


@pytest.mark.parametrize("smooth", [1, 0])
def test_tiny_config_forward_backward(smooth):
    inp = synth.make_config("tiny")
    npi = _np_inputs(inp)
    blk = Block(inp, smooth=smooth)
    blk.fwd()
    ref_fw, g = check_forward(blk, npi, smooth)
    blk.bwd()
    check_backward(blk, npi, ref_fw, g, smooth)


@pytest.mark.parametrize("T,d,f,aligned", [(528, 400, 1040, 0), (1024, 512, 1536, 6), (16, 16, 16, 0)])
def test_ragged_shapes_and_outlier_channels(T, d, f, aligned):
    inp = synth.make_inputs(T, d, f, seed=T + d + f, aligned_channels=aligned)
    npi = _np_inputs(inp)
    blk = Block(inp)
    blk.fwd()
    ref_fw, g = check_forward(blk, npi)
    blk.bwd()
    check_backward(blk, npi, ref_fw, g)


def test_fp32_outputs_bf16_weight_grads_and_pow2_scales():
    inp = synth.make_inputs(256, 256, 512, seed=21)
    npi = _np_inputs(inp)
    blk = Block(inp, y_dtype=ssg.SSG_F32, dw_dtype=ssg.SSG_BF16)
    blk.fwd(); blk.bwd()
    ref_fw, fw_gpu = check_forward(blk, npi)
    check_backward(blk, npi, ref_fw, fw_gpu)
    blk2 = Block(inp, rnd=ssg.SSG_ROUND_POW2)
    blk2.fwd()
    sc = gu.f32(blk2.sv("scales", (8,), torch.float32))
    assert sc[0] == quant.scale_from_amax(quant.amax(npi["x"]), fp8.E4M3, pow2=True)
    assert np.array_equal(gu.u8(blk2.sv("x_q", (256, 256), torch.uint8)),
                          quant.quantize_per_tensor(npi["x"], fp8.E4M3, pow2=True)[0])


def test_two_calls_give_identical_bytes():
    """Atomic maxima are order independent, so the block is deterministic run to run."""
    inp = synth.make_inputs(512, 256, 688, seed=31)
    blk = Block(inp)
    blk.fwd(); blk.bwd()
    first = [t.clone() for t in (blk.y, blk.dx, blk.dW1, blk.dW2, blk.dW3, blk.saved)]
    blk.fwd(); blk.bwd()
    torch.cuda.synchronize()
    for a, b in zip(first, (blk.y, blk.dx, blk.dW1, blk.dW2, blk.dW3, blk.saved)):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))


def test_cached_weights_give_the_same_bytes():
    """weights_cached = 1 reuses Q(w1), Q(w2), their scales and W3's per-channel ranges from an earlier
    call on the same `saved` buffer; every output must equal a call that re-quantizes the weights."""
    inp = synth.make_inputs(512, 256, 688, seed=41)
    other = synth.make_inputs(512, 256, 688, seed=42)
    blk = Block(inp)
    blk.fwd()                                            # fills the weight part of `saved`
    blk.x, blk.dY = gu.dev(other["x"]), gu.dev(other["dY"])   # a new micro-batch, same weights
    blk.desc.weights_cached = 1
    blk.fwd(); blk.bwd()
    ref = Block(dict(inp, x=other["x"], dY=other["dY"]))
    ref.fwd(); ref.bwd()
    for a, b in ((blk.y, ref.y), (blk.dx, ref.dx), (blk.dW1, ref.dW1), (blk.dW2, ref.dW2), (blk.dW3, ref.dW3)):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
    T, d, f = blk.T, blk.d, blk.f
    regions = [("scales", (8,), torch.float32), ("s", (f,), torch.float32), ("sinv", (f,), torch.float32),
               ("h_camax", (f,), torch.float32), ("w3_camax", (f,), torch.float32), ("x_q", (T, d), torch.uint8),
               ("w1_q", (f, d), torch.uint8), ("w2_q", (f, d), torch.uint8), ("h_q", (T, f), torch.uint8),
               ("w3_q", (d, f), torch.uint8), ("U", (T, f), torch.bfloat16), ("G", (T, f), torch.bfloat16)]
    for name, shape, dt in regions:
        assert torch.equal(blk.sv(name, shape, dt).view(torch.uint8), ref.sv(name, shape, dt).view(torch.uint8)), name


def test_graph_capture_replays_match_eager():
    """The whole step is capturable (kernel launches only, no memset nodes, nothing allocated): three replays,
    with eager work and synchronisations in between, give the bytes of the eager call every time."""
    inp = synth.make_inputs(528, 256, 688, seed=61)
    blk = Block(inp)
    blk.fwd(); blk.bwd()
    want = [t.clone() for t in (blk.y, blk.dx, blk.dW1, blk.dW2, blk.dW3)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                     # warm-up on the side stream, as capture requires
        ssg.ssg_mlp_fwd(blk.desc, blk.x, blk.W1, blk.W2, blk.W3, blk.y, blk.saved)
        ssg.ssg_mlp_bwd(blk.desc, blk.dY, blk.saved, blk.dx, blk.dW1, blk.dW2, blk.dW3, blk.work)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ssg.ssg_mlp_fwd(blk.desc, blk.x, blk.W1, blk.W2, blk.W3, blk.y, blk.saved)
        ssg.ssg_mlp_bwd(blk.desc, blk.dY, blk.saved, blk.dx, blk.dW1, blk.dW2, blk.dW3, blk.work)
    for _ in range(3):
        for t in (blk.y, blk.dx, blk.dW1, blk.dW2, blk.dW3):
            t.zero_()                                  # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(want, (blk.y, blk.dx, blk.dW1, blk.dW2, blk.dW3)):
            assert torch.equal(a, b)
