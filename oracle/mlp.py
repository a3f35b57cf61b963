"""The SwiGLU MLP block with FP8 quantization, forward and backward.

Notation follows the paper (Sections 4.1, 4.4): for token t and channel i

    U_ti = x_t . w1_i          (linear branch)
    G_ti = x_t . w2_i          (branch that goes through Swish)
    h_ti = U_ti * G_ti * sigma(G_ti)
    y_t  = sum_i w3_i * h_ti   (last linear layer)

Storage: x [T,d]; W1, W2 [f,d] (row i = w1_i, w2_i); W3 [d,f] (column i = w3_i).

Quantized forms:
  * plain (Figure 4a):   y = sum_i Q(w3)_i * Q(h)_i, every Q per tensor.
  * Smooth-SwiGLU (Figure 4b, Eq. 2): channel i of h is multiplied by its own
    s_i before the cast and the inverse is folded into w3 before *its*
    quantization, w3~_i = Q(s_i^-1 * w3_i) (the display after Eq. 2).

Comparison variant (Section 4.3, Table 3 "FP8 + SwiGLU output in BF16"): the quantization of the last linear
layer is disabled -- the SwiGLU output stays in bf16 and that layer, with its two gradient contractions, runs on
bf16 operands; everything else is FP8 as above (``w3_layer_fp8=False``).

Readings where the paper is silent (all "parity unpinned" by the paper):
  * s_i = fl32(448 / a_i) with a_i = max_t |h_ti| (largest absolute value over
    all tokens of the call), s_i^-1 = fl32(a_i / 448), both 1 when a_i = 0;
    the Q that follows s_i is then a bare cast.
  * h is formed from U and G after they were rounded to bf16 (the stored
    activations), in float64, and rounded once to binary32.
  * Backward uses the straight-through estimator: each Q is the identity for
    gradients and s_i is a constant.  Gradient operands are E5M2, saved
    activations and weights stay E4M3 (Section 6.2).  dU and dG are rounded to
    bf16 and then quantized per tensor with separate scales.
  * Outputs y, dx are bf16; weight gradients are binary32.
  * With the last layer left in bf16: h is rounded once to bf16 (from the binary32 product), W3 and dY are used as
    the bf16 tensors they are, no scales are involved; the rest of the backward pass (E5M2 dU, dG; dX, dW1, dW2 in
    FP8) is unchanged.

Between the named rounding points everything is float64.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

from . import fp8, gemm, quant, swiglu


def round_bf16(v: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bf16 value (8 significant bits,
    ties to even, exponent range of binary32); result stays float64."""
    v = np.asarray(v, dtype=np.float64)
    m, e = np.frexp(v)                       # v = m * 2^e, 0.5 <= |m| < 1
    e = np.maximum(e, -125)                  # below 2^-126 the spacing stops shrinking
    m = v / np.ldexp(1.0, e)
    q = np.rint(m * 256.0)                   # rint rounds half to even
    out = np.ldexp(q, e - 8)
    bf16_max = (2.0 - 2.0 ** -7) * 2.0 ** 127
    return np.where(np.abs(out) > bf16_max, np.copysign(np.inf, out), out)


def round_f32(v: np.ndarray) -> np.ndarray:
    return np.asarray(v, dtype=np.float64).astype(np.float32)


def _round_out(v: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_bf16(v)
    if dtype == "f32":
        return round_f32(v).astype(np.float64)
    if dtype == "f64":
        return np.asarray(v, dtype=np.float64)
    raise ValueError(dtype)


def channel_scales(h: np.ndarray):
    """Per-channel maxima and the Smooth-SwiGLU factors (Section 4.4, the
    three-step recipe: one chunk per channel, its largest magnitude, its s_i)."""
    a = np.abs(np.asarray(h, dtype=np.float32)).max(axis=0).astype(np.float32) if h.shape[0] else \
        np.zeros(h.shape[1], np.float32)
    s = quant.scale_from_amax(a, fp8.E4M3)
    fmax = np.float32(fp8.max_finite(fp8.E4M3))
    sinv = np.where(a > 0, a / fmax, np.float32(1.0)).astype(np.float32)
    return a, s, sinv


@dataclass
class Forward:
    quantized: bool
    smooth: bool
    w3_layer_fp8: bool = True                # False: the last linear layer runs on bf16 operands (Section 4.3)
    h_b: Optional[np.ndarray] = None         # bf16-valued SwiGLU output of that variant
    # quantized operands and their scales (None when quantized=False)
    x_q: Optional[np.ndarray] = None
    sx: Optional[np.float32] = None
    w1_q: Optional[np.ndarray] = None
    sw1: Optional[np.float32] = None
    w2_q: Optional[np.ndarray] = None
    sw2: Optional[np.float32] = None
    w3_q: Optional[np.ndarray] = None
    sw3: Optional[np.float32] = None
    h_q: Optional[np.ndarray] = None
    sh: Optional[np.float32] = None          # plain mode: per-tensor scale of h
    # activations
    U: np.ndarray = field(default=None)      # float64 array holding bf16 values (quantized) or exact
    G: np.ndarray = field(default=None)
    h: np.ndarray = field(default=None)      # float32 (quantized) / float64
    a: Optional[np.ndarray] = None           # per-channel max |h|
    s: Optional[np.ndarray] = None           # per-channel factor
    sinv: Optional[np.ndarray] = None
    Y: np.ndarray = field(default=None)
    # unquantized inputs kept for the unquantized backward
    x: Optional[np.ndarray] = None
    W1: Optional[np.ndarray] = None
    W2: Optional[np.ndarray] = None
    W3: Optional[np.ndarray] = None
    amax: Optional[dict] = None              # ranges of x, w1, w2 seen in this call (for an amax history)


def fold_w3(W3: np.ndarray, sinv: np.ndarray):
    """w3~ = Q(s^-1 * w3): scale column i of W3 [d,f] by sinv_i in binary32,
    then quantize the result per tensor to E4M3."""
    W3s = (np.asarray(W3, np.float32) * np.asarray(sinv, np.float32)[None, :]).astype(np.float32)
    return quant.quantize_per_tensor(W3s, fp8.E4M3)


def forward(x, W1, W2, W3, *, quantized: bool = True, smooth: bool = True,
            y_dtype: str = "bf16", h_scale=None, scales=None, w3_layer_fp8: bool = True) -> Forward:
    """One forward pass of the block.  x, W1, W2, W3 are float arrays holding
    the (bf16-representable) inputs.  ``h_scale`` (plain mode only) is a
    caller-given per-tensor scale for h, as under delayed scaling.  ``scales``
    may give the per-tensor scales of "x", "w1", "w2" (delayed scaling,
    Section 2: the scale comes from earlier iterations; values beyond the range
    it allows saturate); the ranges seen in this call are returned in ``amax``.  ``w3_layer_fp8=False`` leaves
    the last linear layer unquantized (bf16 SwiGLU output times bf16 W3), the comparison variant of Section 4.3."""
    x = np.asarray(x); W1 = np.asarray(W1); W2 = np.asarray(W2); W3 = np.asarray(W3)
    out = Forward(quantized=quantized, smooth=smooth, w3_layer_fp8=w3_layer_fp8)

    if not quantized:
        # Q := identity, no rounding points: the real-valued function.
        x64, W164, W264, W364 = (np.asarray(v, np.float64) for v in (x, W1, W2, W3))
        out.x, out.W1, out.W2, out.W3 = x64, W164, W264, W364
        out.U = x64 @ W164.T
        out.G = x64 @ W264.T
        out.h = swiglu.swiglu(out.U, out.G)
        if smooth:
            a = np.abs(out.h).max(axis=0)
            out.a = a
            out.s = np.where(a > 0, 448.0 / np.where(a > 0, a, 1.0), 1.0)
            out.sinv = np.where(a > 0, a / 448.0, 1.0)
            out.Y = (out.h * out.s[None, :]) @ (W364 * out.sinv[None, :]).T
        else:
            out.Y = out.h @ W364.T
        return out

    # 1. per-tensor E4M3 of the input and of the first two weight matrices
    given = scales or {}
    out.amax = {}
    out.x_q, out.sx, out.amax["x"] = quant.quantize_per_tensor(x, fp8.E4M3, scale=given.get("x"))
    out.w1_q, out.sw1, out.amax["w1"] = quant.quantize_per_tensor(W1, fp8.E4M3, scale=given.get("w1"))
    out.w2_q, out.sw2, out.amax["w2"] = quant.quantize_per_tensor(W2, fp8.E4M3, scale=given.get("w2"))
    # 2. the two inner products of Eq. 2, dequantized, stored as bf16
    out.U = round_bf16(gemm.matmul_nt(out.x_q, fp8.E4M3, out.w1_q, fp8.E4M3)
                       / (np.float64(out.sx) * np.float64(out.sw1)))
    out.G = round_bf16(gemm.matmul_nt(out.x_q, fp8.E4M3, out.w2_q, fp8.E4M3)
                       / (np.float64(out.sx) * np.float64(out.sw2)))
    # 3. SwiGLU product, one rounding to binary32
    out.h = round_f32(swiglu.swiglu(out.U, out.G))

    if not w3_layer_fp8:
        # Section 4.3: the SwiGLU output is not quantized; the last linear layer sees bf16 operands
        out.h_b = round_bf16(out.h)
        out.W3 = np.asarray(W3, np.float64)
        out.Y = _round_out(out.h_b @ out.W3.T, y_dtype)
        return out

    if smooth:
        # 4. per-channel factor and cast
        out.a, out.s, out.sinv = channel_scales(out.h)
        out.h_q = quant.cast_with_scale(out.h, out.s[None, :], fp8.E4M3)
        # 5. inverse factor folded into w3 before its quantization
        out.w3_q, out.sw3, _ = fold_w3(W3, out.sinv)
        # 6. last linear layer; only the per-tensor scale of w3~ is left to undo
        acc = gemm.matmul_nt(out.h_q, fp8.E4M3, out.w3_q, fp8.E4M3)
        out.Y = _round_out(acc / np.float64(out.sw3), y_dtype)
    else:
        out.h_q, out.sh, _ = quant.quantize_per_tensor(out.h, fp8.E4M3, scale=h_scale)
        out.w3_q, out.sw3, _ = quant.quantize_per_tensor(W3, fp8.E4M3)
        acc = gemm.matmul_nt(out.h_q, fp8.E4M3, out.w3_q, fp8.E4M3)
        out.Y = _round_out(acc / (np.float64(out.sh) * np.float64(out.sw3)), y_dtype)
    return out


@dataclass
class Backward:
    dy_q: Optional[np.ndarray] = None
    sdy: Optional[np.float32] = None
    dY: Optional[np.ndarray] = None          # the bf16 upstream gradient as used when the last layer is left in bf16
    dH: np.ndarray = field(default=None)
    dU: np.ndarray = field(default=None)     # bf16 values in quantized mode
    dG: np.ndarray = field(default=None)
    du_q: Optional[np.ndarray] = None
    sdu: Optional[np.float32] = None
    dg_q: Optional[np.ndarray] = None
    sdg: Optional[np.float32] = None
    dX: np.ndarray = field(default=None)
    dW1: np.ndarray = field(default=None)
    dW2: np.ndarray = field(default=None)
    dW3: np.ndarray = field(default=None)
    amax: Optional[dict] = None              # ranges of dy, du, dg seen in this call


def backward_grad_h(fw: Forward, dY, *, scales=None) -> Backward:
    """Steps 7-9 of the quantized backward pass: the upstream gradient to E5M2, the gradient at h (one
    contraction over the model dimension, times the channel factor), and through the SwiGLU product to
    bf16 dU, dG.  ``scales`` may give the per-tensor scale of "dy" (delayed scaling)."""
    bw = Backward()
    given = scales or {}
    bw.amax = {}
    if not fw.w3_layer_fp8:
        # last layer in bf16 (Section 4.3): its input gradient from the bf16 dY and W3, no quantization
        bw.dY = np.asarray(dY, np.float64)
        bw.dH = bw.dY @ fw.W3
        dU, dG = swiglu.swiglu_grads(fw.U, fw.G, bw.dH)
        bw.dU, bw.dG = round_bf16(dU), round_bf16(dG)
        return bw
    # 7. upstream gradient to E5M2
    bw.dy_q, bw.sdy, bw.amax["dy"] = quant.quantize_per_tensor(dY, fp8.E5M2, scale=given.get("dy"))
    sdy, sw3 = np.float64(bw.sdy), np.float64(fw.sw3)
    # 8. gradient at h: contract dY^ with w3~ over the model dimension
    #    (w3_q is [d,f]; its transpose [f,d] has the contraction index last)
    acc = gemm.matmul_nt(bw.dy_q, fp8.E5M2, np.ascontiguousarray(fw.w3_q.T), fp8.E4M3)
    if fw.smooth:
        bw.dH = acc / (sdy * sw3) * fw.s.astype(np.float64)[None, :]
    else:
        bw.dH = acc / (sdy * sw3)
    # 9. through the SwiGLU product, from the stored bf16 U and G
    dU, dG = swiglu.swiglu_grads(fw.U, fw.G, bw.dH)
    bw.dU, bw.dG = round_bf16(dU), round_bf16(dG)
    return bw


def backward_operand_grads(fw: Forward, bw: Backward, *, dx_dtype: str = "bf16", dw_dtype: str = "f32",
                           scales=None) -> Backward:
    """Steps 10-12: quantize the bf16 dU, dG held in ``bw`` (two tensors, two E5M2 scales; ``scales`` may
    give "du", "dg"), then the input gradient and the three weight gradients.  Fills and returns ``bw``."""
    given = scales or {}
    # 10. two tensors, two E5M2 scales
    bw.du_q, bw.sdu, bw.amax["du"] = quant.quantize_per_tensor(bw.dU, fp8.E5M2, scale=given.get("du"))
    bw.dg_q, bw.sdg, bw.amax["dg"] = quant.quantize_per_tensor(bw.dG, fp8.E5M2, scale=given.get("dg"))
    sdu, sdg = np.float64(bw.sdu), np.float64(bw.sdg)
    sx, sw1, sw2 = np.float64(fw.sx), np.float64(fw.sw1), np.float64(fw.sw2)
    # 11. input gradient: two contractions over the channel index
    dX = gemm.matmul_nt(bw.du_q, fp8.E5M2, np.ascontiguousarray(fw.w1_q.T), fp8.E4M3) / (sdu * sw1) \
        + gemm.matmul_nt(bw.dg_q, fp8.E5M2, np.ascontiguousarray(fw.w2_q.T), fp8.E4M3) / (sdg * sw2)
    bw.dX = _round_out(dX, dx_dtype)
    # 12. weight gradients: contractions over the token index
    xT = np.ascontiguousarray(fw.x_q.T)
    bw.dW1 = _round_out(gemm.matmul_nt(np.ascontiguousarray(bw.du_q.T), fp8.E5M2, xT, fp8.E4M3)
                        / (sdu * sx), dw_dtype)
    bw.dW2 = _round_out(gemm.matmul_nt(np.ascontiguousarray(bw.dg_q.T), fp8.E5M2, xT, fp8.E4M3)
                        / (sdg * sx), dw_dtype)
    if not fw.w3_layer_fp8:
        bw.dW3 = _round_out(bw.dY.T @ fw.h_b, dw_dtype)                    # bf16 operands (Section 4.3)
        return bw
    sdy = np.float64(bw.sdy)
    acc3 = gemm.matmul_nt(np.ascontiguousarray(bw.dy_q.T), fp8.E5M2,
                          np.ascontiguousarray(fw.h_q.T), fp8.E4M3)        # [d,f]
    if fw.smooth:
        bw.dW3 = _round_out(acc3 / sdy * fw.sinv.astype(np.float64)[None, :], dw_dtype)
    else:
        bw.dW3 = _round_out(acc3 / (sdy * np.float64(fw.sh)), dw_dtype)
    return bw


def backward(fw: Forward, dY, *, dx_dtype: str = "bf16", dw_dtype: str = "f32", scales=None) -> Backward:
    """Gradients of sum(Y * dY) with respect to x, W1, W2, W3.

    ``scales`` may give the per-tensor scales of "dy", "du", "dg" (delayed scaling).  The quantized pass
    is the two halves above run one after the other."""
    if not fw.quantized:
        bw = Backward()
        bw.amax = {}
        dY64 = np.asarray(dY, np.float64)
        if fw.smooth:
            # Y = (h*s) @ (W3*sinv)^T with s constant
            bw.dH = (dY64 @ (fw.W3 * fw.sinv[None, :])) * fw.s[None, :]
            bw.dW3 = (dY64.T @ (fw.h * fw.s[None, :])) * fw.sinv[None, :]
        else:
            bw.dH = dY64 @ fw.W3
            bw.dW3 = dY64.T @ fw.h
        bw.dU, bw.dG = swiglu.swiglu_grads(fw.U, fw.G, bw.dH)
        bw.dX = bw.dU @ fw.W1 + bw.dG @ fw.W2
        bw.dW1 = bw.dU.T @ fw.x
        bw.dW2 = bw.dG.T @ fw.x
        return bw
    bw = backward_grad_h(fw, dY, scales=scales)
    return backward_operand_grads(fw, bw, dx_dtype=dx_dtype, dw_dtype=dw_dtype, scales=scales)
