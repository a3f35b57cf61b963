"""Inference with the Smooth-SwiGLU factors folded into the weights.  TEST INFRASTRUCTURE ONLY.

The last paragraph of Section 4.4: with the per-channel factors s_i fixed (calibrated beforehand),
the scalar is absorbed once into the weights,

    w1~_i = Q(s_i * w1_i)        w3~_i = Q(s_i^-1 * w3_i)

so that the forward pass does no per-channel work at all: the first layer already produces
s_i * u_i, the SwiGLU product s_i * h_i is cast to E4M3 as it stands, and the last layer undoes the
factor through w3~.  Readings (**parity unpinned** by the paper): s and s^-1 are the two binary32
vectors a calibration forward of the training block produced (s_i = fl32(448 / a_i),
s_i^-1 = fl32(a_i / 448)); every Q is the per-tensor E4M3 quantization of Section 2; the product
is formed from the dequantized binary32 inner products (nothing is rounded to bf16 in between,
since nothing is stored for a backward pass).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import fp8, gemm, mlp, quant, swiglu

F32 = np.float32


@dataclass
class Prepared:
    w1_q: np.ndarray      # [f, d] codes of Q(s_i * w1_i)
    s1: np.float32
    w2_q: np.ndarray      # [f, d] codes of Q(w2)
    s2: np.float32
    w3_q: np.ndarray      # [d, f] codes of Q(s_i^-1 * w3_i)
    s3: np.float32


def prepare(W1, W2, W3, s, sinv) -> Prepared:
    """Fold the factors into w1 (row i of [f,d] times s_i) and w3 (column i of [d,f] times s_i^-1),
    one binary32 multiplication per element, then quantize each matrix per tensor."""
    W1s = (np.asarray(W1, F32) * np.asarray(s, F32)[:, None]).astype(F32)
    w1_q, s1, _ = quant.quantize_per_tensor(W1s, fp8.E4M3)
    w2_q, s2, _ = quant.quantize_per_tensor(W2, fp8.E4M3)
    w3_q, s3, _ = mlp.fold_w3(W3, sinv)
    return Prepared(w1_q, s1, w2_q, s2, w3_q, s3)


@dataclass
class Forward:
    x_q: np.ndarray
    sx: np.float32
    h: np.ndarray         # binary32: (s_i u_i) * Swish(g_i)
    h_q: np.ndarray
    Y: np.ndarray


def forward(x, p: Prepared, y_dtype: str = "bf16", x_scale=None) -> Forward:
    x_q, sx, _ = quant.quantize_per_tensor(x, fp8.E4M3, scale=x_scale)
    u = mlp.round_f32(gemm.matmul_nt(x_q, fp8.E4M3, p.w1_q, fp8.E4M3) / (np.float64(sx) * np.float64(p.s1)))
    g = mlp.round_f32(gemm.matmul_nt(x_q, fp8.E4M3, p.w2_q, fp8.E4M3) / (np.float64(sx) * np.float64(p.s2)))
    h = mlp.round_f32(swiglu.swiglu(u.astype(np.float64), g.astype(np.float64)))
    h_q = fp8.satcast(h, fp8.E4M3)                       # a bare cast: the factor is already inside u
    acc = gemm.matmul_nt(h_q, fp8.E4M3, p.w3_q, fp8.E4M3)
    return Forward(x_q, sx, h, h_q, mlp._round_out(acc / np.float64(p.s3), y_dtype))


def forward_unquantized(x, W1, W2, W3, s, sinv) -> np.ndarray:
    """The same function with Q := identity, in binary64: must equal the plain block."""
    x, W1, W2, W3 = (np.asarray(v, np.float64) for v in (x, W1, W2, W3))
    s, sinv = np.asarray(s, np.float64), np.asarray(sinv, np.float64)
    u = x @ (W1 * s[:, None]).T
    g = x @ W2.T
    return swiglu.swiglu(u, g) @ (W3 * sinv[None, :]).T
