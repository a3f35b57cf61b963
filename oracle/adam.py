"""Adam with both moments stored in FP8 (Section 5).  TEST INFRASTRUCTURE ONLY.

What the paper fixes: the first moment is kept in E4M3 and the second in E5M2
(Section 5.2: the second moment enters through an inverse square root, so its
smallest values matter and it needs the wider exponent range).  Everything
else below is a reading (**parity unpinned** by the paper; pinned here against
the textbook optimizer and against invariants):

  * the optimizer is Adam with bias correction and decoupled weight decay
    (weight_decay = 0 gives plain Adam);
  * each moment tensor carries one scale, chosen from the range of the *new*
    moment exactly as the per-tensor scaling of Section 2
    (scale = fl32(fmax / amax), code = satcast(fl32(value * scale)));
  * a stored moment is read back as fl32(decode(code) * fl32(1 / scale)): one
    reciprocal per tensor, one multiplication per element;
  * the parameter update uses the freshly computed binary32 moments of this
    step, before they are re-encoded; the master weights are binary32.

Every arithmetic step is one correctly rounded binary32 operation ("fl32"), in
the order written in ``step``; the bias corrections are formed in binary64 from
the step count and rounded once.  With ``quantize=False`` the moments stay in
binary32 and the function is the textbook optimizer.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import fp8, quant

F32 = np.float32


@dataclass
class State:
    """Moments of one parameter tensor.  Quantized: uint8 codes and their scales;
    unquantized (``quantize=False``): binary32 values with scales fixed at 1."""
    m: np.ndarray
    v: np.ndarray
    scale_m: np.float32
    scale_v: np.float32
    step: int


def init(n: int, quantize: bool = True) -> State:
    """Zero moments before the first step: codes 0 (the value 0) and scales 1."""
    dt = np.uint8 if quantize else np.float32
    return State(np.zeros(n, dt), np.zeros(n, dt), F32(1.0), F32(1.0), 0)


def bias_corrections(beta1: float, beta2: float, t: int):
    """c1 = 1/(1 - beta1^t), c2 = 1/(1 - beta2^t) with beta as binary32 values, formed in binary64
    and rounded once to binary32."""
    b1, b2 = float(F32(beta1)), float(F32(beta2))
    return F32(1.0 / (1.0 - b1 ** t)), F32(1.0 / (1.0 - b2 ** t))


def moments_from_state(st: State, quantize: bool = True):
    """The stored moments as binary32: fl32(decode(code) * fl32(1 / scale))."""
    if not quantize:
        return st.m.astype(F32), st.v.astype(F32)
    inv_m, inv_v = F32(F32(1.0) / F32(st.scale_m)), F32(F32(1.0) / F32(st.scale_v))
    m = (fp8.decode_table(fp8.E4M3)[st.m].astype(F32) * inv_m).astype(F32)
    v = (fp8.decode_table(fp8.E5M2)[st.v].astype(F32) * inv_v).astype(F32)
    return m, v


def step(w: np.ndarray, g: np.ndarray, st: State, lr: float, beta1: float = 0.9, beta2: float = 0.95,
         eps: float = 1e-8, weight_decay: float = 0.0, quantize: bool = True, pow2: bool = False):
    """One optimizer step on a flat tensor.  Returns (new w as binary32, new State)."""
    w = np.asarray(w, dtype=F32)
    g = np.asarray(g, dtype=F32)
    t = st.step + 1
    b1, b2 = F32(beta1), F32(beta2)
    omb1, omb2 = F32(F32(1.0) - b1), F32(F32(1.0) - b2)
    lr, eps, wd = F32(lr), F32(eps), F32(weight_decay)
    c1, c2 = bias_corrections(beta1, beta2, t)

    m_prev, v_prev = moments_from_state(st, quantize)
    with np.errstate(over="ignore", invalid="ignore", divide="ignore"):
        # exponential moving averages of the gradient and of its square
        m = ((b1 * m_prev).astype(F32) + (omb1 * g).astype(F32)).astype(F32)
        v = ((b2 * v_prev).astype(F32) + ((omb2 * g).astype(F32) * g).astype(F32)).astype(F32)
        # bias-corrected step and decoupled weight decay
        mhat = (m * c1).astype(F32)
        vhat = (v * c2).astype(F32)
        denom = (np.sqrt(vhat).astype(F32) + eps).astype(F32)
        upd = (mhat / denom).astype(F32)
        upd = (upd + (wd * w).astype(F32)).astype(F32)
        w_new = (w - (lr * upd).astype(F32)).astype(F32)

    if not quantize:
        return w_new, State(m, v, F32(1.0), F32(1.0), t)
    mq, sm, _ = quant.quantize_per_tensor(m, fp8.E4M3, pow2=pow2)
    vq, sv, _ = quant.quantize_per_tensor(v, fp8.E5M2, pow2=pow2)
    return w_new, State(mq, vq, sm, sv, t)
