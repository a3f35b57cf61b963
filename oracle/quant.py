"""Scale selection and the quantization function Q of the paper.

Per-tensor scaling (Section 2) multiplies a tensor by one factor chosen from
its range so that it fills the FP8 format; Q (Eq. 2, Section 4.4) is that
scaling followed by the FP8 cast.  The paper prints no formula, so the reading
used throughout (unpinned by the paper) is

    amax  = max |v|                         (NaN ignored)
    scale = fl32(fmax / amax)               one IEEE binary32 division, margin 0
            1                               when amax == 0
            largest finite binary32         when the division overflows
    code  = satcast(fl32(v * scale))        one binary32 multiply, then the cast

"fl32" is a single correctly rounded binary32 operation.  With "given" scaling
the caller supplies the scale (this is how delayed scaling, which the paper
trained with, reaches the block: the scale comes from earlier iterations).

The optional power-of-two rounding replaces scale by 2^floor(log2(scale)), which
makes v*scale exact.
"""
from __future__ import annotations

import numpy as np

from . import fp8

F32_MAX = np.float32(np.finfo(np.float32).max)


def amax(v: np.ndarray) -> np.float32:
    """Largest absolute value, as binary32 (exact: no rounding is involved)."""
    v = np.asarray(v, dtype=np.float32)
    if v.size == 0:
        return np.float32(0.0)
    a = np.abs(v)
    a = np.where(np.isnan(a), np.float32(0.0), a)
    return np.float32(a.max())


def scale_from_amax(a, fmt: fp8.Format, pow2: bool = False) -> np.ndarray:
    """fl32(fmax / amax) with the two guards; works on scalars and vectors."""
    a = np.asarray(a, dtype=np.float32)
    fmax = np.float32(fp8.max_finite(fmt))
    with np.errstate(divide="ignore", over="ignore"):
        s = np.where(a > 0, fmax / np.where(a > 0, a, np.float32(1.0)), np.float32(1.0)).astype(np.float32)
    s = np.minimum(s, F32_MAX).astype(np.float32)
    if pow2:
        # 2^floor(log2 s): frexp gives s = m * 2^e with m in [0.5, 1)
        _, e = np.frexp(s)
        s = np.ldexp(np.float32(1.0), e - 1).astype(np.float32)
    return s


def cast_with_scale(v: np.ndarray, scale, fmt: fp8.Format) -> np.ndarray:
    """satcast(fl32(v * scale)); scale broadcasts (scalar or per-channel row)."""
    v = np.asarray(v, dtype=np.float32)
    with np.errstate(over="ignore", invalid="ignore"):
        scaled = (v * np.asarray(scale, dtype=np.float32)).astype(np.float32)
    return fp8.satcast(scaled, fmt)


def quantize_per_tensor(v: np.ndarray, fmt: fp8.Format, scale=None, pow2: bool = False):
    """Q for one tensor.  Returns (codes uint8, scale float32, amax float32)."""
    v = np.asarray(v, dtype=np.float32)
    a = amax(v)
    if scale is None:
        scale = scale_from_amax(a, fmt, pow2)
    scale = np.float32(scale)
    return cast_with_scale(v, scale, fmt), scale, a


def count_saturated(v: np.ndarray, scale, fmt: fp8.Format) -> int:
    """Number of elements that overflow the format under this scale (Section 3):
    the scaled magnitude lies beyond the rounding interval of the largest
    finite value, i.e. above fmax plus half the spacing of the top binade, so
    that only the clamp keeps it finite.  (A scaled maximum that lands a few
    binary32 ulps above fmax rounds to fmax on its own and is not counted.)"""
    v = np.asarray(v, dtype=np.float32)
    fmax = fp8.max_finite(fmt)
    half_spacing = 2.0 ** (int(np.floor(np.log2(fmax))) - fmt.man_bits - 1)
    with np.errstate(over="ignore", invalid="ignore"):
        scaled = np.abs((v * np.asarray(scale, dtype=np.float32)).astype(np.float32))
    return int(np.count_nonzero(scaled > np.float32(fmax + half_spacing)))


def count_flushed(v: np.ndarray, codes: np.ndarray) -> int:
    """Number of nonzero inputs whose code is +-0 (underflow, Section 3)."""
    v = np.asarray(v, dtype=np.float32)
    return int(np.count_nonzero((v != 0) & ((np.asarray(codes) & 0x7F) == 0)))
