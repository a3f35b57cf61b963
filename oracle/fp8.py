"""OCP 8-bit floating point formats, written out from their definition.

The paper (Section 2) uses the two formats standardised by its FP8 reference:
E4M3 (1 sign, 4 exponent, 3 mantissa bits) for weights and activations and
E5M2 (1 sign, 5 exponent, 2 mantissa bits) for gradients.  The paper gives only
the bit splits; biases, the special codes and the largest finite values are
those of the public OCP FP8 standard it cites:

  E4M3: bias 7, no infinities, NaN = S.1111.111, max finite 448 (code 0x7E),
        min normal 2^-6, min subnormal 2^-9.
  E5M2: bias 15, IEEE-like, Inf = S.11111.00, NaN = S.11111.{01,10,11},
        max finite 57344 (code 0x7B), min normal 2^-14, min subnormal 2^-16.

Encoding here is the definition of round-to-nearest-even with saturation:
search the sorted list of finite representable magnitudes for the nearest one,
resolve an exact tie towards the code whose mantissa LSB is 0, and clamp
anything above the largest finite magnitude to it.  No bit tricks.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Format:
    name: str
    exp_bits: int
    man_bits: int
    bias: int
    max_code: int        # code of the largest finite positive value
    nan_code: int        # canonical NaN (sign bit added by the caller)


E4M3 = Format("e4m3", 4, 3, 7, 0x7E, 0x7F)
E5M2 = Format("e5m2", 5, 2, 15, 0x7B, 0x7F)


def by_name(name: str) -> Format:
    return {"e4m3": E4M3, "e5m2": E5M2}[name]


def code_value(fmt: Format, code: int) -> float:
    """Value of one 8-bit code from (sign, exponent field, mantissa field)."""
    sign = -1.0 if (code >> 7) & 1 else 1.0
    e = (code >> fmt.man_bits) & ((1 << fmt.exp_bits) - 1)
    m = code & ((1 << fmt.man_bits) - 1)
    e_all_ones = (1 << fmt.exp_bits) - 1
    if fmt is E4M3:
        if e == e_all_ones and m == (1 << fmt.man_bits) - 1:
            return math.nan
    else:
        if e == e_all_ones:
            return sign * math.inf if m == 0 else math.nan
    if e == 0:   # subnormal: no implicit one, exponent of the smallest normal
        return sign * (m / (1 << fmt.man_bits)) * 2.0 ** (1 - fmt.bias)
    return sign * (1.0 + m / (1 << fmt.man_bits)) * 2.0 ** (e - fmt.bias)


def decode_table(fmt: Format) -> np.ndarray:
    """All 256 code values as float64 (NaN / Inf where the format says so)."""
    return np.array([code_value(fmt, c) for c in range(256)], dtype=np.float64)


def max_finite(fmt: Format) -> float:
    return code_value(fmt, fmt.max_code)


def decode(codes: np.ndarray, fmt: Format) -> np.ndarray:
    """uint8 codes -> float64 values (exact)."""
    return decode_table(fmt)[np.asarray(codes, dtype=np.uint8)]


def satcast(v: np.ndarray, fmt: Format) -> np.ndarray:
    """Saturating round-to-nearest-even of real values to 8-bit codes.

    |v| is compared against the midpoints between neighbouring finite
    magnitudes (midpoints are exact in float64 because the neighbours have at
    most 4 significant bits).  Below a midpoint -> lower neighbour, above ->
    upper neighbour, exactly on it -> whichever of the two codes is even.
    |v| above the largest finite magnitude (including +-Inf) -> that magnitude.
    NaN -> the canonical NaN code.  The sign bit of v is always kept, so a
    negative value that rounds to zero becomes the code 0x80.
    """
    v = np.asarray(v)
    a = np.abs(v.astype(np.float64))
    mags = decode_table(fmt)[: fmt.max_code + 1]          # codes 0 .. max_code, increasing
    mids = (mags[:-1] + mags[1:]) / 2.0
    a = np.minimum(a, mags[-1])                           # saturation (also maps Inf)
    idx = np.searchsorted(mids, a, side="left")           # number of midpoints strictly below a
    on_mid = np.zeros(a.shape, dtype=bool)
    inside = idx < len(mids)
    on_mid[inside] = mids[idx[inside]] == a[inside]
    # tie between code idx and idx+1: take the even one
    idx = np.where(on_mid & (idx % 2 == 1), idx + 1, idx)
    code = idx.astype(np.uint8)
    code = np.where(np.isnan(v), np.uint8(fmt.nan_code), code)
    sign = np.signbit(v).astype(np.uint8) << 7
    return (code | sign).astype(np.uint8)


def satcast_scalar(v: float, fmt: Format) -> int:
    """Same definition for one Python float, by linear scan (used by tests as
    the brute-force statement of the rule)."""
    if math.isnan(v):
        return fmt.nan_code | (0x80 if math.copysign(1.0, v) < 0 else 0)
    a = min(abs(v), max_finite(fmt))
    best, best_err = 0, math.inf
    for c in range(fmt.max_code + 1):
        err = abs(code_value(fmt, c) - a)
        if err < best_err or (err == best_err and c % 2 == 0):
            best, best_err = c, err
    return best | (0x80 if math.copysign(1.0, v) < 0 else 0)
