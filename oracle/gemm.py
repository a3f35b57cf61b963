"""Contractions of FP8-coded matrices.

``matmul_nt`` is the definition C[m,n] = sum_k A[m,k] * B[n,k] on decoded
values with float64 accumulation (numpy's matmul is the library primitive).
Every FP8 value is an integer multiple of the format's smallest subnormal, so a
product is an exact integer multiple of a fixed power of two; ``matmul_nt_exact``
evaluates the same sum in unbounded Python integers, for tiny shapes, and is the
brute-force pin of the float64 path.
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np

from . import fp8


def matmul_nt(a_codes: np.ndarray, a_fmt: fp8.Format, b_codes: np.ndarray, b_fmt: fp8.Format) -> np.ndarray:
    """A [M,K] codes, B [N,K] codes -> float64 [M,N] of sum_k a*b (no scales)."""
    a = fp8.decode(a_codes, a_fmt)
    b = fp8.decode(b_codes, b_fmt)
    return a @ b.T


def _unit_log2(fmt: fp8.Format) -> int:
    # smallest subnormal = 2^(1 - bias - man_bits)
    return 1 - fmt.bias - fmt.man_bits


def matmul_nt_exact(a_codes, a_fmt: fp8.Format, b_codes, b_fmt: fp8.Format):
    """Triple loop in exact integer arithmetic; returns a list of lists of Fractions."""
    ua, ub = _unit_log2(a_fmt), _unit_log2(b_fmt)
    a_int = [[int(round(fp8.code_value(a_fmt, int(c)) * 2.0 ** (-ua))) for c in row] for row in a_codes]
    b_int = [[int(round(fp8.code_value(b_fmt, int(c)) * 2.0 ** (-ub))) for c in row] for row in b_codes]
    unit = Fraction(2) ** (ua + ub)
    out = []
    for ar in a_int:
        out_row = []
        for br in b_int:
            acc = 0
            for p, q in zip(ar, br):
                acc += p * q
            out_row.append(acc * unit)
        out.append(out_row)
    return out
