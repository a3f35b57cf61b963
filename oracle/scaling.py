"""Delayed per-tensor scaling with an amax history.  TEST INFRASTRUCTURE ONLY.

Section 2 describes the scheme (the scale of a tensor is taken from the ranges
seen in earlier iterations, which avoids a pass over the data before the cast)
and Section 6.2 says the paper's runs used it, "similar to" the recipe of
Nvidia's Transformer Engine.  The paper prints no formula; the reading used
here (**parity unpinned** by the paper) is the common one:

    history   the largest magnitudes of the tensor in its last H calls (H = 16)
    scale     fl32(fmax / max(history)), margin 0; 1 while the history is empty
    cast      satcast(fl32(v * scale)): anything beyond the range saturates
    after the call, the range seen in it replaces the oldest history entry

Smooth-SwiGLU's per-channel factors stay current (they are the point of the
method), and so does the scale of the folded w3, which needs no data pass.
"""
from __future__ import annotations

import numpy as np

from . import fp8, quant

HISTORY = 16
FORMATS = {"x": fp8.E4M3, "w1": fp8.E4M3, "w2": fp8.E4M3, "dy": fp8.E5M2, "du": fp8.E5M2, "dg": fp8.E5M2}


class DelayedScaling:
    def __init__(self, names=tuple(FORMATS), history: int = HISTORY):
        self.hist = {n: np.zeros(history, np.float32) for n in names}
        self.pos = {n: 0 for n in names}

    def scale(self, name: str, pow2: bool = False) -> np.float32:
        """The scale the next call uses for this tensor."""
        return np.float32(quant.scale_from_amax(self.hist[name].max(), FORMATS[name], pow2))

    def scales(self, names, pow2: bool = False) -> dict:
        return {n: self.scale(n, pow2) for n in names}

    def record(self, name: str, amax) -> None:
        """Enter the range seen in the call just finished."""
        h = self.hist[name]
        h[self.pos[name]] = np.float32(amax)
        self.pos[name] = (self.pos[name] + 1) % h.size

    def record_all(self, amaxes: dict) -> None:
        for n, a in amaxes.items():
            self.record(n, a)
