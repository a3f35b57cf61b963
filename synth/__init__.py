"""Seeded synthetic inputs for the FP8 Smooth-SwiGLU MLP block.

This module only draws random numbers and lays them out; it contains none of
the method's arithmetic (no scaling rules, no FP8 casts, no SwiGLU).  It is the
one piece shared by the CPU oracle's tests and the HIP path's tests/bench, so
that both sides receive the same bytes.

All tensors are bf16, returned as ``torch.Tensor`` on the CPU.  The draw order
is fixed (x, W1, W2, W3, dY) from one ``torch.Generator`` so that a seed pins
every byte.  Weight naming follows the paper (Section 4.1): W1 is the linear
branch, W2 the branch that goes through Swish, W3 the last linear layer.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import torch


@dataclass(frozen=True)
class MlpShape:
    name: str
    T: int          # tokens (rows of x)
    d: int          # d_model
    f: int          # d_ffn  (number of SwiGLU channels)
    seed: int
    w_std: float
    backward: bool
    aligned_channels: int = 0   # >0: outlier-stress recipe


# The five workloads of the benchmark description.  "7b" is the shape the
# headline metric is quoted on.
CONFIGS: Dict[str, MlpShape] = {
    "tiny":      MlpShape("tiny",      256,   256,   688,   0, 0.02, True),
    "7b_fwd":    MlpShape("7b_fwd",    4096,  4096,  11008, 2, 0.02, False),
    "7b":        MlpShape("7b",        4096,  4096,  11008, 3, 0.02, True),
    "7b_stress": MlpShape("7b_stress", 16384, 4096,  11008, 4, 0.02, False, aligned_channels=8),
    "large":     MlpShape("large",     8192,  8192,  28672, 5, 0.01, True),
}


def _randn_bf16(gen: torch.Generator, shape, std: float) -> torch.Tensor:
    # Draw in fp32 in bounded row chunks (keeps the peak host footprint small
    # for the large shape), multiply by std, round to bf16.
    rows, cols = shape
    out = torch.empty(rows, cols, dtype=torch.bfloat16)
    step = max(1, (1 << 24) // cols)
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        out[r0:r1] = (torch.randn(r1 - r0, cols, generator=gen, dtype=torch.float32) * std).to(torch.bfloat16)
    return out


def make_inputs(T: int, d: int, f: int, seed: int, w_std: float = 0.02,
                dy_std: float = 1e-3, backward: bool = True,
                aligned_channels: int = 0) -> Dict[str, Optional[torch.Tensor]]:
    """x [T,d] ~ N(0,1); W1, W2 [f,d] and W3 [d,f] ~ N(0, w_std^2); dY [T,d] ~ N(0, dy_std^2).

    ``aligned_channels`` > 0 applies the outlier-stress recipe: that many
    channel indices are picked with a seeded permutation, W2's row is set to
    W1's row plus N(0, 1e-6) noise and both rows are multiplied by 20, which
    mimics the aligned, large-norm channels the paper observes late in
    training (Section 4.3, Figure 2).
    """
    gen = torch.Generator(device="cpu").manual_seed(seed)
    x = _randn_bf16(gen, (T, d), 1.0)
    W1 = _randn_bf16(gen, (f, d), w_std)
    W2 = _randn_bf16(gen, (f, d), w_std)
    W3 = _randn_bf16(gen, (d, f), w_std)
    dY = _randn_bf16(gen, (T, d), dy_std) if backward else None
    chans = None
    if aligned_channels > 0:
        chans = torch.randperm(f, generator=gen)[:aligned_channels]
        noise = torch.randn(aligned_channels, d, generator=gen, dtype=torch.float32) * 1e-3
        w1_rows = W1[chans].to(torch.float32)
        W2[chans] = ((w1_rows + noise) * 20.0).to(torch.bfloat16)
        W1[chans] = (w1_rows * 20.0).to(torch.bfloat16)
    return {"x": x, "W1": W1, "W2": W2, "W3": W3, "dY": dY, "aligned": chans}


def make_config(name: str) -> Dict[str, Optional[torch.Tensor]]:
    c = CONFIGS[name]
    return make_inputs(c.T, c.d, c.f, c.seed, c.w_std, backward=c.backward,
                       aligned_channels=c.aligned_channels)


def bf16_to_f32_numpy(t: torch.Tensor):
    """Exact widening of a bf16 CPU tensor to a float32 numpy array."""
    return t.to(torch.float32).numpy()
