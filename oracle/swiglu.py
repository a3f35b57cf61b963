"""The SwiGLU neuron and its derivatives (Section 4.1), in float64.

    SwiGLU(u, g) = u * Swish(g) = u * g * sigma(g),   sigma(z) = 1 / (1 + e^-z)

u = x^T w1 is the linear branch and g = x^T w2 the gated branch.
"""
from __future__ import annotations

import numpy as np


def sigmoid(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.float64)
    with np.errstate(over="ignore"):
        return 1.0 / (1.0 + np.exp(-z))


def swish(g: np.ndarray) -> np.ndarray:
    g = np.asarray(g, dtype=np.float64)
    return g * sigmoid(g)


def swiglu(u: np.ndarray, g: np.ndarray) -> np.ndarray:
    return np.asarray(u, dtype=np.float64) * swish(g)


def swiglu_grads(u: np.ndarray, g: np.ndarray, dh: np.ndarray):
    """Gradients of h = u * g * sigma(g) with respect to u and g, times dh.

    dh/du = g * sigma(g)
    dh/dg = u * (sigma(g) + g * sigma'(g)) = u * sigma(g) * (1 + g * (1 - sigma(g)))
    """
    u = np.asarray(u, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    dh = np.asarray(dh, dtype=np.float64)
    sg = sigmoid(g)
    du = dh * g * sg
    dg = dh * u * sg * (1.0 + g * (1.0 - sg))
    return du, dg
