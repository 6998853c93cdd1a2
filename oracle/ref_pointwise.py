"""fp64 definitions of the pointwise operators that sit between the matrix
multiplications of a Llama layer: RMS normalisation, rotary position
embedding and the SwiGLU gate, forward and backward.  TEST INFRASTRUCTURE ONLY.

Why they are here: the paper's activation-checkpointing pass lets every
operator outside the attention layer be rematerialised in the backward pass
(Section 3.2, its strategy: operators outside attention take an O(1/s) share of
the work at long context), and the models it evaluates are Llama models
(Section 4 setup).  Outside attention a device holds its S/P tokens with the
full model dimension (Section 2, Figure 1), which is the shape these work on.
The operators themselves are not written out in the paper; the definitions
below are the Llama architecture's published ones.

All functions take and return fp64 arrays; nothing is rounded.
Pinned by tests/test_pointwise_pins.py (torch fp64 autograd, closed forms,
finite differences, group properties of the rotation).
"""
from __future__ import annotations

import numpy as np


# ---------------------------------------------------------------- RMS norm
# y[t, c] = x[t, c] * rstd[t] * w[c],  rstd[t] = 1 / sqrt(mean_c x[t, c]^2 + eps)
def rmsnorm_fwd(x: np.ndarray, w: np.ndarray, eps: float):
    rstd = 1.0 / np.sqrt(np.mean(x * x, axis=1) + eps)
    return x * rstd[:, None] * w[None, :], rstd


def rmsnorm_bwd(x: np.ndarray, w: np.ndarray, dy: np.ndarray, eps: float):
    """Gradients of L = sum(y * dy) with respect to x and w."""
    T, C = x.shape
    rstd = 1.0 / np.sqrt(np.mean(x * x, axis=1) + eps)
    g = dy * w[None, :]                      # dL/d(x * rstd)
    dot = np.sum(g * x, axis=1)              # sum_c g x
    dx = g * rstd[:, None] - x * (rstd ** 3 * dot / C)[:, None]
    dw = np.sum(dy * x * rstd[:, None], axis=0)
    return dx, dw


# ---------------------------------------------------------------- rotary embedding
# The head dim is split into two halves; element i of the first half and element i
# of the second half form a pair that is rotated by the angle of (position, i):
#   out1 = x1 * cos - x2 * sin,   out2 = x2 * cos + x1 * sin
# `conjugate` rotates by the negative angle, which is the gradient operator.
def rope_angles(positions: np.ndarray, D: int, base: float = 10000.0) -> np.ndarray:
    """angles[t, i] = positions[t] * base^(-2i/D), i < D/2."""
    inv = base ** (-np.arange(0, D, 2, dtype=np.float64) / D)
    return positions.astype(np.float64)[:, None] * inv[None, :]


def rope(x: np.ndarray, cos: np.ndarray, sin: np.ndarray, conjugate: bool = False) -> np.ndarray:
    """x [T, H, D], cos/sin [T, D/2]."""
    T, H, D = x.shape
    h = D // 2
    x1, x2 = x[..., :h], x[..., h:]
    c = cos[:, None, :]
    s = (-sin if conjugate else sin)[:, None, :]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


# ---------------------------------------------------------------- SwiGLU gate
# y = silu(g) * u,  silu(g) = g * sigmoid(g)
def swiglu_fwd(g: np.ndarray, u: np.ndarray) -> np.ndarray:
    return g / (1.0 + np.exp(-g)) * u


def swiglu_bwd(g: np.ndarray, u: np.ndarray, dy: np.ndarray):
    sig = 1.0 / (1.0 + np.exp(-g))
    dg = dy * u * sig * (1.0 + g * (1.0 - sig))
    du = dy * g * sig
    return dg, du
