"""CPU oracle for the nonlinearity between the two linear layers of a feed-forward block, and for the
Monarch layer with that nonlinearity attached.

TEST INFRASTRUCTURE ONLY (see the package docstring).  float64 numpy throughout.

The paper swaps the dense weight matrices of the attention and feed-forward blocks of ViT, MLP-Mixer, BERT
and GPT-2 for Monarch matrices and leaves the rest of each block as it is (Section 4; Section 5.1); it
never writes the block's nonlinearity down.  All four models use GELU there.  This oracle takes the form
GPT-2 uses (GPT-2 medium is the largest stated workload),

    gelu(v) = v / 2 * (1 + tanh( sqrt(2/pi) * (v + 0.044715 v^3) )),

the "tanh form" of Hendrycks & Gimpel's GELU, whose exact form is  v * Phi(v)  with the standard normal
distribution function Phi.  The two differ by less than 1e-3 everywhere (pinned in the tests).

    fwd_bias_gelu(x, R, L, bias)        -> (y_pre, y):  y_pre = x M^T + bias,  y = gelu(y_pre)
    bwd_bias_gelu_in(dy, x_pre, R, L)   -> (dx_pre, dR, dL, dbias) for  y = gelu(x_pre) M^T + bias:
                                           the chain rule through the multiply, then through gelu

Each is the composition of the package's step-by-step multiply with the elementwise formulas below, with
nothing reordered.
"""
from __future__ import annotations

import numpy as np

from . import READING_A, bwd_bias, fwd_bias

_C0 = np.sqrt(2.0 / np.pi)
_C1 = 0.044715


def gelu(v):
    """Tanh-form GELU, elementwise."""
    v = np.asarray(v, dtype=np.float64)
    return 0.5 * v * (1.0 + np.tanh(_C0 * (v + _C1 * v ** 3)))


def gelu_grad(v):
    """d gelu / d v, elementwise: product rule on  v/2 * (1 + tanh(u(v))),  u = c0 (v + c1 v^3)."""
    v = np.asarray(v, dtype=np.float64)
    t = np.tanh(_C0 * (v + _C1 * v ** 3))
    du = _C0 * (1.0 + 3.0 * _C1 * v ** 2)
    return 0.5 * (1.0 + t) + 0.5 * v * (1.0 - t * t) * du


def fwd_bias_gelu(x, R, L, bias, reading: int = READING_A):
    """(y_pre, y) of the layer  y = gelu(x M^T + bias)."""
    y_pre = fwd_bias(x, R, L, bias, reading)
    return y_pre, gelu(y_pre)


def bwd_bias_gelu_in(dy, x_pre, R, L, reading: int = READING_A, x=None):
    """Gradients of  y = gelu(x_pre) M^T + bias  for the upstream gradient dy.

    The multiply sees x = gelu(x_pre): dR, dL and dbias are those of the plain layer at that x, and the
    gradient with respect to x goes through gelu elementwise:  dx_pre = dx * gelu'(x_pre).
    `x`: the layer's input as the caller holds it (gelu(x_pre) rounded to a storage type), used in place
    of the exact gelu(x_pre) when given.
    """
    x_pre = np.asarray(x_pre, dtype=np.float64)
    x = gelu(x_pre) if x is None else np.asarray(x, dtype=np.float64)
    dx, dR, dL, dbias = bwd_bias(dy, x, R, L, reading)
    return dx * gelu_grad(x_pre), dR, dL, dbias
