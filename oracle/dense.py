"""The Monarch matrix written out densely, from the literal definition.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Tiny sizes only.

Definition 3.1 gives ``M = P L P^T R`` with L, R block-diagonal and P the
permutation "reshape as a grid, transpose, flatten".  This module builds every
one of those matrices explicitly as a dense float64 array -- no index tricks in
the product, just ``@`` -- so that it is independent of the step-by-step
implementation in ``monarch_oracle.c``.
"""
from __future__ import annotations

import numpy as np


def block_diag(blocks: np.ndarray) -> np.ndarray:
    """diag(blocks[0], ..., blocks[k-1]) for blocks of shape (k, rows, cols)."""
    k, rows, cols = blocks.shape
    out = np.zeros((k * rows, k * cols), dtype=np.float64)
    for b in range(k):
        out[b * rows:(b + 1) * rows, b * cols:(b + 1) * cols] = blocks[b]
    return out


def transpose_perm(rows: int, cols: int) -> np.ndarray:
    """0/1 matrix T with  T @ v == v.reshape(rows, cols).T.ravel()  for every v."""
    n = rows * cols
    T = np.zeros((n, n), dtype=np.float64)
    for a in range(rows):
        for b in range(cols):
            # element (a, b) of the grid, flat index a*cols + b, lands at (b, a): b*rows + a
            T[b * rows + a, a * cols + b] = 1.0
    return T


def mid_perm(k: int, q: int, reading: int = 0) -> np.ndarray:
    """The permutation between the two block-diagonal factors (P^T of Def. 3.1).

    reading 0: take the (k, q) grid, transpose to (q, k), flatten.
    reading 1: take the flat vector as a (q, k) grid, transpose to (k, q), flatten.
    """
    return transpose_perm(k, q) if reading == 0 else transpose_perm(q, k)


def out_perm(k: int, s: int) -> np.ndarray:
    """The outer P: the (k, s) grid of stage-2 outputs transposed to (s, k)."""
    return transpose_perm(k, s)


def monarch_dense(R: np.ndarray, L: np.ndarray, reading: int = 0) -> np.ndarray:
    """Dense (k*s) x (k*p) matrix  Pout @ BD(L) @ Pmid @ BD(R)."""
    R = np.asarray(R, dtype=np.float64)
    L = np.asarray(L, dtype=np.float64)
    k, q, p = R.shape
    k2, s, q2 = L.shape
    assert k2 == k and q2 == q
    return out_perm(k, s) @ block_diag(L) @ mid_perm(k, q, reading) @ block_diag(R)


def eq1_dense_square(R: np.ndarray, L: np.ndarray) -> np.ndarray:
    """Equation (1): M[l*m + j, k*m + i] = L[j, l, k] * R[k, j, i]  (square case, 0-based)."""
    m = R.shape[0]
    assert R.shape == (m, m, m) and L.shape == (m, m, m)
    M = np.zeros((m * m, m * m), dtype=np.float64)
    for l in range(m):
        for j in range(m):
            for k in range(m):
                for i in range(m):
                    M[l * m + j, k * m + i] = L[j, l, k] * R[k, j, i]
    return M
