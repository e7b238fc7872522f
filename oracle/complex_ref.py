"""Complex-valued Monarch multiply and the (inverse) DFT as a Monarch matrix.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).

The paper's results hold over the complex numbers as well (Notation Review), and its MRI model
(mSENSE) is one complex Monarch matrix initialised to the inverse FFT and then trained.  This module
writes the same steps as the real oracle -- Section 3.3, steps 1-3, with the permutations of
Definition 3.1 -- in numpy complex128, one block at a time, with plain loops over the blocks and
``@`` inside a block.

Gradients follow the convention of automatic differentiation for a real loss and complex
parameters: the gradient of z is dLoss/dRe(z) + i dLoss/dIm(z).  For y = x M^T and upstream
gradient dy that is  dx = dy conj(M),  dL[c] = dW[c]^T conj(U[c]),  dR[kk] = dY1[kk]^T conj(x[kk])
(no transposes are conjugated by the multiply itself: M^T, not M^*).

DFT.  With n = m*m, w_n = exp(-2 pi i / n) and the input read as an m x m grid that is transposed
first, the 4-step (Cooley-Tukey) splitting of the DFT is literally a Monarch product:
    F_n P = P L P^T R,   R[kk][j][i] = w_m^(i j),   L[j][l][kk] = w_n^(kk j) * w_m^(kk l)
because for input position i*m + kk and output position l*m + j
    w_n^((i m + kk)(l m + j)) = w_m^(i j) * w_n^(kk j) * w_m^(kk l).
The inverse transform conjugates the factors and carries 1/n (put into L here).
"""
from __future__ import annotations

import numpy as np


def _mid_source(f: int, k: int, q: int, reading: int) -> tuple[int, int]:
    """(kk, j) of the stage-1 output that lands at position f of the stage-2 input."""
    if reading == 0:  # the (k, q) grid transposed to (q, k), flattened
        return f % k, f // k
    g = (f % q) * k + f // q  # the inverse permutation: flat (q, k) grid transposed to (k, q)
    return g // q, g % q


def fwd(x, R, L, reading: int = 0):
    """y = x M^T for complex x (B, k*p), R (k, q, p), L (k, s, q); returns complex128 (B, k*s)."""
    x = np.asarray(x, dtype=np.complex128)
    R = np.asarray(R, dtype=np.complex128)
    L = np.asarray(L, dtype=np.complex128)
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    Y1 = np.zeros((B, k, q), dtype=np.complex128)
    for kk in range(k):
        Y1[:, kk, :] = x[:, kk * p:(kk + 1) * p] @ R[kk].T
    U = np.zeros((B, k * q), dtype=np.complex128)
    for f in range(k * q):
        kk, j = _mid_source(f, k, q, reading)
        U[:, f] = Y1[:, kk, j]
    y = np.zeros((B, k * s), dtype=np.complex128)
    for c in range(k):
        W = U[:, c * q:(c + 1) * q] @ L[c].T  # (B, s)
        for l in range(s):
            y[:, l * k + c] = W[:, l]
    return y


def bwd(dy, x, R, L, reading: int = 0):
    """(dx, dR, dL) for a real loss, in the dRe + i dIm convention (see the module text)."""
    x = np.asarray(x, dtype=np.complex128)
    dy = np.asarray(dy, dtype=np.complex128)
    R = np.asarray(R, dtype=np.complex128)
    L = np.asarray(L, dtype=np.complex128)
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    Y1 = np.zeros((B, k, q), dtype=np.complex128)
    for kk in range(k):
        Y1[:, kk, :] = x[:, kk * p:(kk + 1) * p] @ R[kk].T
    U = np.zeros((B, k * q), dtype=np.complex128)
    for f in range(k * q):
        kk, j = _mid_source(f, k, q, reading)
        U[:, f] = Y1[:, kk, j]
    dU = np.zeros((B, k * q), dtype=np.complex128)
    dL = np.zeros_like(L)
    for c in range(k):
        dW = np.stack([dy[:, l * k + c] for l in range(s)], axis=1)  # (B, s)
        dL[c] = dW.T @ np.conj(U[:, c * q:(c + 1) * q])
        dU[:, c * q:(c + 1) * q] = dW @ np.conj(L[c])
    dY1 = np.zeros((B, k, q), dtype=np.complex128)
    for f in range(k * q):
        kk, j = _mid_source(f, k, q, reading)
        dY1[:, kk, j] = dU[:, f]
    dx = np.zeros_like(x)
    dR = np.zeros_like(R)
    for kk in range(k):
        dR[kk] = dY1[:, kk, :].T @ np.conj(x[:, kk * p:(kk + 1) * p])
        dx[:, kk * p:(kk + 1) * p] = dY1[:, kk, :] @ np.conj(R[kk])
    return dx, dR, dL


def fwd_h(x, R, L, reading: int = 0):
    """y = x conj(M): every row multiplied by the conjugate transpose M* of the Monarch matrix, the second factor
    of the products M1 M2* of Section 3.1 ("Products of Monarch Matrices"; M* = conjugate transpose, Notation
    Review).  x (B, k*s) -> y (B, k*p).  With M = Pout BD(L) Pmid BD(R), M* = BD(R)* Pmid^T BD(L)* Pout^T: undo the
    outer permutation, multiply by the conjugate-transposed blocks of L, undo the mid permutation, multiply by the
    conjugate-transposed blocks of R."""
    x = np.asarray(x, dtype=np.complex128)
    R = np.asarray(R, dtype=np.complex128)
    L = np.asarray(L, dtype=np.complex128)
    k, q, p = R.shape
    s = L.shape[1]
    B = x.shape[0]
    V = np.zeros((B, k * q), dtype=np.complex128)        # BD(L)* applied to Pout^T x
    for c in range(k):
        Wc = np.stack([x[:, l * k + c] for l in range(s)], axis=1)   # (B, s): entries (c, l) of the (k, s) grid
        V[:, c * q:(c + 1) * q] = Wc @ np.conj(L[c])                  # sum_l conj(L[c][l][r]) W[c][l]
    T = np.zeros((B, k, q), dtype=np.complex128)         # Pmid^T: position f of the stage-2 input goes back to (kk, j)
    for f in range(k * q):
        kk, j = _mid_source(f, k, q, reading)
        T[:, kk, j] = V[:, f]
    y = np.zeros((B, k * p), dtype=np.complex128)
    for kk in range(k):
        y[:, kk * p:(kk + 1) * p] = T[:, kk, :] @ np.conj(R[kk])     # sum_j conj(R[kk][j][i]) T[kk][j]
    return y


def dft_factors(m: int, inverse: bool = False):
    """(R, L), each (m, m, m) complex128, with  P L P^T R = F_n P  (or F_n^{-1} P), n = m*m."""
    n = m * m
    sign = 1.0 if inverse else -1.0
    wm = np.exp(sign * 2j * np.pi / m)
    wn = np.exp(sign * 2j * np.pi / n)
    R = np.zeros((m, m, m), dtype=np.complex128)
    L = np.zeros((m, m, m), dtype=np.complex128)
    for kk in range(m):
        for j in range(m):
            for i in range(m):
                R[kk, j, i] = wm ** (i * j)
    for j in range(m):
        for l in range(m):
            for kk in range(m):
                L[j, l, kk] = wn ** (kk * j) * wm ** (kk * l) / (n if inverse else 1.0)
    return R, L
