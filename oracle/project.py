"""Projection of a dense matrix onto the set of (square) Monarch matrices.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).

Section 3.3 ("Projection on the Set M of Monarch Matrices"), Theorem 1 and Algorithm 1: view the
n x n matrix A, n = m^2, as the 4-D tensor At[l, j, k, i] = A[l*m + j, k*m + i].  By Equation (1) a
Monarch matrix has M[l, j, k, i] = L[j, l, k] * R[k, j, i], i.e. for every pair (j, k) the m x m slice
M[:, j, k, :] is the rank-1 matrix  L[j, :, k] R[k, j, :]^T.  The Frobenius objective therefore splits
into m*m independent best-rank-1 problems, each solved by the leading singular triple of the slice
(Eckart-Young).  The SVD itself is the library routine (numpy.linalg.svd, float64).

A rank-1 matrix u v^T fixes u and v only up to u -> a*u, v -> v/a; this file splits the singular
value evenly (both factors carry sqrt(sigma_1)).  Comparisons must therefore be made on the products
L[j, l, k] * R[k, j, i] (the Monarch matrix itself), which are unique whenever sigma_1 > sigma_2.
"""
from __future__ import annotations

import math

import numpy as np


def project_square(A):
    """Return (L, R), each (m, m, m) float64, with  P L P^T R  the Monarch matrix closest to A."""
    A = np.asarray(A, dtype=np.float64)
    n = A.shape[0]
    m = math.isqrt(n)
    if A.shape != (n, n) or m * m != n:
        raise ValueError("A must be n x n with n a perfect square, got %s" % (A.shape,))
    At = A.reshape(m, m, m, m)  # [l, j, k, i]
    L = np.zeros((m, m, m), dtype=np.float64)
    R = np.zeros((m, m, m), dtype=np.float64)
    for j in range(m):
        for k in range(m):
            slice_jk = At[:, j, k, :]  # rows l, columns i
            U, S, Vt = np.linalg.svd(slice_jk)
            root = math.sqrt(S[0])
            L[j, :, k] = U[:, 0] * root
            R[k, j, :] = Vt[0, :] * root
    return L, R


def monarch_square(L, R):
    """The dense n x n Monarch matrix of factors (L, R) through Equation (1), as one einsum."""
    L = np.asarray(L, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    m = L.shape[0]
    return np.einsum("jlk,kji->ljki", L, R).reshape(m * m, m * m)
