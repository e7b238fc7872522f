"""CPU oracle for the Monarch multiply (forward and backward).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
module; only the test-suite, the smoke check and the benchmark's CPU-baseline
leg do.  It shares no code with the GPU library.

Two independent formulations live here:

* ``fwd`` / ``bwd`` -- the step-by-step method of the paper (Section 3.3, steps
  1-3, with the permutation P of Definition 3.1), in plain C, double precision
  (``monarch_oracle.c``; built with gcc by :func:`build`).
* ``dense`` -- the literal definition ``M = P L P^T R`` materialised from
  explicit 0/1 permutation matrices and explicit block-diagonal matrices
  (``dense.py``, numpy, tiny sizes only).

``fwd_bias`` / ``bwd_bias`` add the bias vector of the linear layer whose weight matrix the
Monarch matrix replaces (Section 4: the dense weight matrices are swapped for Monarch ones, the rest
of the layer stays; the appendix on BERT pretraining lists the matrix product with the bias add, and
the bias gradient in the backward pass, as steps worth fusing with the product).

``project`` (``project.py``) is Algorithm 1, the projection of a dense matrix onto the square Monarch
matrices by one best-rank-1 approximation per slice.

All arrays are float64, row-major.  Low-precision inputs must be converted
exactly to float64 by the caller.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "monarch_oracle.c")
_LIB = os.path.join(_HERE, "libmonarch_oracle.so")
_lib = None

READING_A = 0  # (k, q) grid transposed to (q, k), flattened, cut into k chunks of q
READING_B = 1  # the inverse permutation


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP over batch rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-o", tmp, _SRC]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.monarch_oracle_fwd.restype = ctypes.c_int
        lib.monarch_oracle_fwd.argtypes = [dp, dp, dp, dp, ctypes.c_int64] + [ctypes.c_int] * 5
        lib.monarch_oracle_bwd.restype = ctypes.c_int
        lib.monarch_oracle_bwd.argtypes = [dp] * 7 + [ctypes.c_int64] + [ctypes.c_int] * 5
        lib.monarch_oracle_pi.restype = ctypes.c_int64
        lib.monarch_oracle_pi.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.monarch_oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a, shape):
    a = np.ascontiguousarray(np.asarray(a, dtype=np.float64))
    if a.shape != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (tuple(shape), a.shape))
    return a


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def num_threads() -> int:
    """Number of OpenMP threads the C oracle will use."""
    return int(_load().monarch_oracle_num_threads())


def pi(f: int, k: int, q: int, reading: int = READING_A) -> int:
    """Mid permutation: U[f] = Y1flat[pi(f)]."""
    return int(_load().monarch_oracle_pi(f, k, q, reading))


def fwd(x, R, L, reading: int = READING_A):
    """y = x M^T with M = Pout BD(L) Pmid BD(R).  x (B, k*p), R (k,q,p), L (k,s,q) -> y (B, k*s)."""
    R = np.asarray(R)
    L = np.asarray(L)
    k, q, p = R.shape
    k2, s, q2 = L.shape
    if k2 != k or q2 != q:
        raise ValueError("R %s and L %s do not chain" % (R.shape, L.shape))
    x = np.asarray(x)
    B = x.shape[0]
    x = _f64(x, (B, k * p))
    R = _f64(R, (k, q, p))
    L = _f64(L, (k, s, q))
    y = np.empty((B, k * s), dtype=np.float64)
    rc = _load().monarch_oracle_fwd(_ptr(x), _ptr(R), _ptr(L), _ptr(y), B, k * p, k, q, s, reading)
    if rc != 0:
        raise RuntimeError("monarch_oracle_fwd failed: %d" % rc)
    return y


def bwd(dy, x, R, L, reading: int = READING_A):
    """Adjoint of :func:`fwd`: returns (dx, dR, dL) for upstream gradient dy (B, k*s)."""
    R = np.asarray(R)
    L = np.asarray(L)
    k, q, p = R.shape
    k2, s, q2 = L.shape
    if k2 != k or q2 != q:
        raise ValueError("R %s and L %s do not chain" % (R.shape, L.shape))
    x = np.asarray(x)
    B = x.shape[0]
    x = _f64(x, (B, k * p))
    dy = _f64(dy, (B, k * s))
    R = _f64(R, (k, q, p))
    L = _f64(L, (k, s, q))
    dx = np.empty((B, k * p), dtype=np.float64)
    dR = np.empty((k, q, p), dtype=np.float64)
    dL = np.empty((k, s, q), dtype=np.float64)
    rc = _load().monarch_oracle_bwd(
        _ptr(dy), _ptr(x), _ptr(R), _ptr(L), _ptr(dx), _ptr(dR), _ptr(dL), B, k * p, k, q, s, reading
    )
    if rc != 0:
        raise RuntimeError("monarch_oracle_bwd failed: %d" % rc)
    return dx, dR, dL


def fwd_t(x, R, L, reading: int = READING_A):
    """y = x M: the transposed Monarch matrix M^T = R^T P L^T P^T applied to every row (M* of
    Section 3.1, "Products of Monarch Matrices", for real factors).  x (B, k*s) -> y (B, k*p).

    These are the adjoint steps of the multiply taken in reverse order -- undo the outer permutation,
    multiply by the transposed blocks of L, undo the mid permutation, multiply by the transposed blocks
    of R -- which is exactly the input-gradient part of :func:`bwd`, whose C code is used here with the
    upstream gradient set to x (the activations argument does not enter dx)."""
    R = np.asarray(R)
    L = np.asarray(L)
    k, q, p = R.shape
    x = np.asarray(x)
    return bwd(x, np.zeros((x.shape[0], k * p)), R, L, reading)[0]


def fwd_bias(x, R, L, bias, reading: int = READING_A):
    """y[b][o] = (x M^T)[b][o] + bias[o]: the affine layer built on the Monarch matrix."""
    y = fwd(x, R, L, reading)
    bias = _f64(bias, (y.shape[1],))
    for b in range(y.shape[0]):
        y[b, :] = y[b, :] + bias
    return y


def bwd_bias(dy, x, R, L, reading: int = READING_A):
    """Adjoint of :func:`fwd_bias`: (dx, dR, dL, dbias) with dbias[o] = sum_b dy[b][o].

    The bias enters every row of y with coefficient one, so its gradient is the column sum of the
    upstream gradient; dx, dR and dL do not depend on the bias at all.
    """
    dx, dR, dL = bwd(dy, x, R, L, reading)
    dy = np.asarray(dy, dtype=np.float64)
    dbias = np.zeros(dy.shape[1], dtype=np.float64)
    for b in range(dy.shape[0]):
        dbias += dy[b, :]
    return dx, dR, dL, dbias


def rel_fro(got, want) -> float:
    """Relative Frobenius error  ||got - want||_F / ||want||_F  (0 if both are empty/zero)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = float(np.linalg.norm(want.ravel()))
    num = float(np.linalg.norm((got - want).ravel()))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den
