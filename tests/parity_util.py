"""Comparison rule of the parity tests (CPU-only code, so that the rule itself can be unit-tested).

Two bounds, both against the oracle's result:
  * the relative Frobenius error of the whole tensor <= tol (the stated tolerance), and
  * a local bound at LOCAL_FACTOR x tol on every slice along the first axis -- every row of an activation
    tensor (y, dx, ...), every block of a weight-gradient tensor (dR, dL) -- so that a few wholly wrong
    rows (a bad tail tile, one mis-addressed workgroup) cannot hide inside a large tensor's global ratio.
A slice whose expected norm is far below the typical one is measured against the typical norm instead
(an all-zero expected row must not divide by zero, and must still come back as ~zero)."""
import zlib

import numpy as np

LOCAL_FACTOR = 4.0


def stable_seed(name, modulus=7):
    """A seed derived from a case name that is the same in every process (str hashes are not)."""
    return zlib.crc32(name.encode("utf-8")) % modulus


def rel_fro(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = np.linalg.norm(want.ravel())
    num = np.linalg.norm((got - want).ravel())
    return num / den if den > 0 else num


def local_errors(got, want):
    """Relative error of every slice along axis 0 (rows of a matrix, blocks of a 3-D weight tensor)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.ndim < 2 or want.shape[0] == 0:
        return np.zeros(0)
    w = want.reshape(want.shape[0], -1)
    d = got.reshape(want.shape[0], -1) - w
    wn = np.sqrt(np.einsum("ij,ij->i", w, w))
    dn = np.sqrt(np.einsum("ij,ij->i", d, d))
    typical = np.sqrt(np.mean(wn * wn))
    den = np.maximum(wn, 0.05 * typical)
    return np.where(den > 0, dn / np.where(den > 0, den, 1.0), dn)


def check(name, got, want, tol):
    """Raise AssertionError unless `got` matches `want` under both bounds; returns the global error."""
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, "%s: shape %s, expected %s" % (name, got.shape, want.shape)
    err = rel_fro(got, want)
    assert err <= tol, "%s: relative Frobenius error %.3e > %.1e" % (name, err, tol)
    loc = local_errors(got, want)
    if loc.size:
        worst = int(np.argmax(loc))
        assert loc[worst] <= LOCAL_FACTOR * tol, "%s: slice %d of axis 0 is off by %.3e (> %.1e) while the whole tensor is at %.3e" % (
            name, worst, loc[worst], LOCAL_FACTOR * tol, err)
    return err
