"""Shared by the GPU parity tests: the two measures every comparison with the CPU oracle is gated on."""
import sys

import numpy as np

TOL_F3M = 1e-5      # GPU F3M against CPU F3M, relative L2
TOL_EXACT = 1e-3    # F3M against the exact product, relative L2
MAX_FACTOR = 4.0    # element-wise bar: max|got - want| <= MAX_FACTOR * tol * max|want|


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def rel(a, b):
    """relative L2 distance of a from b"""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def maxrel(a, b):
    """largest element-wise difference over the largest magnitude of b"""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.max(np.abs(a - b)) / np.max(np.abs(b)))


def assert_close(got, want, tol, what=""):
    """Relative L2 <= tol AND no single element further off than MAX_FACTOR * tol * max|want|: the norm alone
    would let one wrong box among many pass.  Returns (relative L2, element-wise figure)."""
    e2, em = rel(got, want), maxrel(got, want)
    if what:
        say("  %s: rel L2 %.3e, max|diff|/max|ref| %.3e" % (what, e2, em))
    assert e2 <= tol, (what, e2, tol)
    assert em <= MAX_FACTOR * tol, (what, em, MAX_FACTOR * tol)
    return e2, em
