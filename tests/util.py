"""Helpers shared by the tests: error norms and a stage-level oracle/HIP comparison harness."""
import numpy as np


def rel_err(got, ref):
    """max |got - ref| / max |ref|  (the tolerance of the parity bar is stated in this norm)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(got - ref)) / (np.max(np.abs(ref)) + 1e-30))


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / (np.linalg.norm(ref) + 1e-30))


def frac_outside(got, ref, tol):
    """Fraction of elements whose error exceeds tol * max|ref|."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.mean(np.abs(got - ref) > tol * (np.max(np.abs(ref)) + 1e-30)))


TOL = {"f32": 1e-4, "bf16": 2e-2}
