import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


# Element-wise parity bar: |g - o| <= max(atol, rtol * |o|).
TOL = {
    np.dtype(np.float32): (1e-5, 1e-6),
    np.dtype(np.float16): (3e-3, 1e-6),
}


def assert_parity(got, oracle, dtype, what=""):
    """Compare a kernel result (widened to float64) with the oracle, element by element."""
    rtol, atol = TOL[np.dtype(dtype)]
    g = np.asarray(got, dtype=np.float64)
    o = np.asarray(oracle, dtype=np.float64)
    assert g.shape == o.shape, f"{what}: shape {g.shape} vs {o.shape}"
    assert np.isfinite(g).all(), f"{what}: non-finite kernel output"
    err = np.abs(g - o)
    bound = np.maximum(atol, rtol * np.abs(o))
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(
            f"{what}: {int(bad.sum())} of {bad.size} elements out of tolerance; worst at {i}: "
            f"got {g[i]!r}, oracle {o[i]!r}, |diff| {err[i]:.3e} > {bound[i]:.3e}")
    # (largest absolute error, largest relative error among elements whose relative bound is the binding one, largest
    # error as a fraction of the element's bound)
    rel_zone = rtol * np.abs(o) >= atol
    max_rel = float((err[rel_zone] / np.abs(o[rel_zone])).max()) if rel_zone.any() else 0.0
    return float(err.max()) if err.size else 0.0, max_rel, float((err / bound).max()) if err.size else 0.0
