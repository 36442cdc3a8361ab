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


def assert_parity(got, oracle, dtype, what="", bound_scale=None):
    """Compare a kernel result (widened to float64) with the oracle, element by element.

    bound_scale (broadcastable to the result, >= 1) widens the bound where the caller has derived that the inputs'
    conditioning, not the kernel, limits what binary32 arithmetic can reach (see layernorm_bound_scale)."""
    rtol, atol = TOL[np.dtype(dtype)]
    g = np.asarray(got, dtype=np.float64)
    o = np.asarray(oracle, dtype=np.float64)
    assert g.shape == o.shape, f"{what}: shape {g.shape} vs {o.shape}"
    assert np.isfinite(g).all(), f"{what}: non-finite kernel output"
    err = np.abs(g - o)
    bound = np.maximum(atol, rtol * np.abs(o))
    if bound_scale is not None:
        bound = bound * np.maximum(1.0, np.asarray(bound_scale, dtype=np.float64))
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


def layernorm_bound_scale(x, residual, bias, eps):
    """Per-row factor by which the rounding of t = x + bias + residual can exceed the ordinary bar.

    binary32 forms t with two roundings, each at most 2^-24 relative to a partial sum of magnitude at most
    T = max_j (|x_j| + |bias_j| + |residual_j|); the oracle adds in double.  So every t_j is off by up to 2^-23 T, and
    through (t_j - mean) / sigma an output near zero moves by up to |gamma_j| * 2 * 2^-23 T / sigma = 2.4e-7 * kappa,
    kappa = T / sigma (one part from t_j itself, one from the mean; the part through sigma vanishes with the output).
    That reaches the absolute floor of 1e-6 at kappa = 4, the value of well-spread rows (standard normal x and
    residual give T about 5.5 and sigma about 1.4), so the bar is scaled by max(1, kappa / 4): rows of two or three
    nearly equal values stay checked, against the bound binary32 can meet."""
    t_abs = np.abs(np.asarray(x, dtype=np.float64))
    t = np.asarray(x, dtype=np.float64).copy()
    if residual is not None:
        t_abs = t_abs + np.abs(np.asarray(residual, dtype=np.float64))
        t = t + np.asarray(residual, dtype=np.float64)
    if bias is not None:
        t_abs = t_abs + np.abs(np.asarray(bias, dtype=np.float64))[None, :]
        t = t + np.asarray(bias, dtype=np.float64)[None, :]
    sigma = np.sqrt(t.var(axis=1) + float(eps))
    kappa = t_abs.max(axis=1) / np.maximum(sigma, 1e-300)
    return np.maximum(1.0, kappa / 4.0)[:, None]
