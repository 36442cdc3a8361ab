"""Derives the coefficients of the branch-free erfc approximation used by gelu_erf() in elementwise_kernels.h.

    erfc(u) ~= exp(-u^2) * sum_{k=1..7} c_k w^k,   w = 1 / (1 + u/2),   u >= 0

The polynomial in w is fitted to erfc(u) exp(u^2) on [0, 9.5] by iteratively re-weighted least squares (a Lawson
iteration towards the minimax relative error).  The script then evaluates the binary32 evaluation order of the kernel
against the double-precision definition t * erfc(-t/sqrt 2)/2 and prints the worst error relative to the parity
bound max(1e-6, 1e-5 |gelu|).  Run it to regenerate or to check the constants; nothing imports it.
"""
import numpy as np
from scipy.special import erfc, erfcx

P = 0.5
N = 7


def fit(p=P, n=N, umax=9.5, iters=60):
    u = np.concatenate([np.linspace(0, 4, 6000), np.linspace(4, umax, 2000)])
    g = erfcx(u)
    w = 1.0 / (1.0 + p * u)
    basis = np.stack([w ** k for k in range(1, n + 1)], 1)
    weight = np.ones_like(u)
    for _ in range(iters):
        scale = weight / g
        c, *_ = np.linalg.lstsq(basis * scale[:, None], g * scale, rcond=None)
        rel = np.abs(basis @ c / g - 1)
        weight = weight * (1 + 5 * rel / rel.max())
        weight /= weight.mean()
    return c, rel.max()


def check(c, p=P):
    f = np.float32
    t = np.linspace(-9, 9, 2000001).astype(f)
    u = np.abs(t) * f(0.70710678118654752)
    w = f(1) / (f(1) + f(p) * u)
    poly = np.zeros_like(w)
    for ck in c[::-1]:
        poly = (poly + f(ck)) * w
    half = f(0.5) * poly * np.exp2(-(u * u) * f(1.4426950408889634)).astype(f)
    got = (t * np.where(t < 0, half, f(1) - half)).astype(np.float64)
    t64 = t.astype(np.float64)
    want = t64 * 0.5 * erfc(-t64 / np.sqrt(2))
    err = np.abs(got - want)
    return err.max(), (err / np.maximum(1e-6, 1e-5 * np.abs(want))).max()


if __name__ == "__main__":
    coeffs, rel = fit()
    print("max relative error of the fit to erfc(u) exp(u^2):", rel)
    print("coefficients c_1..c_7 (binary32):", ", ".join(f"{np.float32(v)!r}" for v in coeffs))
    print("binary32 gelu: max abs error %.3e, worst error / parity bound %.3f" % check(coeffs))
