"""Derives the coefficients of the branch-free normal-tail approximation used by gelu_erf() in elementwise_kernels.h.

    Phi(-u) ~= 2^Q(u),   Q a polynomial of degree n,   0 <= u <= 8        (Phi = standard normal CDF)
    gelu(t) = t Phi(t) = max(t, 0) - |t| Phi(-|t|)   (the kernel clamps |t| to 8 in both factors)

log2 Phi(-u) is smooth and nearly quadratic, so a low degree reaches the accuracy the storage type can show:
degree 5 for binary16 outputs, degree 8 for binary32.  Q is fitted by iteratively re-weighted least squares (a Lawson
iteration towards the minimax error), each sample weighted by what an error in Q costs against the parity bound
max(1e-6, rtol |gelu|).  The script then evaluates the kernel's binary32 evaluation order against the double-precision
definition and prints the worst error relative to that bound.  Run it to regenerate or to check the constants;
nothing imports it.
"""
import numpy as np
from scipy.special import log_ndtr, ndtr

LOG2E = 1.4426950408889634
U_MAX = 8.0  # |t| is clamped here: 8 Phi(-8) < 1e-14, far below the absolute bound


def fit(degree, rtol, iters=100):
    u = np.concatenate([np.linspace(0, 5.6, 8000), np.linspace(5.6, U_MAX, 800)])
    q = log_ndtr(-u) * LOG2E
    basis = np.stack([u ** k for k in range(degree + 1)], 1)
    tail = u * ndtr(-u)  # |gelu(-u)|; an error dQ moves both gelu(-u) and gelu(u) by tail * ln 2 * dQ
    cost = np.log(2) * np.maximum(tail / np.maximum(1e-6, rtol * tail), tail / np.maximum(1e-6, rtol * u * ndtr(u))) + 1e-3
    weight = np.ones_like(u)
    for _ in range(iters):
        w = weight * cost
        c, *_ = np.linalg.lstsq(basis * w[:, None], q * w, rcond=None)
        err = np.abs((basis @ c - q) * cost)
        weight = weight * (1 + 5 * err / err.max())
        weight /= weight.mean()
    return c


def kernel_order(c, t):
    """binary32 evaluation as in the kernel: Horner with fused multiply-adds, exp2, one final fused multiply-add."""
    f = np.float32
    fma = lambda a, b, d: (a.astype(np.float64) * b.astype(np.float64) + np.float64(d)).astype(f)
    u = np.minimum(np.abs(t), f(U_MAX))
    p = np.full_like(t, f(c[-1]))
    for ck in c[-2::-1]:
        p = fma(p, u, f(ck))
    e = np.exp2(p)
    return (np.maximum(t, f(0)).astype(np.float64) - u.astype(np.float64) * e.astype(np.float64)).astype(f)


def check(c, rtol, to_half):
    worst = 0.0
    half = np.arange(65536, dtype=np.uint16).view(np.float16)
    for t in (half[np.isfinite(half)].astype(np.float32), np.linspace(-12, 12, 4000001).astype(np.float32)):
        got = kernel_order(c, t)
        if to_half:
            with np.errstate(over="ignore"):
                got = got.astype(np.float16)
            keep = np.isfinite(got)
            got, t = got[keep], t[keep]
        t64 = t.astype(np.float64)
        want = t64 * ndtr(t64)
        worst = max(worst, (np.abs(got.astype(np.float64) - want) / np.maximum(1e-6, rtol * np.abs(want))).max())
    return worst


if __name__ == "__main__":
    for name, degree, rtol, to_half in (("binary16 storage", 5, 3e-3, True), ("binary32 storage", 8, 1e-5, False)):
        coeffs = fit(degree, rtol)
        print(f"{name}: degree {degree}, c_0..c_{degree} (binary32):")
        print("   ", ", ".join(f"{np.float32(v)!r}" for v in coeffs))
        print("    worst error / parity bound (rtol %g, atol 1e-6): %.3f" % (rtol, check(coeffs, rtol, to_half)))
