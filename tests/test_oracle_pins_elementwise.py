"""Pins for the oracle's element-wise fused kernels (bias + GELU, bias + head split, head merge).

Expected values come from closed forms, a 60-digit series for the normal distribution function, invariants and
library special cases, never from the oracle or the HIP path.
"""
import decimal

import numpy as np
import pytest
import torch

from oracle import turbo_oracle as orc


# ----------------------------------------------------------------- GELU

def _phi_series(x: float) -> float:
    """Phi(x) = 1/2 + (1/sqrt(2 pi)) sum_n (-1)^n x^(2n+1) / (n! 2^n (2n+1)), in 60-digit arithmetic."""
    ctx = decimal.Context(prec=60)
    X = ctx.create_decimal(repr(float(x)))
    term = X  # x^(2n+1) / (n! 2^n)
    total = decimal.Decimal(0)
    for n in range(400):
        total = ctx.add(total, ctx.divide(term, decimal.Decimal(2 * n + 1)) * (1 if n % 2 == 0 else -1))
        term = ctx.divide(ctx.multiply(ctx.multiply(term, X), X), decimal.Decimal(2 * (n + 1)))
        if abs(term) < decimal.Decimal(10) ** -70:
            break
    pi = ctx.create_decimal("3.14159265358979323846264338327950288419716939937510582097494")
    return float(decimal.Decimal("0.5") + ctx.divide(total, ctx.sqrt(2 * pi)))


def test_gelu_textbook_values():
    # Phi(1) and Phi(2) as printed in any normal table, to the table's digits
    y = orc.add_bias_gelu(np.array([[0.0, 1.0, 2.0, -1.0]]), None)[0]
    assert y[0] == 0.0
    assert y[1] == pytest.approx(0.8413447, abs=5e-8)
    assert y[2] == pytest.approx(2 * 0.9772499, abs=2e-7)
    assert y[3] == pytest.approx(-(1 - 0.8413447), abs=5e-8)


def test_gelu_against_60_digit_series():
    t = np.array([-6.0, -3.3, -1.7, -0.4, -1e-3, 1e-3, 0.25, 0.9, 2.2, 4.1, 5.9])
    got = orc.add_bias_gelu(t[None, :], None)[0]
    want = np.array([v * _phi_series(v) for v in t])
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-18)


@pytest.mark.parametrize("approximate", [False, True])
def test_gelu_odd_part_identity_and_limits(approximate):
    rng = np.random.default_rng(0)
    t = rng.normal(size=(7, 33)) * 3
    y = orc.add_bias_gelu(t, None, approximate)
    ym = orc.add_bias_gelu(-t, None, approximate)
    np.testing.assert_allclose(y - ym, t, rtol=1e-13, atol=1e-14)  # t Phi(t) + t Phi(-t) = t
    far = orc.add_bias_gelu(np.array([[40.0, -40.0, 12.0, -12.0]]), None, approximate)[0]
    assert far[0] == 40.0 and far[2] == pytest.approx(12.0, rel=1e-15)
    assert abs(far[1]) < 1e-300 and -1e-30 < far[3] <= 0.0
    assert np.isfinite(far).all()


@pytest.mark.parametrize("approximate,name", [(False, "none"), (True, "tanh")])
def test_gelu_matches_torch_float64(approximate, name):
    rng = np.random.default_rng(1)
    x = rng.normal(size=(19, 50)) * 2
    b = rng.normal(size=50)
    got = orc.add_bias_gelu(x, b, approximate)
    want = torch.nn.functional.gelu(torch.from_numpy(x + b[None, :]), approximate=name).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-15)
    # the two forms are close but not equal: the flag really selects a different formula
    other = orc.add_bias_gelu(x, b, not approximate)
    assert 1e-6 < np.abs(other - got).max() < 1e-2


def test_gelu_bias_is_per_column_and_optional():
    x = np.zeros((3, 4))
    b = np.array([0.0, 1.0, -1.0, 2.0])
    y = orc.add_bias_gelu(x, b)
    assert (y == y[0]).all()
    np.testing.assert_allclose(y[0], orc.add_bias_gelu(b[None, :], None)[0], rtol=0, atol=0)


# ----------------------------------------------------------------- head split / merge

def _coded(shape):
    """A tensor whose every element encodes its own multi-index in mixed radix (exact in float64)."""
    idx = np.indices(shape)
    code = np.zeros(shape)
    for axis, n in enumerate(shape):
        code = code * 10 + idx[axis]
    return code


def test_split_heads_moves_every_element_to_its_place():
    B, S, K, H, D = 2, 5, 3, 4, 6
    x = _coded((B, S, K, H, D))
    out = orc.add_bias_split_heads(x, None)
    assert out.shape == (K, B, H, S, D)
    for k, b, h, s, d in [(0, 0, 0, 0, 0), (2, 1, 3, 4, 5), (1, 0, 2, 3, 1), (2, 1, 0, 4, 0)]:
        assert out[k, b, h, s, d] == ((((b * 10 + s) * 10 + k) * 10 + h) * 10 + d)
    np.testing.assert_array_equal(out, x.transpose(2, 0, 3, 1, 4))


def test_split_heads_adds_bias_along_split_head_and_feature():
    rng = np.random.default_rng(2)
    B, S, K, H, D = 3, 4, 3, 2, 8
    x = rng.normal(size=(B, S, K, H, D))
    bias = rng.normal(size=(K, H, D))
    out = orc.add_bias_split_heads(x, bias)
    want = (x + bias[None, None]).transpose(2, 0, 3, 1, 4)
    np.testing.assert_array_equal(out, want)
    # bias only: every (b, s) sees the same [K,H,D] block
    only = orc.add_bias_split_heads(np.zeros_like(x), bias)
    np.testing.assert_array_equal(only, np.broadcast_to(bias[:, None, :, None, :], (K, B, H, S, D)))


def test_merge_heads_is_the_inverse_permutation():
    B, H, S, D = 2, 3, 5, 4
    x = _coded((B, H, S, D))
    out = orc.merge_heads(x)
    assert out.shape == (B, S, H, D)
    np.testing.assert_array_equal(out, x.transpose(0, 2, 1, 3))
    assert out[1, 4, 2, 3] == ((1 * 10 + 2) * 10 + 4) * 10 + 3
    # split (one projection, no bias) followed by merge is the identity
    y = np.random.default_rng(3).normal(size=(B, S, 1, H, D))
    back = orc.merge_heads(orc.add_bias_split_heads(y, None)[0])
    np.testing.assert_array_equal(back, y[:, :, 0])
