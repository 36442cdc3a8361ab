"""Pins for the CPU oracle: closed forms, invariants, library special cases, high-precision brute force.

None of the expected values here comes from the oracle or from the HIP path.
"""
import decimal
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import turbo_oracle as orc
from paper_2010_05680_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_cases.json")
_ENV = {"log": math.log, "exp": math.exp, "sqrt": math.sqrt, "__builtins__": {}}


def _val(expr):
    return float(eval(expr, _ENV)) if isinstance(expr, str) else float(expr)


def _vals(exprs):
    return None if exprs is None else np.array([_val(e) for e in exprs], dtype=np.float64)


with open(GOLDEN) as fh:
    HAND = json.load(fh)


# ----------------------------------------------------------------- softmax: hand cases

@pytest.mark.parametrize("case", HAND["softmax"], ids=lambda c: c["name"])
def test_softmax_hand_case(case):
    s = _vals(case["scores"])
    m = _vals(case["mask"])
    got = orc.masked_softmax(s.reshape(1, 1, 1, -1), m, 0, 0, case["scale"]).reshape(-1)
    want = _vals(case["expect"])
    np.testing.assert_allclose(got, want, rtol=1e-14, atol=1e-16)
    if case["name"] == "logs_with_masked_key":
        assert got[3] == 0.0  # exactly zero, not merely small


def test_softmax_two_keys_is_logistic():
    rng = np.random.default_rng(1)
    a, b = rng.normal(size=50) * 4, rng.normal(size=50) * 4
    s = np.stack([a, b], -1).reshape(1, 1, 50, 2)
    got = orc.masked_softmax(s, scale=0.7)
    want0 = 1.0 / (1.0 + np.exp(0.7 * (b - a)))
    np.testing.assert_allclose(got[0, 0, :, 0], want0, rtol=1e-13)
    np.testing.assert_allclose(got[0, 0, :, 1], 1.0 - want0, rtol=1e-12, atol=1e-16)


def _decimal_softmax(z):
    ctx = decimal.Context(prec=60)
    zs = [ctx.create_decimal(repr(float(v))) for v in z]
    m = max(zs)
    e = [ctx.exp(ctx.subtract(v, m)) for v in zs]
    tot = sum(e, decimal.Decimal(0))
    return np.array([float(ctx.divide(v, tot)) for v in e])


def test_softmax_against_60_digit_arithmetic():
    rng = np.random.default_rng(2)
    for Sk in (1, 2, 3, 7, 16, 33):
        s = rng.normal(size=Sk) * 3
        a = rng.choice([0.0, -10000.0], size=Sk, p=[0.8, 0.2])
        a[0] = 0.0
        got = orc.masked_softmax(s.reshape(1, 1, 1, Sk), a, 0, 0, 0.125).reshape(-1)
        # scale = 1/8 and the mask values are exact in binary, so z is exact in Decimal too
        want = _decimal_softmax([Fraction(float(v)) / 8 + Fraction(float(m)) for v, m in zip(s, a)])
        np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-300)


# ----------------------------------------------------------------- softmax: invariants

def _cfg0_softmax():
    case = wl.softmax_case(wl.config_spec(0))
    return case, orc.masked_softmax(case.scores, case.mask, case.mask_stride_b, case.mask_stride_q, case.scale)


def test_softmax_rows_sum_to_one_and_lie_in_unit_interval():
    for kind in ("none", "key", "causal", "dense"):
        c = wl.random_softmax_case(11, 3, 2, 9, 37, mask_kind=kind)
        y = orc.masked_softmax(c.scores, c.mask, c.mask_stride_b, c.mask_stride_q, c.scale)
        np.testing.assert_allclose(y.sum(-1), 1.0, rtol=0, atol=1e-12)
        assert (y >= 0).all() and (y <= 1).all()


def test_softmax_masked_entries_are_exactly_zero_cfg0():
    case, y = _cfg0_softmax()
    assert y.shape == (1, 12, 16, 16)
    assert (y[..., 12:] == 0.0).all()
    assert (y[..., :12] > 0.0).all()
    np.testing.assert_allclose(y.sum(-1), 1.0, atol=1e-12)


def test_softmax_masked_entries_zero_for_every_mask_layout():
    for kind in ("key", "causal", "dense"):
        c = wl.random_softmax_case(5, 4, 3, 10, 10, mask_kind=kind)
        y = orc.masked_softmax(c.scores, c.mask, c.mask_stride_b, c.mask_stride_q, c.scale)
        if kind == "key":
            full = np.broadcast_to(c.mask[:, None, None, :], y.shape)
        elif kind == "causal":
            full = np.broadcast_to(c.mask[None, None, :, :], y.shape)
        else:
            full = np.broadcast_to(c.mask[:, None, :, :], y.shape)
        assert (y[full < 0] == 0.0).all()
        assert (y[full == 0] > 0.0).all()


def test_softmax_shift_invariance():
    c = wl.random_softmax_case(3, 2, 2, 5, 19)
    y0 = orc.masked_softmax(c.scores, scale=c.scale)
    shift = np.full((2, 5, 19), 3.25)  # a constant additive "mask" is a shift
    y1 = orc.masked_softmax(c.scores, shift, 5 * 19, 19, c.scale)
    np.testing.assert_allclose(y1, y0, rtol=1e-13)


def test_softmax_order_preserving_and_permutation_equivariant():
    c = wl.random_softmax_case(4, 1, 1, 6, 23)
    s = c.scores.astype(np.float64)
    y = orc.masked_softmax(s, scale=c.scale)
    assert (np.argsort(s, -1, kind="stable") == np.argsort(y, -1, kind="stable")).all()
    perm = np.random.default_rng(0).permutation(23)
    yp = orc.masked_softmax(s[..., perm], scale=c.scale)
    np.testing.assert_allclose(yp, y[..., perm], rtol=1e-13)


def test_softmax_large_scores_do_not_overflow():
    s = np.array([1e4, 1e4 - 1.0, -1e4]).reshape(1, 1, 1, 3)
    y = orc.masked_softmax(s, scale=1.0).reshape(-1)
    e = math.exp(-1.0)
    np.testing.assert_allclose(y, [1 / (1 + e), e / (1 + e), 0.0], rtol=1e-14)


# ----------------------------------------------------------------- softmax: library special case

@pytest.mark.parametrize("kind", ["none", "key", "causal", "dense"])
@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (2, 3, 5, 7), (1, 12, 10, 10), (20, 2, 10, 10), (3, 4, 17, 100)])
def test_softmax_matches_torch_float64(kind, shape):
    B, H, Sq, Sk = shape
    c = wl.random_softmax_case(100 + Sk, B, H, Sq, Sk, mask_kind=kind, scale=0.3)
    got = orc.masked_softmax(c.scores, c.mask, c.mask_stride_b, c.mask_stride_q, c.scale)
    z = torch.from_numpy(c.scores.astype(np.float64)) * c.scale
    if kind == "key":
        z = z + torch.from_numpy(c.mask.astype(np.float64))[:, None, None, :]
    elif kind == "causal":
        z = z + torch.from_numpy(c.mask.astype(np.float64))[None, None, :, :]
    elif kind == "dense":
        z = z + torch.from_numpy(c.mask.astype(np.float64))[:, None, :, :]
    want = torch.softmax(z, dim=-1).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-300)


def test_softmax_fp16_inputs_are_widened_exactly():
    c = wl.random_softmax_case(9, 2, 2, 4, 24, dtype=np.float16, mask_kind="causal")
    got = orc.masked_softmax(c.scores, c.mask, c.mask_stride_b, c.mask_stride_q, c.scale)
    z = torch.from_numpy(c.scores.astype(np.float64)) * c.scale + torch.from_numpy(c.mask.astype(np.float64))
    np.testing.assert_allclose(got, torch.softmax(z, -1).numpy(), rtol=1e-12, atol=1e-300)


# ----------------------------------------------------------------- layernorm: hand cases

@pytest.mark.parametrize("case", HAND["layernorm"], ids=lambda c: c["name"])
def test_layernorm_hand_case(case):
    args = [_vals(case[k]) for k in ("x", "residual", "bias", "gamma", "beta")]
    got = orc.add_bias_layernorm(args[0][None, :], args[1][None, :], args[2], args[3], args[4], case["eps"])[0]
    np.testing.assert_allclose(got, _vals(case["expect"]), rtol=1e-14, atol=1e-15)


def _decimal_layernorm(t, gamma, beta, eps):
    ctx = decimal.Context(prec=60)
    D = lambda v: ctx.create_decimal(repr(float(v)))
    ts = [D(v) for v in t]
    n = decimal.Decimal(len(ts))
    mu = ctx.divide(sum(ts, decimal.Decimal(0)), n)
    var = ctx.divide(sum(((v - mu) * (v - mu) for v in ts), decimal.Decimal(0)), n)
    sd = ctx.sqrt(var + D(eps))
    return np.array([float(ctx.divide(v - mu, sd) * D(g) + D(b)) for v, g, b in zip(ts, gamma, beta)])


def test_layernorm_against_60_digit_arithmetic():
    rng = np.random.default_rng(3)
    for hidden in (2, 3, 8, 31, 64):
        x, r = rng.normal(size=hidden), rng.normal(size=hidden)
        b, g, be = rng.normal(size=hidden) * .1, 1 + rng.normal(size=hidden) * .1, rng.normal(size=hidden) * .1
        # make t exactly representable so both sides start from the same t
        x, r, b = (np.round(v * 1024) / 1024 for v in (x, r, b))
        got = orc.add_bias_layernorm(x[None], r[None], b, g, be, 1e-5)[0]
        want = _decimal_layernorm(x + b + r, g, be, 1e-5)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)


# ----------------------------------------------------------------- layernorm: invariants

def test_layernorm_pre_affine_output_has_mean_zero_and_unit_variance():
    c = wl.layernorm_case(wl.config_spec(0))
    ones, zeros = np.ones(768), np.zeros(768)
    y = orc.add_bias_layernorm(c.x, c.residual, c.bias, ones, zeros, c.eps)
    assert y.shape == (16, 768)
    np.testing.assert_allclose(y.mean(-1), 0.0, atol=1e-12)
    np.testing.assert_allclose(y.var(-1), 1.0, rtol=1e-9)
    # with a visible eps the variance is var/(var+eps)
    t = c.x.astype(np.float64) + c.bias.astype(np.float64) + c.residual.astype(np.float64)
    y2 = orc.add_bias_layernorm(c.x, c.residual, c.bias, ones, zeros, 0.5)
    np.testing.assert_allclose(y2.var(-1), t.var(-1) / (t.var(-1) + 0.5), rtol=1e-12)


def test_layernorm_affine_input_invariance_and_symmetries():
    c = wl.random_layernorm_case(8, 5, 96)
    x, r, b, g, be = (v.astype(np.float64) for v in (c.x, c.residual, c.bias, c.gamma, c.beta))
    base = orc.add_bias_layernorm(x, r, b, g, be, 0.0)
    # LN(a*t + c) = LN(t) for a > 0 when eps = 0
    np.testing.assert_allclose(orc.add_bias_layernorm(2.5 * x + 4.0, 2.5 * r, 2.5 * b, g, be, 0.0), base,
                               rtol=1e-11, atol=1e-12)
    # x and residual are interchangeable; bias can be folded into x; NULL means zero
    np.testing.assert_allclose(orc.add_bias_layernorm(r, x, b, g, be, 0.0), base, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(orc.add_bias_layernorm(x + b, r, None, g, be, 0.0), base, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(orc.add_bias_layernorm(x + b + r, None, None, g, be, 0.0), base, rtol=1e-12,
                               atol=1e-14)
    # negating the input negates the normalised part
    np.testing.assert_allclose(orc.add_bias_layernorm(-x, -r, -b, g, be, 0.0) - be, -(base - be), rtol=1e-12,
                               atol=1e-14)
    # gamma and beta act per column after normalisation
    plain = orc.add_bias_layernorm(x, r, b, np.ones(96), np.zeros(96), 0.0)
    np.testing.assert_allclose(base, plain * g + be, rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("shape", [(1, 1), (1, 2), (7, 5), (16, 768), (3, 1000), (2, 4096)])
@pytest.mark.parametrize("eps", [1e-12, 1e-5])
def test_layernorm_matches_torch_float64(shape, eps):
    rows, hidden = shape
    c = wl.random_layernorm_case(200 + hidden, rows, hidden)
    got = orc.add_bias_layernorm(c.x, c.residual, c.bias, c.gamma, c.beta, eps)
    T = lambda a: torch.from_numpy(a.astype(np.float64))
    want = torch.nn.functional.layer_norm(T(c.x) + T(c.bias) + T(c.residual), (hidden,), T(c.gamma), T(c.beta), eps)
    if hidden == 1:
        np.testing.assert_allclose(got, np.broadcast_to(c.beta.astype(np.float64), (rows, 1)), atol=1e-15)
    else:
        np.testing.assert_allclose(got, want.numpy(), rtol=1e-11, atol=1e-13)


def test_layernorm_rows_are_independent():
    c = wl.random_layernorm_case(12, 6, 40)
    full = orc.add_bias_layernorm(c.x, c.residual, c.bias, c.gamma, c.beta, 1e-5)
    for r in (0, 3, 5):
        one = orc.add_bias_layernorm(c.x[r:r + 1], c.residual[r:r + 1], c.bias, c.gamma, c.beta, 1e-5)
        np.testing.assert_array_equal(one[0], full[r])


# ----------------------------------------------------------------- Equation 1

def test_equation_1_three_variance_algorithms_agree():
    rng = np.random.default_rng(4)
    for n in (1, 2, 5, 768, 4096):
        x = rng.normal(size=n) * 1.4 + 0.3
        ref = float(np.var(x))
        for f in (orc.variance_two_pass, orc.variance_sum_of_squares, orc.variance_welford):
            assert f(x) == pytest.approx(ref, rel=1e-11, abs=1e-14)
    assert orc.variance_two_pass([1, 2, 3, 4]) == 1.25  # population (divide by n), not sample, variance


def test_equation_1_second_form_cancels_when_mean_dominates():
    # The E(x^2) - E^2(x) form loses digits once |mean| >> std; Welford and two-pass do not.
    x = 1e8 + np.array([0.0, 1.0, 2.0, 3.0])
    assert orc.variance_two_pass(x) == 1.25
    assert orc.variance_welford(x) == pytest.approx(1.25, rel=1e-12)
    assert abs(orc.variance_sum_of_squares(x) - 1.25) > 0.1


def test_welford_merge_equals_whole_row():
    rng = np.random.default_rng(5)
    x = rng.normal(size=100) + 2
    for cut in (0, 1, 37, 64, 100):
        a, b = x[:cut], x[cut:]
        sa = (len(a), a.mean() if len(a) else 0.0, ((a - a.mean()) ** 2).sum() if len(a) else 0.0)
        sb = (len(b), b.mean() if len(b) else 0.0, ((b - b.mean()) ** 2).sum() if len(b) else 0.0)
        n, mean, m2 = orc.welford_merge(sa, sb)
        assert n == 100
        assert mean == pytest.approx(x.mean(), rel=1e-13)
        assert m2 / n == pytest.approx(x.var(), rel=1e-12)


# ----------------------------------------------------------------- workloads

def test_config_shapes_follow_the_stated_workloads():
    s2 = wl.config_spec(2)
    assert s2.lengths.shape == (32,) and s2.lengths.min() >= 5 and s2.lengths.max() <= 500
    assert s2.Sk == s2.lengths.max() and s2.rows == 32 * s2.Sk
    c0 = wl.softmax_case(wl.config_spec(0))
    assert c0.scores.shape == (1, 12, 16, 16) and (c0.mask[0, 12:] == -10000).all() and (c0.mask[0, :12] == 0).all()
    c = wl.causal_mask(4, 4, np.float16)
    iu = np.triu_indices(4, 1)
    assert c.dtype == np.float16 and (c[iu] == -10000).all() and (np.tril(c) == 0).all() and c.sum() == -60000
    a, b = wl.softmax_case(wl.config_spec(0)), wl.softmax_case(wl.config_spec(0))
    np.testing.assert_array_equal(a.scores, b.scores)  # seeded: identical on every call


def test_oracle_threads_do_not_change_results():
    c = wl.random_softmax_case(6, 2, 3, 16, 50, mask_kind="key")
    orc.set_threads(1)
    y1 = orc.masked_softmax(c.scores, c.mask, c.mask_stride_b, c.mask_stride_q, c.scale)
    orc.set_threads(4)
    y4 = orc.masked_softmax(c.scores, c.mask, c.mask_stride_b, c.mask_stride_q, c.scale)
    orc.set_threads(1)
    np.testing.assert_array_equal(y1, y4)


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The oracle is the reference everything else is judged by, so its own memory accesses are checked: every
    function runs on exactly sized heap buffers in a build with -fsanitize=address,undefined (tests/native/oracle_sanitize.c)."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = tmp_path / "oracle_sanitize"
    subprocess.check_call(["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
                           os.path.join(root, "tests", "native", "oracle_sanitize.c"), "-o", str(exe), "-lm"])
    res = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300,
                         env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))
    assert res.returncode == 0 and res.stdout.startswith("ok"), res.stdout + res.stderr
