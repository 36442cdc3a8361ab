"""Parity of the HIP path (through the C ABI) against the CPU oracle.

Bar: |gpu - oracle| <= max(atol, rtol*|oracle|) with (rtol, atol) = (1e-5, 1e-6) for binary32 and
(3e-3, 1e-6) for binary16 storage, element by element (conftest.assert_parity).
"""
import os

import numpy as np
import pytest
import torch

from paper_2010_05680_amd import binding as tb
from paper_2010_05680_amd import workloads as wl

from conftest import assert_parity, layernorm_bound_scale
import gpu_util as gu

pytestmark = pytest.mark.gpu

F32, F16 = np.float32, np.float16


def _np(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


# ------------------------------------------------------------------ the five configurations

@pytest.mark.parametrize("idx", [0, 1])
def test_softmax_small_configs_full_parity(idx):
    case = wl.softmax_case(wl.config_spec(idx))
    got = _np(gu.run_softmax(case))
    err = assert_parity(got, gu.oracle_softmax(case), case.scores.dtype, f"softmax cfg{idx}")
    print(f"error report: softmax cfg{idx} (all elements): max abs {err[0]:.3e}, max rel {err[1]:.3e}, {100 * err[2]:.0f} % of the bound", flush=True)


@pytest.mark.parametrize("idx", [0, 1])
def test_layernorm_small_configs_full_parity(idx):
    case = wl.layernorm_case(wl.config_spec(idx))
    got = _np(gu.run_layernorm(case))
    err = assert_parity(got, gu.oracle_layernorm(case), case.x.dtype, f"layernorm cfg{idx}")
    print(f"error report: layernorm cfg{idx} (all elements): max abs {err[0]:.3e}, max rel {err[1]:.3e}, {100 * err[2]:.0f} % of the bound", flush=True)


@pytest.mark.parametrize("idx", [2, 3, 4])
def test_softmax_full_size_configs_sampled_rows_and_invariants(idx):
    spec = wl.config_spec(idx)
    case = wl.softmax_case(spec)
    print(f"softmax cfg{idx} shape {case.shape} dtype {case.scores.dtype}", flush=True)
    out = gu.run_softmax(case)
    B, H, Sq, Sk = case.shape
    n_rows = B * H * Sq
    rows = gu.sample_rows(n_rows, 600, seed=idx)
    got = _np(out.view(n_rows, Sk)[torch.from_numpy(rows).cuda()])
    err = assert_parity(got, gu.oracle_softmax_rows(case, rows), case.scores.dtype, f"softmax cfg{idx} sampled rows")
    print(f"error report: softmax cfg{idx} ({len(rows)} sampled rows): max abs {err[0]:.3e}, max rel {err[1]:.3e}, {100 * err[2]:.0f} % of the bound", flush=True)
    # properties that hold at any size, checked on every row
    sums = out.view(n_rows, Sk).float().sum(-1)
    tol = 1e-5 if case.scores.dtype == F32 else 2e-3
    assert torch.isfinite(out).all()
    assert (sums - 1).abs().max().item() < tol
    assert out.min().item() >= 0.0 and out.max().item() <= 1.0
    if case.mask_kind == "key":
        k = torch.arange(Sk, device="cuda")[None, :]
        dead = (k >= torch.from_numpy(case.lengths).cuda()[:, None])[:, None, None, :].expand(B, H, Sq, Sk)
        assert (out[dead] == 0).all()
    if case.mask_kind == "causal":
        dead = torch.triu(torch.ones(Sq, Sk, dtype=torch.bool, device="cuda"), 1)
        assert (out[:, :, dead] == 0).all()


@pytest.mark.parametrize("idx", [2, 3, 4])
def test_layernorm_full_size_configs_sampled_rows_and_invariants(idx):
    spec = wl.config_spec(idx)
    case = wl.layernorm_case(spec)
    print(f"layernorm cfg{idx} shape {case.shape} dtype {case.x.dtype}", flush=True)
    out = gu.run_layernorm(case)
    rows = gu.sample_rows(spec.rows, 600, seed=10 + idx)
    got = _np(out[torch.from_numpy(rows).cuda()])
    err = assert_parity(got, gu.oracle_layernorm(case, rows=rows), case.x.dtype, f"layernorm cfg{idx} sampled rows")
    print(f"error report: layernorm cfg{idx} ({len(rows)} sampled rows): max abs {err[0]:.3e}, max rel {err[1]:.3e}, {100 * err[2]:.0f} % of the bound", flush=True)
    assert torch.isfinite(out).all()
    # undo the affine part on the device: mean 0, variance 1 per row
    g, b = gu.dev(case.gamma).float(), gu.dev(case.beta).float()
    y = (out.float() - b) / g
    tol = 1e-4 if case.x.dtype == F32 else 2e-2
    assert y.mean(-1).abs().max().item() < tol
    assert (y.var(-1, unbiased=False) - 1).abs().max().item() < 10 * tol


# ------------------------------------------------------------------ shape sweeps (full oracle)

TABLE2_GRID = [(1, 10), (1, 100), (1, 500), (20, 10), (20, 100), (20, 500)]


@pytest.mark.parametrize("batch,seq", TABLE2_GRID)
@pytest.mark.parametrize("dtype", [F32, F16])
def test_softmax_table2_grid(batch, seq, dtype):
    H = 12 if batch * seq < 5000 else 3
    case = wl.random_softmax_case(1000 + batch * seq, batch, H, seq, seq, dtype=dtype, mask_kind="key")
    got = _np(gu.run_softmax(case))
    assert_parity(got, gu.oracle_softmax(case), dtype, f"softmax ({batch},{seq})")


@pytest.mark.parametrize("batch,seq", TABLE2_GRID)
@pytest.mark.parametrize("dtype", [F32, F16])
def test_layernorm_table2_grid(batch, seq, dtype):
    case = wl.random_layernorm_case(2000 + batch * seq, batch * seq, 768, dtype=dtype)
    got = _np(gu.run_layernorm(case))
    assert_parity(got, gu.oracle_layernorm(case), dtype, f"layernorm ({batch},{seq})")


RAGGED_SK = [1, 2, 3, 4, 5, 7, 8, 15, 16, 17, 31, 33, 63, 64, 65, 100, 127, 129, 255, 257, 497, 498, 500, 513, 1000,
             1023, 1025, 2047, 2052, 4099]


@pytest.mark.parametrize("wide", [True, False], ids=["element-aligned-wide", "aligned-narrow"])
@pytest.mark.parametrize("dtype", [F32, F16])
@pytest.mark.parametrize("kind", ["none", "key", "causal", "dense"])
def test_softmax_ragged_row_lengths(dtype, kind, wide):
    """Row lengths that are not multiples of the vector width: by default 16-byte accesses at element
    alignment with an overlapping last vector; with a width cap, the aligned 2/4/8-byte kernels."""
    with gu.overrides(max_vec_bytes=-1 if wide else 16):
        for Sk in RAGGED_SK:
            Sq = Sk if kind == "causal" and Sk <= 129 else 5
            if kind == "causal" and Sq != Sk:
                continue
            case = wl.random_softmax_case(300 + Sk, 3, 2, Sq, Sk, dtype=dtype, mask_kind=kind)
            got = _np(gu.run_softmax(case))
            assert_parity(got, gu.oracle_softmax(case), dtype, f"softmax Sk={Sk} {kind}")


RAGGED_HIDDEN = [1, 2, 3, 5, 8, 9, 63, 64, 100, 255, 256, 257, 768, 771, 1000, 1024, 1027, 1536, 1540, 2048, 3001, 4096, 4100, 4101,
                 6144, 6147, 8000, 8190, 8192, 12288, 16000, 16382, 16384, 16388]


@pytest.mark.parametrize("wide", [True, False], ids=["element-aligned-wide", "aligned-narrow"])
@pytest.mark.parametrize("dtype", [F32, F16])
def test_layernorm_ragged_hidden_sizes(dtype, wide):
    with gu.overrides(max_vec_bytes=-1 if wide else 16):
        for hidden in RAGGED_HIDDEN:
            rows = 37 if hidden < 2000 else 9
            case = wl.random_layernorm_case(400 + hidden, rows, hidden, dtype=dtype, eps=1e-5)
            if hidden == 1:
                continue  # a single column has zero variance: the result is eps-dominated, see the dedicated test
            got = _np(gu.run_layernorm(case))
            assert_parity(got, gu.oracle_layernorm(case), dtype, f"layernorm hidden={hidden}")


# ------------------------------------------------------------------ every kernel family and vector width

@pytest.mark.parametrize("path", [tb.PATH_WAVE, tb.PATH_BLOCK, tb.PATH_STREAM])
@pytest.mark.parametrize("dtype", [F32, F16])
def test_softmax_forced_families(path, dtype):
    for Sk, kind in [(16, "key"), (64, "none"), (257, "dense"), (1000, "key"), (1001, "key"), (2048, "none"),
                     (4096, "key"), (5001, "none")]:
        case = wl.random_softmax_case(500 + Sk, 2, 3, 7, Sk, dtype=dtype, mask_kind=kind)
        with gu.overrides(path=path):
            got = _np(gu.run_softmax(case))
        assert_parity(got, gu.oracle_softmax(case), dtype, f"softmax path={path} Sk={Sk}")


@pytest.mark.parametrize("path", [tb.PATH_WAVE, tb.PATH_BLOCK, tb.PATH_STREAM])
@pytest.mark.parametrize("dtype", [F32, F16])
def test_layernorm_forced_families(path, dtype):
    for hidden in (8, 64, 300, 301, 768, 1024, 2048, 2049, 4096, 5001):
        case = wl.random_layernorm_case(600 + hidden, 19, hidden, dtype=dtype, eps=1e-5)
        with gu.overrides(path=path):
            got = _np(gu.run_layernorm(case))
        assert_parity(got, gu.oracle_layernorm(case), dtype, f"layernorm path={path} hidden={hidden}")


@pytest.mark.parametrize("vec_bytes", [2, 4, 8, 16])
@pytest.mark.parametrize("dtype", [F32, F16])
def test_every_vector_width(vec_bytes, dtype):
    if vec_bytes < np.dtype(dtype).itemsize:
        pytest.skip("narrower than one element")
    with gu.overrides(max_vec_bytes=vec_bytes):
        for Sk in (64, 512, 1024):
            case = wl.random_softmax_case(700 + Sk, 2, 2, 33, Sk, dtype=dtype, mask_kind="key")
            assert_parity(_np(gu.run_softmax(case)), gu.oracle_softmax(case), dtype, f"softmax vec={vec_bytes} Sk={Sk}")
        for hidden in (64, 768, 1024):
            case = wl.random_layernorm_case(800 + hidden, 45, hidden, dtype=dtype, eps=1e-5)
            assert_parity(_np(gu.run_layernorm(case)), gu.oracle_layernorm(case), dtype,
                          f"layernorm vec={vec_bytes} hidden={hidden}")


def test_long_rows_block_and_stream_families():
    for Sk in (8192, 32768, 40000, 70001):
        case = wl.random_softmax_case(900 + Sk, 1, 2, 3, Sk, mask_kind="key", score_std=5.0)
        assert_parity(_np(gu.run_softmax(case)), gu.oracle_softmax(case), F32, f"softmax Sk={Sk}")
    for hidden in (8192, 16384, 20000, 65537):
        case = wl.random_layernorm_case(950 + hidden, 5, hidden, eps=1e-5)
        assert_parity(_np(gu.run_layernorm(case)), gu.oracle_layernorm(case), F32, f"layernorm hidden={hidden}")
    case = wl.random_softmax_case(990, 1, 1, 3, 40000, dtype=F16, mask_kind="none")
    assert_parity(_np(gu.run_softmax(case)), gu.oracle_softmax(case), F16, "softmax f16 Sk=40000")
    case = wl.random_layernorm_case(991, 3, 40000, dtype=F16, eps=1e-5)
    assert_parity(_np(gu.run_layernorm(case)), gu.oracle_layernorm(case), F16, "layernorm f16 hidden=40000")


@pytest.mark.parametrize("dtype", [F32, F16])
def test_rows_around_the_lds_row_cache_of_the_stream_family(dtype):
    """The stream family parks the first 128 KB of a row in LDS between its two sweeps and reads the rest twice.
    Row lengths on both sides of that boundary, with every size of leftover group of vectors in both parts."""
    es = np.dtype(dtype).itemsize
    vec = 16 // es
    cached = (128 * 1024) // es           # softmax: columns that wait in LDS
    chunk = 1024 * vec                    # columns one pass of the workgroup covers
    lengths = [cached + vec, cached + chunk + vec, cached + 2 * chunk + 3 * vec, cached + 3 * chunk, cached + 4 * chunk + vec,
               cached - chunk + vec, cached + 1, cached + 7 * vec + 2]
    for n, Sk in enumerate(lengths):
        for mask_kind in ("none", "key"):
            case = wl.random_softmax_case(1200 + n, 1, 1, 2, Sk, dtype=dtype, mask_kind=mask_kind, score_std=4.0)
            with gu.overrides(path=tb.PATH_STREAM):
                got = _np(gu.run_softmax(case))
            assert_parity(got, gu.oracle_softmax(case), dtype, f"softmax {np.dtype(dtype).name} Sk={Sk} mask={mask_kind}")
    ln_cached = 32768                     # LayerNorm: columns of t (binary32) that wait in LDS
    for n, hidden in enumerate([ln_cached + vec, ln_cached + chunk + vec, ln_cached + 2 * chunk + 3 * vec, ln_cached + 3 * chunk,
                                ln_cached - chunk + vec, ln_cached + 1, 3 * ln_cached + 5 * vec]):
        case = wl.random_layernorm_case(1300 + n, 3, hidden, dtype=dtype, eps=1e-5)
        with gu.overrides(path=tb.PATH_STREAM):
            got = _np(gu.run_layernorm(case))
        assert_parity(got, gu.oracle_layernorm(case), dtype, f"layernorm {np.dtype(dtype).name} hidden={hidden}")


def test_small_grid_makes_workgroups_loop_over_tiles():
    with gu.overrides(grid_waves=1):
        case = wl.softmax_case(wl.config_spec(1))
        assert_parity(_np(gu.run_softmax(case)), gu.oracle_softmax(case), F32, "softmax cfg1, 1 workgroup per CU")
        lc = wl.layernorm_case(wl.config_spec(1))
        assert_parity(_np(gu.run_layernorm(lc)), gu.oracle_layernorm(lc), F32, "layernorm cfg1, 1 workgroup per CU")
        for path in (tb.PATH_BLOCK, tb.PATH_STREAM):
            with gu.overrides(path=path, grid_waves=1):
                c = wl.random_softmax_case(77, 2, 2, 700, 300, mask_kind="causal" if False else "key")
                assert_parity(_np(gu.run_softmax(c)), gu.oracle_softmax(c), F32, f"softmax looped path={path}")
                l2 = wl.random_layernorm_case(78, 3000, 300, eps=1e-5)
                assert_parity(_np(gu.run_layernorm(l2)), gu.oracle_layernorm(l2), F32, f"layernorm looped path={path}")


# ------------------------------------------------------------------ edge cases

def test_softmax_base_entry_point_takes_dense_mask():
    case = wl.random_softmax_case(31, 3, 4, 9, 40, mask_kind="dense")
    s, m = gu.dev(case.scores), gu.dev(case.mask)
    tb.turbo_masked_softmax(s, m, case.scale)
    torch.cuda.synchronize()
    assert_parity(_np(s), gu.oracle_softmax(case), F32, "dense mask entry point")
    case = wl.random_softmax_case(32, 3, 4, 9, 40, mask_kind="none")
    s = gu.dev(case.scores)
    tb.turbo_masked_softmax(s, None, case.scale)
    torch.cuda.synchronize()
    assert_parity(_np(s), gu.oracle_softmax(case), F32, "NULL mask")


@pytest.mark.parametrize("dtype", [F32, F16])
def test_unaligned_base_pointers_and_guard_bands(dtype):
    """Tensors that start 1 element past a 16-byte boundary, inside NaN-filled buffers that must stay untouched."""
    tdt = torch.float32 if dtype == F32 else torch.float16
    for Sk in (16, 128, 500, 4096):
        case = wl.random_softmax_case(40 + Sk, 2, 2, 11, Sk, dtype=dtype, mask_kind="key")
        n = case.scores.size
        buf = torch.full((n + 64,), float("nan"), dtype=tdt, device="cuda")
        view = buf[33:33 + n].view(case.scores.shape)
        view.copy_(torch.from_numpy(case.scores))
        mbuf = torch.full((case.mask.size + 9,), float("nan"), dtype=tdt, device="cuda")
        mview = mbuf[5:5 + case.mask.size].view(case.mask.shape)
        mview.copy_(torch.from_numpy(case.mask))
        tb.turbo_masked_softmax_ex(view, mview, case.mask_stride_b, case.mask_stride_q, case.scale)
        torch.cuda.synchronize()
        assert_parity(_np(view), gu.oracle_softmax(case), dtype, f"softmax offset view Sk={Sk}")
        assert torch.isnan(buf[:33]).all() and torch.isnan(buf[33 + n:]).all(), "softmax wrote outside its tensor"
    for hidden in (64, 768, 1000, 4096):
        case = wl.random_layernorm_case(60 + hidden, 13, hidden, dtype=dtype, eps=1e-5)
        n = case.x.size
        obuf = torch.full((n + 64,), float("nan"), dtype=tdt, device="cuda")
        out = obuf[31:31 + n].view(case.x.shape)
        xbuf = torch.zeros(n + 8, dtype=tdt, device="cuda")
        x = xbuf[3:3 + n].view(case.x.shape)
        x.copy_(torch.from_numpy(case.x))
        tb.turbo_add_bias_layernorm_dt(x, gu.dev(case.residual), gu.dev(case.bias), gu.dev(case.gamma),
                                       gu.dev(case.beta), case.eps, out)
        torch.cuda.synchronize()
        assert_parity(_np(out), gu.oracle_layernorm(case), dtype, f"layernorm offset view hidden={hidden}")
        assert torch.isnan(obuf[:31]).all() and torch.isnan(obuf[31 + n:]).all(), "layernorm wrote outside its tensor"


@pytest.mark.parametrize("dtype", [F32, F16])
def test_softmax_key_mask_read_once_per_wavefront_for_unaligned_rows(dtype):
    """Rows that are not 16-byte aligned read a per-request key mask (query stride 0) once for all rows a wavefront
    holds, when those rows belong to one request.  Requests of 1, 3, 5 and 16 rows make wavefronts straddle requests
    (no sharing there), larger ones do not; every request has its own mask, so a mask taken from the wrong request
    shows."""
    seed = 9700
    for Sk in (7, 33, 77, 129, 197, 255, 333, 493, 777, 1001):
        for B, H, Sq in ((9, 1, 1), (7, 1, 3), (5, 1, 5), (4, 2, 8), (3, 2, 33), (2, 3, 64)):
            seed += 1
            case = wl.random_softmax_case(seed, B, H, Sq, Sk, dtype=dtype, mask_kind="key")
            what = f"key mask, unaligned rows: Sk={Sk} B={B} H={H} Sq={Sq}"
            assert_parity(_np(gu.run_softmax(case)), gu.oracle_softmax(case), dtype, what)


def test_layernorm_optional_inputs_and_aliasing():
    case = wl.random_layernorm_case(70, 50, 768, eps=1e-5)
    for residual, bias in [(True, False), (False, True), (False, False)]:
        got = _np(gu.run_layernorm(case, residual=residual, bias=bias))
        assert_parity(got, gu.oracle_layernorm(case, residual=residual, bias=bias), F32,
                      f"layernorm residual={residual} bias={bias}")
    want = gu.oracle_layernorm(case)
    x, r = gu.dev(case.x), gu.dev(case.residual)
    args = (gu.dev(case.bias), gu.dev(case.gamma), gu.dev(case.beta), case.eps)
    tb.turbo_add_bias_layernorm(x, r, *args, x)  # out aliases x
    torch.cuda.synchronize()
    assert_parity(_np(x), want, F32, "layernorm out == x")
    x = gu.dev(case.x)
    tb.turbo_add_bias_layernorm(x, r, *args, r)  # out aliases residual
    torch.cuda.synchronize()
    assert_parity(_np(r), want, F32, "layernorm out == residual")


@pytest.mark.parametrize("path,hidden", [(tb.PATH_WAVE, 1000), (tb.PATH_BLOCK, 4100), (tb.PATH_BLOCK, 12288), (tb.PATH_STREAM, 20000),
                                         (tb.PATH_STREAM, 771)])
@pytest.mark.parametrize("dtype", [F32, F16])
def test_layernorm_in_place_in_every_family(path, hidden, dtype):
    """out == x and out == residual must work whichever kernel family serves the row length: the workgroup-per-row
    kernels prefetch the next row before they store the current one, the two-sweep kernels read every row twice."""
    case = wl.random_layernorm_case(75 + hidden, 37, hidden, dtype=dtype, eps=1e-5)
    want = gu.oracle_layernorm(case)
    args = (gu.dev(case.bias), gu.dev(case.gamma), gu.dev(case.beta), case.eps)
    with gu.overrides(path=path):
        x, r = gu.dev(case.x), gu.dev(case.residual)
        tb.turbo_add_bias_layernorm_dt(x, r, *args, x)
        torch.cuda.synchronize()
        assert_parity(_np(x), want, dtype, f"layernorm out == x, path {path}, hidden {hidden}")
        x = gu.dev(case.x)
        tb.turbo_add_bias_layernorm_dt(x, r, *args, r)
        torch.cuda.synchronize()
        assert_parity(_np(r), want, dtype, f"layernorm out == residual, path {path}, hidden {hidden}")


def test_layernorm_zero_rows_give_beta_and_single_column():
    case = wl.random_layernorm_case(71, 8, 256, eps=1e-5)
    case.x[:] = 0
    case.residual[:] = 0
    case.bias[:] = 0
    got = _np(gu.run_layernorm(case))
    np.testing.assert_array_equal(got, np.broadcast_to(case.beta, got.shape))
    one = wl.random_layernorm_case(72, 6, 1, eps=1e-5)
    got = _np(gu.run_layernorm(one))
    np.testing.assert_allclose(got, np.broadcast_to(one.beta, got.shape), rtol=0, atol=1e-6)


@pytest.mark.parametrize("path", [-1, 1, 2], ids=["planned", "block", "stream"])
def test_layernorm_mean_far_from_zero_keeps_its_digits(path):
    """Rows with |mean| = 1000 standard deviations: the case that separates the one-pass algorithms of Equation 1.

    The inputs are exact for both sides (x alone, no bias or residual, so nothing is rounded before the statistics).
    binary32 cannot hold the 1e-5 bar here: the mean itself is only known to ulp(1000) = 6.1e-5, which moves every
    normalised output by up to that much in units of the standard deviation.  The bound used is 8 ulp(1000) ~ 5e-4
    absolute on outputs of order one.  E(x^2) - E(x)^2 in binary32 would miss it by two orders of magnitude: it
    subtracts two numbers near 1e6 whose ulp is 0.06 to get a variance of 1.
    """
    for hidden in (768, 1024, 4100):
        case = wl.random_layernorm_case(73 + hidden, 64, hidden, eps=1e-5)
        case.x[:] = (case.x + np.float32(1000.0)).astype(F32)
        case.gamma[:] = 1
        case.beta[:] = 0
        with gu.overrides(path=path):
            got = _np(gu.run_layernorm(case, residual=False, bias=False)).astype(np.float64)
        want = gu.oracle_layernorm(case, residual=False, bias=False)
        err = np.abs(got - want).max()
        assert err < 8 * 6.1e-5, f"hidden={hidden}: max abs error {err:.2e}"
        # the naive one-pass form, evaluated in binary32 on the same rows, is far outside that bound
        x32 = case.x
        naive_var = (x32 * x32).mean(-1, dtype=F32) - x32.mean(-1, dtype=F32) ** 2
        naive = (x32 - x32.mean(-1, dtype=F32)[:, None]) / np.sqrt(np.maximum(naive_var, 0) + F32(1e-5))[:, None]
        assert np.abs(naive - want).max() > 20 * err


def test_softmax_degenerate_rows():
    # single key: weight 1 whatever the score
    case = wl.random_softmax_case(80, 2, 3, 4, 1)
    np.testing.assert_array_equal(_np(gu.run_softmax(case)), np.ones(case.shape, F32))
    # equal scores: uniform weights
    case = wl.random_softmax_case(81, 1, 1, 3, 48)
    case.scores[:] = 2.5
    np.testing.assert_allclose(_np(gu.run_softmax(case)), 1.0 / 48, rtol=1e-6)
    # large scores must not overflow
    case = wl.random_softmax_case(82, 1, 2, 5, 100, score_std=3000.0, scale=1.0)
    assert_parity(_np(gu.run_softmax(case)), gu.oracle_softmax(case), F32, "softmax with |z| in the thousands")


@pytest.mark.parametrize("path", [tb.PATH_BLOCK, tb.PATH_STREAM], ids=["block", "stream"])
@pytest.mark.parametrize("Sk", [2048, 4096, 20000])
def test_softmax_shift_invariance_when_a_row_spans_several_wavefronts(path, Sk):
    """softmax(z + c) = softmax(z).  With scale 1 and no mask z = s exactly, so scores + 1000 is an input whose
    result must meet the ordinary bar.  When a row spans several wavefronts (or, in the two-sweep family, several
    running maxima per lane) each part subtracts its own reference: the rescaling between parts has to use the very
    numbers that were subtracted, or the rounding of reference * log2(e) -- about 1000 * 2^-24 in the exponent here,
    6e-5 relative on the result -- stays in the output."""
    case = wl.random_softmax_case(8400 + Sk, 1, 2, 5, Sk, score_std=3.0, scale=1.0)
    case.scores[:] = (case.scores + np.float32(1000.0)).astype(F32)
    with gu.overrides(path=path):
        got = _np(gu.run_softmax(case))
    err = assert_parity(got, gu.oracle_softmax(case), F32, f"softmax of scores + 1000, Sk={Sk}, path={path}")
    centred = wl.SoftmaxCase((case.scores - np.float32(1000.0)).astype(F32), None, 0, 0, 1.0, "none")
    with gu.overrides(path=path):
        got0 = _np(gu.run_softmax(centred))
    assert_parity(got0, gu.oracle_softmax(centred), F32, f"softmax of the centred scores, Sk={Sk}, path={path}")
    print(f"error report: softmax scores+1000 Sk={Sk} path={path}: max abs {err[0]:.3e}, max rel {err[1]:.3e}", flush=True)


def test_softmax_all_keys_masked_row():
    """Additive semantics: a fully masked row is the softmax of its scores.  binary32 rounds
    scale*s - 10000 to multiples of 2^-10, so the bar here is the one that rounding allows:
    |dz| <= 2^-11 per element, i.e. a relative error of about 2*2^-11 on each weight."""
    case = wl.random_softmax_case(83, 1, 1, 4, 64, mask_kind="key")
    case.mask[:] = wl.MASK_VALUE
    got = _np(gu.run_softmax(case))
    want = gu.oracle_softmax(case)
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got.sum(-1), 1.0, atol=1e-5)
    np.testing.assert_allclose(got, want, rtol=2.5 * 2.0 ** -10, atol=1e-6)


def test_non_default_stream_and_repeat_calls():
    st = torch.cuda.Stream()
    case = wl.softmax_case(wl.config_spec(1))
    lc = wl.layernorm_case(wl.config_spec(1))
    with torch.cuda.stream(st):
        got_s = gu.run_softmax(case, stream=st)
        got_l = gu.run_layernorm(lc, stream=st)
    st.synchronize()
    assert_parity(_np(got_s), gu.oracle_softmax(case), F32, "softmax on a side stream")
    assert_parity(_np(got_l), gu.oracle_layernorm(lc), F32, "layernorm on a side stream")
    # softmax of a softmax output is a valid input too: the call is repeatable on its own output
    again = wl.SoftmaxCase(_np(got_s), None, 0, 0, 1.0, "none")
    assert_parity(_np(gu.run_softmax(again)), gu.oracle_softmax(again), F32, "softmax applied twice")


def test_hip_graph_capture_and_replay():
    """The library allocates nothing and never synchronises, so its launches can be captured into a HIP graph.
    Every replay is checked against the eager result, with eager work and synchronisations in between."""
    spec = wl.config_spec(1)
    sc, lc = wl.softmax_case(spec), wl.layernorm_case(spec)
    st = torch.cuda.Stream()
    src = gu.dev(sc.scores)
    work = torch.empty_like(src)
    x, r = gu.dev(lc.x), gu.dev(lc.residual)
    b, g, be = gu.dev(lc.bias), gu.dev(lc.gamma), gu.dev(lc.beta)
    out = torch.empty_like(x)
    want_s, want_l = gu.oracle_softmax(sc), gu.oracle_layernorm(lc)
    with torch.cuda.stream(st):
        work.copy_(src)
        tb.turbo_masked_softmax(work, None, sc.scale, stream=st)       # eager reference run (also warms up)
        tb.turbo_add_bias_layernorm(x, r, b, g, be, lc.eps, out, stream=st)
        st.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st):
            work.copy_(src)
            tb.turbo_masked_softmax(work, None, sc.scale, stream=st)
            tb.turbo_add_bias_layernorm(x, r, b, g, be, lc.eps, out, stream=st)
        for replay in range(4):
            work.fill_(float("nan"))
            out.fill_(float("nan"))
            st.synchronize()
            graph.replay()
            st.synchronize()
            assert_parity(_np(work), want_s, F32, f"softmax, graph replay {replay}")
            assert_parity(_np(out), want_l, F32, f"layernorm, graph replay {replay}")
            tb.turbo_add_bias_layernorm(x, r, b, g, be, lc.eps, out, stream=st)  # eager work between replays
            st.synchronize()


_FIRST_USE_UNDER_CAPTURE = r"""
import sys
import numpy as np, torch
sys.path.insert(0, sys.argv[1]); sys.path.insert(0, sys.argv[1] + "/tests")
from paper_2010_05680_amd import binding as tb, workloads as wl
import gpu_util as gu
case = wl.random_layernorm_case(77, 300, 5120, dtype=np.float16, eps=1e-5)
x, r, b, g, be = (gu.dev(v) for v in (case.x, case.residual, case.bias, case.gamma, case.beta))
out = torch.full(case.x.shape, float("nan"), dtype=torch.float16, device="cuda")
st = torch.cuda.Stream()
with torch.cuda.stream(st):
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=st):   # the very first call of this kernel in the process is the captured one
        tb.turbo_add_bias_layernorm_dt(x, r, b, g, be, case.eps, out, stream=st)
    for _ in range(2):
        out.fill_(float("nan")); st.synchronize(); graph.replay(); st.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        want = gu.oracle_layernorm(case)
        assert np.all(np.abs(got - want) <= np.maximum(1e-6, 3e-3 * np.abs(want))), float(np.abs(got - want).max())
print("captured first use ok", tb.turbo_describe_plan(1, 300, 5120, tb.TURBO_F16))
"""


def test_first_use_of_a_looping_kernel_inside_graph_capture():
    """The looping LayerNorm kernel asks the runtime once per kernel for its resident workgroups per compute unit.
    In a fresh process that first call may come during stream capture: the capture must survive it."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, "-c", _FIRST_USE_UNDER_CAPTURE, root], capture_output=True, text=True, timeout=240)
    assert res.returncode == 0 and "captured first use ok" in res.stdout, res.stdout + res.stderr


@pytest.mark.parametrize("chunk", range(int(os.environ.get("TURBO_TEST_SWEEP_CHUNKS", "8"))))  # more chunks: a longer hunt
def test_randomized_shapes_alignments_and_variants(chunk):
    """Seeded sweep over shapes, element types, mask layouts, pointer offsets and forced kernel variants."""
    rng = np.random.default_rng(9000 + chunk)
    rng_w = np.random.default_rng(9500 + chunk)  # its own stream: the forced workgroup size of the block family
    special = [1, 2, 3, 4, 7, 8, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513, 768, 1000,
               1023, 1024, 1025, 1536, 2047, 2048, 2049, 3000, 4095, 4096, 4097, 5000, 8191, 8192]
    for case_no in range(60):
        block_waves = int(rng_w.choice([-1, -1, -1] + list(range(2, 17))))
        dtype = F32 if rng.random() < 0.5 else F16
        tdt = torch.float32 if dtype == F32 else torch.float16
        L = int(rng.choice(special)) if rng.random() < 0.7 else int(rng.integers(1, 6000))
        path = int(rng.choice([-1, -1, tb.PATH_WAVE, tb.PATH_BLOCK, tb.PATH_STREAM]))
        vec_bytes = int(rng.choice([-1, -1, -1, 2, 4, 8, 16]))
        if vec_bytes != -1 and vec_bytes < np.dtype(dtype).itemsize:
            vec_bytes = -1
        grid = int(rng.choice([-1, -1, 1, 3]))
        offset = int(rng.integers(0, 8))
        seed = int(rng.integers(1 << 30))
        what = (f"chunk {chunk} case {case_no}: L={L} dtype={np.dtype(dtype).name} path={path} vec={vec_bytes} grid={grid} "
                f"off={offset} block_waves={block_waves}")
        if rng.random() < 0.5:
            B, H = int(rng.integers(1, 4)), int(rng.integers(1, 4))
            Sq = int(rng.integers(1, max(2, min(40, 60000 // (L * B * H) + 1))))
            kind = str(rng.choice(["none", "key", "dense"] + (["causal"] if L <= 300 else [])))
            if kind == "causal":
                Sq = L
            case = wl.random_softmax_case(seed, B, H, Sq, L, dtype=dtype, mask_kind=kind)
            n = case.scores.size
            buf = torch.full((n + 16,), float("nan"), dtype=tdt, device="cuda")
            view = buf[offset:offset + n].view(case.scores.shape)
            view.copy_(torch.from_numpy(case.scores))
            mask = None if case.mask is None else gu.dev(case.mask)
            with gu.overrides(path=path, max_vec_bytes=vec_bytes, grid_waves=grid, block_waves=block_waves):
                tb.turbo_masked_softmax_ex(view, mask, case.mask_stride_b, case.mask_stride_q, case.scale)
                torch.cuda.synchronize()
            assert_parity(_np(view), gu.oracle_softmax(case), dtype, "softmax " + what)
            assert torch.isnan(buf[:offset]).all() and torch.isnan(buf[offset + n:]).all(), "softmax guard band " + what
        else:
            if L == 1:
                continue
            rows = int(rng.integers(1, max(2, min(60, 120000 // L + 1))))
            case = wl.random_layernorm_case(seed, rows, L, dtype=dtype, eps=1e-5)
            n = case.x.size
            obuf = torch.full((n + 16,), float("nan"), dtype=tdt, device="cuda")
            out = obuf[offset:offset + n].view(rows, L)
            use_res, use_bias = bool(rng.random() < 0.8), bool(rng.random() < 0.8)
            with gu.overrides(path=path, max_vec_bytes=vec_bytes, grid_waves=grid, block_waves=block_waves):
                tb.turbo_add_bias_layernorm_dt(gu.dev(case.x), gu.dev(case.residual) if use_res else None,
                                               gu.dev(case.bias) if use_bias else None, gu.dev(case.gamma),
                                               gu.dev(case.beta), case.eps, out)
                torch.cuda.synchronize()
            # raw inputs, tiny rows included: two or three values that nearly coincide make the result hinge on the
            # rounding of x + bias + residual, so the bar follows the row's condition number (1 for well-spread rows)
            scale = layernorm_bound_scale(case.x, case.residual if use_res else None, case.bias if use_bias else None, case.eps)
            assert_parity(_np(out), gu.oracle_layernorm(case, residual=use_res, bias=use_bias), dtype, "layernorm " + what,
                          bound_scale=scale)
            assert torch.isnan(obuf[:offset]).all() and torch.isnan(obuf[offset + n:]).all(), "layernorm guard band " + what
