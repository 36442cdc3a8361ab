"""Parity of the element-wise fused kernels (bias+GELU, bias+head split, head merge) against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import turbo_oracle as orc
from paper_2010_05680_amd import binding as tb

from conftest import assert_parity
import gpu_util as gu

pytestmark = pytest.mark.gpu
F32, F16 = np.float32, np.float16


def _np(t):
    return t.detach().cpu().numpy()


def _rand(rng, shape, dtype, std=1.0):
    return (rng.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(dtype)


def _gelu(x, bias, approximate, out=None):
    xd = gu.dev(x)
    bd = None if bias is None else gu.dev(bias)
    od = torch.full_like(xd, float("nan")) if out is None else out
    tb.turbo_add_bias_gelu(xd, bd, approximate, od)
    torch.cuda.synchronize()
    return od


@pytest.mark.parametrize("approximate", [False, True], ids=["erf", "tanh"])
@pytest.mark.parametrize("dtype", [F32, F16])
def test_gelu_shapes(dtype, approximate):
    rng = np.random.Generator(np.random.Philox(11))
    shapes = [(1, 1), (3, 5), (7, 64), (16, 768), (33, 3072), (5, 1001), (2, 4099), (257, 130), (1, 100003), (640, 3072)]
    for rows, hidden in shapes:
        x = _rand(rng, (rows, hidden), dtype, 1.5)
        b = _rand(rng, (hidden,), dtype, 0.5)
        got = _np(_gelu(x, b, approximate))
        assert_parity(got, orc.add_bias_gelu(x, b, approximate), dtype, f"gelu {rows}x{hidden} approximate={approximate}")


def test_gelu_wide_range_no_bias_in_place_and_narrow_kernel():
    rng = np.random.Generator(np.random.Philox(12))
    x = np.concatenate([np.linspace(-12, 12, 4096, dtype=F32), _rand(rng, (4096,), F32, 4.0)]).reshape(8, 1024)
    for approximate in (False, True):
        got = _np(_gelu(x, None, approximate))
        assert_parity(got, orc.add_bias_gelu(x, None, approximate), F32, f"gelu wide range approximate={approximate}")
    xd = gu.dev(x)
    tb.turbo_add_bias_gelu(xd, None, False, xd)  # out aliases x
    torch.cuda.synchronize()
    assert_parity(_np(xd), orc.add_bias_gelu(x, None), F32, "gelu in place")
    b = _rand(rng, (1024,), F32, 0.3)
    with gu.overrides(max_vec_bytes=4):
        assert_parity(_np(_gelu(x, b, False)), orc.add_bias_gelu(x, b), F32, "gelu 4-byte kernel")


def test_gelu_every_binary16_input_and_a_dense_binary32_grid():
    """The erf form's tail approximation is a fit: check it over its whole domain, not on random draws.

    binary16: all 63488 finite inputs (outputs that overflow binary16 are excluded: the oracle has no infinity there);
    binary32: two million points over [-12, 12], where every regime of the bound max(atol, rtol |gelu|) occurs.
    The margin that comes out (worst error / bound) is asserted to stay below 1/2, so a drift in the constants
    shows before it reaches the parity bound itself.
    """
    half = np.arange(65536, dtype=np.uint16).view(F16)
    half = half[np.isfinite(half)]
    half = half[np.abs(half.astype(np.float64)) < 65000]
    n16 = half.size - half.size % 8
    cases = [(half[:n16].reshape(-1, 8), F16, 3e-3), (np.linspace(-12, 12, 1 << 21, dtype=F32).reshape(-1, 4096), F32, 1e-5)]
    for x, dtype, rtol in cases:
        for approximate in (False, True):
            got = _np(_gelu(x, None, approximate)).astype(np.float64)
            want = orc.add_bias_gelu(x, None, approximate)
            assert_parity(got, want, dtype, f"gelu whole domain {np.dtype(dtype).name} approximate={approximate}")
            if not approximate and dtype == F32:
                margin = (np.abs(got - want) / np.maximum(1e-6, rtol * np.abs(want))).max()
                assert margin < 0.5, f"binary32 erf gelu uses {margin:.2f} of the parity bound"


@pytest.mark.parametrize("dtype", [F32, F16])
def test_gelu_unaligned_pointers_and_guard_bands(dtype):
    rng = np.random.Generator(np.random.Philox(13))
    tdt = torch.float32 if dtype == F32 else torch.float16
    for rows, hidden in [(9, 768), (5, 1003), (1, 7)]:
        x = _rand(rng, (rows, hidden), dtype)
        b = _rand(rng, (hidden,), dtype, 0.2)
        n = x.size
        xbuf = torch.zeros(n + 16, dtype=tdt, device="cuda")
        xv = xbuf[3:3 + n].view(rows, hidden)
        xv.copy_(torch.from_numpy(x))
        obuf = torch.full((n + 64,), float("nan"), dtype=tdt, device="cuda")
        ov = obuf[29:29 + n].view(rows, hidden)
        bbuf = torch.zeros(hidden + 8, dtype=tdt, device="cuda")
        bv = bbuf[1:1 + hidden]
        bv.copy_(torch.from_numpy(b))
        tb.turbo_add_bias_gelu(xv, bv, False, ov)
        torch.cuda.synchronize()
        assert_parity(_np(ov), orc.add_bias_gelu(x, b), dtype, f"gelu offset views {rows}x{hidden}")
        assert torch.isnan(obuf[:29]).all() and torch.isnan(obuf[29 + n:]).all(), "gelu wrote outside its tensor"


@pytest.mark.parametrize("dtype", [F32, F16])
@pytest.mark.parametrize("path", [-1, 0, 2], ids=["planned", "no-lds", "flat"])
def test_split_and_merge_heads(dtype, path):
    """planned: small heads go through the LDS-tiled kernel (whole and partial tiles, one dimension shorter than a tile,
    with and without bias); no-lds / flat: the two kernels without LDS on the same shapes."""
    rng = np.random.Generator(np.random.Philox(14))
    tdt = torch.float32 if dtype == F32 else torch.float16
    for B, S, K, H, D in [(1, 1, 1, 1, 1), (2, 5, 3, 4, 64), (20, 128, 3, 12, 64), (3, 17, 1, 5, 20), (2, 9, 2, 3, 6),
                          (2, 7, 3, 2, 5), (1, 300, 3, 16, 64), (2, 37, 3, 5, 32), (1, 70, 2, 33, 16), (3, 33, 1, 7, 8),
                          (2, 19, 3, 3, 128), (1, 5, 1, 70, 8), (2, 64, 3, 16, 32), (1, 129, 1, 2, 4), (1, 2, 2, 130, 16)]:
        x = _rand(rng, (B, S, K, H, D), dtype)
        bias = _rand(rng, (K, H, D), dtype, 0.3)
        for use_bias in (True, False):
            out = torch.full((K, B, H, S, D), float("nan"), dtype=tdt, device="cuda")
            with gu.overrides(path=path):
                tb.turbo_add_bias_split_heads(gu.dev(x), gu.dev(bias) if use_bias else None, out)
            torch.cuda.synchronize()
            want = orc.add_bias_split_heads(x, bias if use_bias else None)
            if use_bias:
                assert_parity(_np(out), want, dtype, f"split heads {B,S,K,H,D}")
            else:
                np.testing.assert_array_equal(_np(out).astype(np.float64), want)  # a pure permutation is bit-exact
        y = _rand(rng, (B, H, S, D), dtype)
        out = torch.full((B, S, H, D), float("nan"), dtype=tdt, device="cuda")
        with gu.overrides(path=path):
            tb.turbo_merge_heads(gu.dev(y), out)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(_np(out).astype(np.float64), orc.merge_heads(y))


def test_elementwise_full_size_sampled():
    """GPT-2-medium feed-forward activation [32768, 4096] fp16 and QKV split [64,512,3,16,64] fp16, sampled rows."""
    rng = np.random.Generator(np.random.Philox(15))
    rows, hidden = 32768, 4096
    x = _rand(rng, (rows, hidden), F16, 1.5)
    b = _rand(rng, (hidden,), F16, 0.5)
    out = _gelu(x, b, False)
    pick = gu.sample_rows(rows, 300, seed=5)
    assert_parity(_np(out[torch.from_numpy(pick).cuda()]), orc.add_bias_gelu(x[pick], b), F16, "gelu full size, sampled rows")
    assert torch.isfinite(out).all()
    B, S, K, H, D = 64, 512, 3, 16, 64
    x5 = _rand(rng, (B, S, K, H, D), F16)
    bias = _rand(rng, (K, H, D), F16, 0.3)
    o5 = torch.full((K, B, H, S, D), float("nan"), dtype=torch.float16, device="cuda")
    tb.turbo_add_bias_split_heads(gu.dev(x5), gu.dev(bias), o5)
    torch.cuda.synchronize()
    for bsel in (0, 31, 63):
        want = orc.add_bias_split_heads(x5[bsel:bsel + 1], bias)
        assert_parity(_np(o5[:, bsel:bsel + 1]), want, F16, f"split heads full size, batch {bsel}")
    assert torch.isfinite(o5).all()


def test_elementwise_error_paths_need_no_gpu_work():
    L = tb.lib()
    fake = 0x10000
    assert L.turbo_add_bias_gelu(None, None, 4, 4, 0, fake, tb.TURBO_F32, None) == tb.TURBO_ERR_NULL
    assert L.turbo_add_bias_gelu(fake, None, 0, 4, 0, fake, tb.TURBO_F32, None) == tb.TURBO_ERR_SHAPE
    assert L.turbo_add_bias_gelu(fake, None, 4, 4, 0, fake, 9, None) == tb.TURBO_ERR_DTYPE
    assert L.turbo_add_bias_gelu(fake + 2, None, 4, 4, 0, fake, tb.TURBO_F32, None) == tb.TURBO_ERR_ALIGN
    assert L.turbo_add_bias_split_heads(fake, None, 1, 1, 0, 1, 1, fake, tb.TURBO_F32, None) == tb.TURBO_ERR_SHAPE
    assert L.turbo_merge_heads(fake, 1, 1, 1, 1, None, tb.TURBO_F32, None) == tb.TURBO_ERR_NULL
    big = 2 ** 31 - 1  # the element count is checked factor by factor: no overflow on the way to the verdict
    assert L.turbo_add_bias_split_heads(fake, None, big, big, big, big, big, fake, tb.TURBO_F32, None) == tb.TURBO_ERR_SHAPE
    assert L.turbo_merge_heads(fake, big, big, big, 4, fake, tb.TURBO_F16, None) == tb.TURBO_ERR_SHAPE


def test_stream_probe_copies_and_adds():
    """The measurement aid behind the bench's stream ceilings: out = in0 (+ in1), exact in binary32."""
    rng = np.random.Generator(np.random.Philox(16))
    for n in (4, 1024 * 4, 1024 * 4 + 4, 3 * 4096 * 4 + 8, 1 << 20):
        a, b = _rand(rng, (n,), F32), _rand(rng, (n,), F32)
        out = torch.full((n + 8,), float("nan"), device="cuda")
        tb.turbo_stream_probe(gu.dev(a), gu.dev(b), out[4:4 + n])
        torch.cuda.synchronize()
        np.testing.assert_array_equal(_np(out[4:4 + n]), a + b)
        assert torch.isnan(out[:4]).all() and torch.isnan(out[4 + n:]).all()
        ad = gu.dev(a)
        tb.turbo_stream_probe(ad, None, ad)  # in place: the softmax mix
        torch.cuda.synchronize()
        np.testing.assert_array_equal(_np(ad), a)
    h = _rand(rng, (4096,), F16)  # any dtype: the bytes are what is moved
    od = torch.zeros(4096, dtype=torch.float16, device="cuda")
    tb.turbo_stream_probe(gu.dev(h), None, od)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(_np(od), h)


import os


@pytest.mark.parametrize("chunk", range(int(os.environ.get("TURBO_TEST_SWEEP_CHUNKS", "4"))))
def test_randomized_elementwise_cases(chunk):
    rng = np.random.default_rng(8000 + chunk)
    for case_no in range(40):
        dtype = F32 if rng.random() < 0.5 else F16
        tdt = torch.float32 if dtype == F32 else torch.float16
        es = np.dtype(dtype).itemsize
        cap = int(rng.choice([-1, -1, es, 4, 8]))
        if cap != -1 and cap < es:
            cap = -1
        off = int(rng.integers(0, 4))
        kind = str(rng.choice(["gelu", "split", "merge"]))
        what = f"chunk {chunk} case {case_no}: {kind} {np.dtype(dtype).name} cap={cap} off={off}"

        def place(host):  # the array in device memory, `off` elements past an aligned address
            buf = torch.zeros(host.size + off, dtype=tdt, device="cuda")
            view = buf[off:].view(host.shape)
            view.copy_(torch.from_numpy(host))
            return view

        if kind == "gelu":
            rows, hidden = int(rng.integers(1, 40)), int(rng.choice([1, 2, 3, 5, 7, 8, 9, 64, 100, 768, 1001, 3072]))
            x, b = _rand(rng, (rows, hidden), dtype, 1.5), _rand(rng, (hidden,), dtype, 0.5)
            approximate, use_bias = bool(rng.random() < 0.5), bool(rng.random() < 0.8)
            obuf = torch.full((x.size + off + 8,), float("nan"), dtype=tdt, device="cuda")
            ov = obuf[off:off + x.size].view(rows, hidden)
            with gu.overrides(max_vec_bytes=cap, path=2 if rng.random() < 0.3 else -1):
                tb.turbo_add_bias_gelu(place(x), place(b) if use_bias else None, approximate, ov)
            torch.cuda.synchronize()
            assert_parity(_np(ov), orc.add_bias_gelu(x, b if use_bias else None, approximate), dtype,
                          what + f" rows={rows} hidden={hidden} approximate={approximate} bias={use_bias}")
            assert torch.isnan(obuf[:off]).all() and torch.isnan(obuf[off + x.size:]).all(), what
        else:
            B, S, H = int(rng.integers(1, 4)), int(rng.integers(1, 20)), int(rng.integers(1, 9))
            D = int(rng.choice([1, 2, 3, 4, 5, 6, 8, 12, 16, 20, 32, 64, 80]))
            flat = int(rng.choice([-1, -1, 0, 2]))  # planned (LDS-tiled where the shape allows), no LDS, flat
            with gu.overrides(max_vec_bytes=cap, path=flat):
                if kind == "split":
                    K = int(rng.choice([1, 2, 3]))
                    x5, bias = _rand(rng, (B, S, K, H, D), dtype), _rand(rng, (K, H, D), dtype, 0.3)
                    use_bias = bool(rng.random() < 0.7)
                    out = torch.full((K, B, H, S, D), float("nan"), dtype=tdt, device="cuda")
                    tb.turbo_add_bias_split_heads(place(x5), place(bias) if use_bias else None, out)
                    torch.cuda.synchronize()
                    assert_parity(_np(out), orc.add_bias_split_heads(x5, bias if use_bias else None), dtype,
                                  what + f" {B,S,K,H,D} bias={use_bias} flat={flat}")
                else:
                    y = _rand(rng, (B, H, S, D), dtype)
                    out = torch.full((B, S, H, D), float("nan"), dtype=tdt, device="cuda")
                    tb.turbo_merge_heads(place(y), out)
                    torch.cuda.synchronize()
                    np.testing.assert_array_equal(_np(out).astype(np.float64), orc.merge_heads(y), err_msg=what + f" {B,H,S,D} flat={flat}")
