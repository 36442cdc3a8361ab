"""Every kernel shape the dispatcher can choose runs at least once against the oracle.

The library compiles some two thousand instantiations of a handful of kernel templates (element type x vector
width x lanes per row x vectors per lane x mask kind or residual flag x row mode ...).  The other parity tests reach
them through shapes that matter in practice; this one walks the planner instead: it scans row lengths under every
vector-width cap, forced family and pointer alignment, keeps one row length per distinct plan, and runs each plan with
every mask kind (softmax) or residual / length-aware combination (LayerNorm) on a small batch.
"""
import numpy as np
import pytest
import torch

from oracle import turbo_oracle as orc
from paper_2010_05680_amd import binding as tb

from conftest import assert_parity
import gpu_util as gu

pytestmark = pytest.mark.gpu
F32, F16 = np.float32, np.float16

B, H, SQ = 4, 1, 10           # 40 rows: a ragged tile for the lane-group kernels, several rows for the others
ROWS = B * H * SQ
_NV = (1, 2, 3, 4, 5, 6, 8, 12, 16)
# every row length below 2200, a coarse scan above, and the lengths that lane groups or workgroups tile exactly
LENGTHS = sorted(set(list(range(1, 2200)) + list(range(2200, 70001, 37)) +
                     [lanes * nv * vec for lanes in (4, 8, 16, 32) + tuple(64 * w for w in range(1, 17)) for nv in _NV for vec in (1, 2, 4, 8)
                      if lanes * nv * vec <= 70000]))


def _distinct_plans(op, code, shortest=1):
    """{plan text: (row length, aligned, vector cap, forced family)} over the scan; the first length found is kept."""
    plans = {}
    try:
        for cap in (-1, 2, 4, 8, 16):
            tb.turbo_set_override(tb.TURBO_OVR_MAX_VEC_BYTES, cap)
            for path in (-1, tb.PATH_WAVE, tb.PATH_BLOCK, tb.PATH_STREAM):
                tb.turbo_set_override(tb.TURBO_OVR_PATH, path)
                for aligned in (True, False):
                    for L in LENGTHS:
                        if L < shortest:
                            continue
                        text = tb.turbo_describe_plan(op, ROWS, L, code, aligned)
                        plans.setdefault(text, (L, aligned, cap, path))
    finally:
        tb.turbo_set_override(tb.TURBO_OVR_MAX_VEC_BYTES, -1)
        tb.turbo_set_override(tb.TURBO_OVR_PATH, -1)
    return plans


def _device_view(host: np.ndarray, aligned: bool) -> torch.Tensor:
    """The array in device memory; when not `aligned`, one element past a 256-byte boundary."""
    if aligned:
        return gu.dev(host)
    tdt = torch.float32 if host.dtype == F32 else torch.float16
    buf = torch.zeros(host.size + 1, dtype=tdt, device="cuda")
    view = buf[1:].view(host.shape)
    view.copy_(torch.from_numpy(host))
    return view


@pytest.mark.parametrize("dtype", [F32, F16])
def test_every_softmax_plan(dtype):
    code = tb.TURBO_F32 if dtype == F32 else tb.TURBO_F16
    plans = _distinct_plans(0, code)
    rng = np.random.Generator(np.random.Philox(51))
    ran = 0
    for text, (L, aligned, cap, path) in plans.items():
        scores = (rng.standard_normal((B, H, SQ, L), dtype=np.float32) * 3).astype(dtype)
        k_len = rng.integers(0, L + 1, size=B).astype(np.int32)
        k_len[0] = L
        q_len = np.array([SQ, SQ - 3, 0, 1], dtype=np.int32)
        mask = np.where(rng.random((B, SQ, L)) < 0.3, -10000.0, 0.0).astype(dtype)
        mask[..., 0] = 0
        for kind in ("none", "additive", "lengths", "causal"):
            what = f"{text} | L={L} aligned={aligned} cap={cap} path={path} mask={kind}"
            s = _device_view(scores, aligned)
            print_on_failure = what  # shown by pytest with the traceback if a launch is refused
            with gu.overrides(path=path, max_vec_bytes=cap):
                if kind == "none":
                    tb.turbo_masked_softmax_ex(s, None, 0, 0, 0.125)
                    want = orc.masked_softmax(scores, None, 0, 0, 0.125)
                elif kind == "additive":
                    tb.turbo_masked_softmax_ex(s, _device_view(mask, aligned), SQ * L, L, 0.125)
                    want = orc.masked_softmax(scores, mask, SQ * L, L, 0.125)
                elif kind == "lengths":
                    tb.turbo_masked_softmax_varlen(s, gu.dev(q_len), gu.dev(k_len), 0.125)
                    want = orc.masked_softmax_varlen(scores, q_len, k_len, 0.125)
                else:
                    tb.turbo_masked_softmax_causal(s, None, gu.dev(k_len), 0.125)
                    want = orc.masked_softmax_causal(scores, None, k_len, 0.125)
            torch.cuda.synchronize()
            assert_parity(s.cpu().numpy(), want, dtype, what)
            ran += 1
            if ran % 200 == 0:
                print(f"softmax {np.dtype(dtype).name}: {ran} launches", flush=True)
    print(f"softmax {np.dtype(dtype).name}: {len(plans)} plans, {ran} launches")
    assert len(plans) > 150


@pytest.mark.parametrize("dtype", [F32, F16])
def test_every_layernorm_plan(dtype):
    code = tb.TURBO_F32 if dtype == F32 else tb.TURBO_F16
    plans = _distinct_plans(1, code, shortest=2)  # a single column has zero variance: eps-dominated, its own test
    rng = np.random.Generator(np.random.Philox(52))
    tdt = torch.float32 if dtype == F32 else torch.float16
    ran = 0
    for text, (L, aligned, cap, path) in plans.items():
        normal = lambda shape, std, mean=0.0: (rng.standard_normal(shape, dtype=np.float32) * np.float32(std) + np.float32(mean)).astype(dtype)
        x, res = normal((ROWS, L), 1.0), normal((ROWS, L), 1.0)
        # rows of two or three columns are ill-conditioned when their values nearly coincide (the result then depends on
        # the rounding of x + bias + residual); an alternating offset keeps every row's spread well above that
        x = (x + np.where(np.arange(L) % 2 == 0, -8.0, 8.0).astype(dtype)).astype(dtype)
        bias, gamma, beta = normal((L,), 0.1), normal((L,), 0.1, 1.0), normal((L,), 0.1)
        lens = np.array([SQ, 0, SQ - 4, 1], dtype=np.int32)
        for residual in (True, False):
            for varlen in (False, True):
                what = f"{text} | L={L} aligned={aligned} cap={cap} path={path} residual={residual} varlen={varlen}"
                xd = _device_view(x, aligned)
                rd = gu.dev(res) if residual else None
                out = torch.full((ROWS, L), -7.25, dtype=tdt, device="cuda")
                args = (gu.dev(bias), gu.dev(gamma), gu.dev(beta))
                with gu.overrides(path=path, max_vec_bytes=cap):
                    if varlen:
                        tb.turbo_add_bias_layernorm_varlen(xd.view(B, SQ, L), None if rd is None else rd.view(B, SQ, L), *args,
                                                           gu.dev(lens), 1e-5, out.view(B, SQ, L))
                        before = np.full((B, SQ, L), -7.25)
                        want = orc.add_bias_layernorm_varlen(x.reshape(B, SQ, L), res.reshape(B, SQ, L) if residual else None,
                                                             bias, gamma, beta, lens, 1e-5, before).reshape(ROWS, L)
                    else:
                        tb.turbo_add_bias_layernorm_dt(xd, rd, *args, 1e-5, out)
                        want = orc.add_bias_layernorm(x, res if residual else None, bias, gamma, beta, 1e-5)
                torch.cuda.synchronize()
                assert_parity(out.cpu().numpy(), want, dtype, what)
                ran += 1
                if ran % 200 == 0:
                    print(f"layernorm {np.dtype(dtype).name}: {ran} launches", flush=True)
    print(f"layernorm {np.dtype(dtype).name}: {len(plans)} plans, {ran} launches")
    assert len(plans) > 120


@pytest.mark.parametrize("dtype", [F32, F16])
def test_block_family_with_every_workgroup_size(dtype):
    """The workgroup-per-row kernels take their number of wavefronts from the launch, 2 to 16; the planner uses only
    some of them.  Force each one in turn on rows that it tiles exactly, rows with a ragged tail and rows of odd
    length, with and without per-request lengths."""
    code = tb.TURBO_F32 if dtype == F32 else tb.TURBO_F16
    vec = 16 // np.dtype(dtype).itemsize
    rng = np.random.Generator(np.random.Philox(53))
    tdt = torch.float32 if dtype == F32 else torch.float16
    ran = 0
    for w in range(2, 17):
        for L in (64 * w * vec, 64 * w * 2 * vec, 64 * w * 2 * vec - 3 * vec, 64 * w * vec + 5, 64 * w * 3 * vec - 1):
            with gu.overrides(path=tb.PATH_BLOCK, block_waves=w):
                plans = [tb.turbo_describe_plan(op, ROWS, L, code) for op in (0, 1)]
            scores = (rng.standard_normal((B, H, SQ, L), dtype=np.float32) * 3).astype(dtype)
            k_len = rng.integers(0, L + 1, size=B).astype(np.int32)
            q_len = np.array([SQ, SQ - 3, 0, 1], dtype=np.int32)
            for kind in ("none", "lengths"):
                what = f"softmax {plans[0]} | forced waves={w} L={L} mask={kind}"
                s = gu.dev(scores)
                with gu.overrides(path=tb.PATH_BLOCK, block_waves=w):
                    if kind == "none":
                        tb.turbo_masked_softmax_ex(s, None, 0, 0, 0.125)
                        want = orc.masked_softmax(scores, None, 0, 0, 0.125)
                    else:
                        tb.turbo_masked_softmax_varlen(s, gu.dev(q_len), gu.dev(k_len), 0.125)
                        want = orc.masked_softmax_varlen(scores, q_len, k_len, 0.125)
                torch.cuda.synchronize()
                assert_parity(s.cpu().numpy(), want, dtype, what)
                ran += 1
            normal = lambda shape, std, mean=0.0: (rng.standard_normal(shape, dtype=np.float32) * np.float32(std) + np.float32(mean)).astype(dtype)
            x, res = normal((ROWS, L), 1.0), normal((ROWS, L), 1.0)
            bias, gamma, beta = normal((L,), 0.1), normal((L,), 0.1, 1.0), normal((L,), 0.1)
            for residual in (True, False):
                what = f"layernorm {plans[1]} | forced waves={w} L={L} residual={residual}"
                out = torch.full((ROWS, L), -7.25, dtype=tdt, device="cuda")
                with gu.overrides(path=tb.PATH_BLOCK, block_waves=w):
                    tb.turbo_add_bias_layernorm_dt(gu.dev(x), gu.dev(res) if residual else None, gu.dev(bias), gu.dev(gamma),
                                                   gu.dev(beta), 1e-5, out)
                torch.cuda.synchronize()
                assert_parity(out.cpu().numpy(), orc.add_bias_layernorm(x, res if residual else None, bias, gamma, beta, 1e-5),
                              dtype, what)
                ran += 1
        print(f"workgroup sizes {np.dtype(dtype).name}: waves={w} done, {ran} launches", flush=True)


@pytest.mark.parametrize("dtype", [F32, F16])
def test_every_elementwise_kernel_variant(dtype):
    """bias+GELU: both forms x (hidden a multiple of the vector or not) x (16-byte aligned or not) x (wide or
    one-element accesses); head permutations: split / merge x bias x vector widths 16..2 bytes x the grouped and
    the flat kernel."""
    rng = np.random.Generator(np.random.Philox(53))
    tdt = torch.float32 if dtype == F32 else torch.float16
    es = np.dtype(dtype).itemsize
    rand = lambda shape, std=1.0: (rng.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(dtype)
    ran = 0
    for hidden, flat in ((64, False), (37, False), (1, False), (130, False), (768, False), (768, True), (1000, False), (3072, False)):
        for aligned in (True, False):
            for cap in (-1, es):
                for approximate in (False, True):
                    for use_bias in (True, False):
                        x, b = rand((23, hidden), 1.5), rand((hidden,), 0.5)
                        out = torch.full((23 * hidden + 1,), float("nan"), dtype=tdt, device="cuda")
                        ov = out[(0 if aligned else 1):][:23 * hidden].view(23, hidden)
                        with gu.overrides(max_vec_bytes=cap, path=2 if flat else -1):
                            tb.turbo_add_bias_gelu(_device_view(x, aligned), _device_view(b, aligned) if use_bias else None,
                                                   approximate, ov)
                        torch.cuda.synchronize()
                        assert_parity(ov.cpu().numpy(), orc.add_bias_gelu(x, b if use_bias else None, approximate), dtype,
                                      f"gelu hidden={hidden} flat={flat} aligned={aligned} cap={cap} approximate={approximate} bias={use_bias}")
                        ran += 1
    for D in (64, 36, 6, 5):            # 16-, 8-, 4- and 2-byte vectors for binary16; 16, 16, 8, 4 for binary32
        for S, Hh in ((8, 4), (7, 3)):  # multiples of four take the grouped kernel, others the flat one
            for aligned in (True, False):
                for flat in (False, True):
                    x5, bias = rand((2, S, 3, Hh, D)), rand((3, Hh, D), 0.3)
                    y4 = rand((2, Hh, S, D))
                    with gu.overrides(path=2 if flat else -1):
                        for use_bias in (True, False):
                            o5 = torch.full((3, 2, Hh, S, D), float("nan"), dtype=tdt, device="cuda")
                            tb.turbo_add_bias_split_heads(_device_view(x5, aligned), gu.dev(bias) if use_bias else None, o5)
                            torch.cuda.synchronize()
                            assert_parity(o5.cpu().numpy(), orc.add_bias_split_heads(x5, bias if use_bias else None), dtype,
                                          f"split heads D={D} S={S} H={Hh} aligned={aligned} flat={flat} bias={use_bias}")
                            ran += 1
                        o4 = torch.full((2, S, Hh, D), float("nan"), dtype=tdt, device="cuda")
                        tb.turbo_merge_heads(_device_view(y4, aligned), o4)
                        torch.cuda.synchronize()
                        np.testing.assert_array_equal(o4.cpu().numpy().astype(np.float64), orc.merge_heads(y4))
                        ran += 1
    print(f"element-wise {np.dtype(dtype).name}: {ran} launches")
