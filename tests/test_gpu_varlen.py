"""Parity of the length-aware variants (zero-padded variable-length batches) against the CPU oracle, and proof that
padding is neither read into the result nor written."""
import numpy as np
import pytest
import torch

from oracle import turbo_oracle as orc
from paper_2010_05680_amd import binding as tb
from paper_2010_05680_amd import workloads as wl

from conftest import assert_parity
import gpu_util as gu

pytestmark = pytest.mark.gpu
F32, F16 = np.float32, np.float16


def _np(t):
    return t.detach().cpu().numpy()


def _run_softmax(scores, q_len, k_len, scale):
    s = gu.dev(scores)
    ql = None if q_len is None else torch.from_numpy(np.asarray(q_len, dtype=np.int32)).cuda()
    kl = torch.from_numpy(np.asarray(k_len, dtype=np.int32)).cuda()
    tb.turbo_masked_softmax_varlen(s, ql, kl, scale)
    torch.cuda.synchronize()
    return s


@pytest.mark.parametrize("dtype", [F32, F16])
@pytest.mark.parametrize("path", [-1, tb.PATH_WAVE, tb.PATH_BLOCK, tb.PATH_STREAM])
def test_varlen_softmax_shapes(dtype, path):
    rng = np.random.Generator(np.random.Philox(21))
    for B, H, S in [(1, 1, 1), (3, 2, 7), (4, 3, 16), (5, 2, 33), (6, 2, 64), (4, 2, 100), (3, 2, 128), (4, 1, 257), (2, 1, 493),
                    (2, 1, 1000), (1, 1, 2048), (2, 1, 4100),
                    # row lengths whose vectors tile 32 or 16 lanes exactly (96, 160, 48 vectors): without per-row key
                    # counts they get a kernel shape that exists only without bounds checks
                    (2, 1, 384), (1, 1, 640), (2, 1, 192), (1, 1, 768), (1, 1, 1280)]:
        scores = (rng.standard_normal((B, H, S, S), dtype=np.float32) * 3).astype(dtype)
        lens = rng.integers(0, S + 1, size=B)
        lens[0] = S                       # one request fills the batch, as the padded layout implies
        if B > 1:
            lens[1] = min(S, 1)
        for q_len in (lens, None):
            with gu.overrides(path=path):
                got = _np(_run_softmax(scores, q_len, lens, 0.125))
            want = orc.masked_softmax_varlen(scores, q_len, lens, 0.125)
            assert_parity(got, want, dtype, f"varlen softmax B={B} H={H} S={S} path={path} q_len={'yes' if q_len is not None else 'no'}")
            # padding rows must be bit-identical to the input (never written)
            if q_len is not None:
                for b in range(B):
                    np.testing.assert_array_equal(got[b, :, lens[b]:, :], scores[b, :, lens[b]:, :])


@pytest.mark.parametrize("dtype", [F32, F16])
def test_varlen_softmax_live_tile_loop_and_large_batches(dtype):
    """With query lengths and up to 63 requests the lane-group kernels loop over the tiles that hold live rows only
    (found from the length table inside every wavefront); 64 requests or more keep one tile of consecutive rows per
    workgroup.  Both sides of that limit, requests without rows or without keys anywhere in the batch, different
    query and key lengths, a grid so small that every workgroup loops, and padding poisoned with NaN."""
    rng = np.random.Generator(np.random.Philox(27))
    for B, H, Sq, Sk in [(63, 1, 9, 40), (64, 1, 9, 40), (70, 2, 5, 24), (7, 3, 50, 50), (5, 2, 33, 128), (9, 1, 20, 300),
                         (3, 2, 100, 493), (2, 1, 37, 1000)]:
        scores = (rng.standard_normal((B, H, Sq, Sk), dtype=np.float32) * 3).astype(dtype)
        q_len = rng.integers(0, Sq + 1, size=B)
        k_len = rng.integers(0, Sk + 1, size=B)
        q_len[0], k_len[0] = Sq, Sk
        q_len[B // 2] = 0                 # a request without rows in the middle of the batch
        k_len[B - 1] = 0                  # and one without keys at its end
        if B > 3:
            q_len[1], k_len[1] = Sq, 1
        poisoned = scores.copy()
        for b in range(B):
            poisoned[b, :, :, k_len[b]:] = np.nan
            poisoned[b, :, q_len[b]:, :] = np.nan
        want = orc.masked_softmax_varlen(scores, q_len, k_len, 0.125)
        for mode in ({}, {"grid_waves": 1}, {"path": tb.PATH_WAVE, "grid_waves": 3}):
            with gu.overrides(**mode):
                got = _np(_run_softmax(poisoned, q_len, k_len, 0.125))
            for b in range(B):
                what = f"varlen softmax B={B} H={H} Sq={Sq} Sk={Sk} {mode} request {b} (q {q_len[b]}, k {k_len[b]})"
                if k_len[b] > 0 and q_len[b] > 0:
                    assert_parity(got[b, :, :q_len[b], :], want[b, :, :q_len[b], :], dtype, what)
                    assert (got[b, :, :q_len[b], k_len[b]:] == 0).all(), what
                    assert np.isnan(got[b, :, q_len[b]:, :]).all(), what + ": a padding row was written"
                else:  # nothing to do for this request: every element keeps its bits
                    np.testing.assert_array_equal(got[b].view(np.uint16 if dtype == F16 else np.uint32),
                                                  poisoned[b].view(np.uint16 if dtype == F16 else np.uint32), what)


def test_varlen_softmax_rows_too_long_for_registers():
    """Rows beyond 32768 keys go through the two-sweep kernels; padding is poisoned with NaN."""
    rng = np.random.Generator(np.random.Philox(24))
    for dtype, S_k in ((F32, 40000), (F16, 70008), (F32, 33001)):
        B, H, S_q = 3, 2, 3
        scores = (rng.standard_normal((B, H, S_q, S_k), dtype=np.float32) * 3).astype(dtype)
        k_len = np.array([S_k, 1, S_k // 2 + 3])
        q_len = np.array([3, 2, 0])
        poisoned = scores.copy()
        for b in range(B):
            poisoned[b, :, :, k_len[b]:] = np.nan
            poisoned[b, :, q_len[b]:, :] = np.nan
        got = _np(_run_softmax(poisoned, q_len, k_len, 0.125))
        want = orc.masked_softmax_varlen(scores, q_len, k_len, 0.125)
        for b in range(B):
            live = got[b, :, :q_len[b], :]
            if q_len[b] > 0:
                assert_parity(live, want[b, :, :q_len[b], :], dtype, f"varlen two-sweep softmax Sk={S_k} request {b}")
                assert (live[..., k_len[b]:] == 0).all()
            assert np.isnan(got[b, :, q_len[b]:, :]).all(), "a padding row was written"


def test_varlen_softmax_ignores_what_lies_beyond_the_lengths():
    """NaNs planted in every padded key and padded query row must not reach any real output."""
    rng = np.random.Generator(np.random.Philox(22))
    B, H, S = 6, 3, 200
    lens = np.array([200, 5, 77, 128, 1, 199])
    scores = (rng.standard_normal((B, H, S, S), dtype=np.float32) * 3)
    poisoned = scores.copy()
    for b, n in enumerate(lens):
        poisoned[b, :, :, n:] = np.nan
        poisoned[b, :, n:, :] = np.nan
    got = _np(_run_softmax(poisoned, lens, lens, 0.125))
    want = orc.masked_softmax_varlen(scores, lens, lens, 0.125)
    for b, n in enumerate(lens):
        assert_parity(got[b, :, :n, :], want[b, :, :n, :], F32, f"request {b}")
        assert (got[b, :, :n, n:] == 0).all()


def test_varlen_softmax_matches_the_padded_kernel_on_config_2():
    spec = wl.config_spec(2)
    case = wl.softmax_case(spec)
    lens = spec.lengths.astype(np.int32)
    padded = gu.run_softmax(case)
    got = _run_softmax(case.scores, lens, lens, case.scale)
    B, H, Sq, Sk = case.shape
    rows = gu.sample_rows(B * H * Sq, 400, seed=3)
    # oracle on the sampled rows: build per-row lengths through a [n,1,1,Sk] view (one "request" per row)
    b_of = rows // (H * Sq)
    q_of = rows % Sq
    sub = case.scores.reshape(-1, Sk)[rows].reshape(len(rows), 1, 1, Sk)
    k_len = lens[b_of]
    q_len = (q_of < lens[b_of]).astype(np.int32)  # 1 row per pseudo-request: active iff 0 < q_len
    want = orc.masked_softmax_varlen(sub, q_len, k_len, case.scale).reshape(len(rows), Sk)
    got_rows = _np(got.view(-1, Sk)[torch.from_numpy(rows).cuda()])
    assert_parity(got_rows, want, F32, "config 2 varlen, sampled rows")
    # on real rows the two kernels agree with each other to rounding (identical zeros on the padding keys)
    real = torch.from_numpy(np.repeat(np.arange(Sq)[None, :] < lens[:, None], H, axis=0).reshape(-1)).cuda()
    a, b = got.view(-1, Sk)[real], padded.view(-1, Sk)[real]
    assert (a - b).abs().max().item() < 2e-7
    assert ((a == 0) == (b == 0)).all()


@pytest.mark.parametrize("dtype", [F32, F16])
@pytest.mark.parametrize("path", [-1, tb.PATH_BLOCK, tb.PATH_STREAM])
def test_varlen_layernorm(dtype, path):
    rng = np.random.Generator(np.random.Philox(23))
    tdt = torch.float32 if dtype == F32 else torch.float16
    for B, S, hidden in [(1, 1, 8), (3, 5, 64), (4, 37, 768), (2, 9, 1000), (3, 7, 4096), (32, 50, 768)]:
        x = rng.standard_normal((B, S, hidden), dtype=np.float32).astype(dtype)
        r = rng.standard_normal((B, S, hidden), dtype=np.float32).astype(dtype)
        bias, gamma, beta = (rng.standard_normal((hidden,), dtype=np.float32).astype(dtype) for _ in range(3))
        lens = rng.integers(0, S + 1, size=B).astype(np.int32)
        lens[0] = S
        # poison the padding of the inputs and mark the padding of the output
        xp, rp = x.copy(), r.copy()
        for b, n in enumerate(lens):
            xp[b, n:] = np.nan
            rp[b, n:] = np.nan
        out = torch.full((B, S, hidden), -7.25, dtype=tdt, device="cuda")
        with gu.overrides(path=path):
            tb.turbo_add_bias_layernorm_varlen(gu.dev(xp), gu.dev(rp), gu.dev(bias), gu.dev(gamma), gu.dev(beta),
                                               torch.from_numpy(lens).cuda(), 1e-5, out)
            torch.cuda.synchronize()
        want = orc.add_bias_layernorm_varlen(x, r, bias, gamma, beta, lens, 1e-5, np.full((B, S, hidden), -7.25))
        assert_parity(_np(out), want, dtype, f"varlen layernorm B={B} S={S} hidden={hidden} path={path}")
        for b, n in enumerate(lens):
            assert (_np(out[b, n:]) == -7.25).all(), "a padding row was written"


def test_varlen_error_paths():
    L = tb.lib()
    fake = 0x10000
    assert L.turbo_masked_softmax_varlen(fake, None, None, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_NULL
    assert L.turbo_masked_softmax_varlen(fake, None, fake + 2, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_ALIGN
    assert L.turbo_masked_softmax_varlen(fake, None, fake, 1, 1, 0, 70000, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_SHAPE
    assert L.turbo_add_bias_layernorm_varlen(fake, fake, fake, fake, fake, None, 1, 4, 8, 1e-5, fake, tb.TURBO_F32, None) \
        == tb.TURBO_ERR_NULL
    assert L.turbo_add_bias_layernorm_varlen(fake, fake, fake, fake, fake, fake, 0, 4, 8, 1e-5, fake, tb.TURBO_F32, None) \
        == tb.TURBO_ERR_SHAPE


# ------------------------------------------------------------------ row-packed layout (no padding in memory)

def _run_packed(blocks_flat, lengths, H, scale, dtype, max_len=None, lead=0, tail=0):
    """Upload the flat packed scores into a buffer with `lead`/`tail` guard elements, run, return (result, buffer)."""
    tdt = torch.float32 if dtype == F32 else torch.float16
    cu, off = wl.packed_layout(lengths, H)
    n = blocks_flat.size
    buf = torch.full((lead + n + tail,), float("nan"), dtype=tdt, device="cuda")
    view = buf[lead:lead + n]
    view.copy_(torch.from_numpy(blocks_flat))
    tb.turbo_masked_softmax_packed(view, torch.from_numpy(cu).cuda(), torch.from_numpy(off).cuda(), H, int(cu[-1]),
                                   int(max(lengths)) if max_len is None else max_len, scale)
    torch.cuda.synchronize()
    return _np(view), buf


@pytest.mark.parametrize("dtype", [F32, F16])
def test_packed_softmax_shapes(dtype):
    rng = np.random.Generator(np.random.Philox(31))
    cases = [([1], 1), ([5], 2), ([3, 0, 1, 2], 3), ([8, 63, 64, 65], 2), ([100, 7, 257, 31, 4], 3), ([493, 5, 128, 500, 17], 12),
             ([1000, 3], 1), ([1500, 2], 1), ([2049, 40], 1), ([3000, 77], 1), ([4096, 9, 4095], 1),
             ([3, 1, 4, 1, 5, 9, 2, 6, 0] * 7, 2), ([3, 1, 4, 1, 5, 9, 2, 6] * 9, 2)]  # 63 and 72 requests: both table look-ups
    if dtype == F16:
        cases.append(([8192, 11, 5000], 1))
    for lengths, H in cases:
        total = H * sum(n * n for n in lengths)
        flat = (rng.standard_normal(total, dtype=np.float32) * 3).astype(dtype)
        want = orc.masked_softmax_packed(flat, lengths, H, 0.125)
        # the request-shaped kernel (up to 63 requests) with its own grid and with so small a grid that every
        # wavefront loops over several tasks, and the kernel that gives every row a whole wavefront
        for mode in ({}, {"grid_waves": 1}, {"path": 0}):
            for lead in (0, 3):  # row starts are only element-aligned either way; an odd base pointer on top
                with gu.overrides(**mode):
                    got, buf = _run_packed(flat, lengths, H, 0.125, dtype, lead=lead, tail=16)
                assert_parity(got, want, dtype, f"packed softmax lengths={lengths} H={H} lead={lead} {mode}")
                assert torch.isnan(buf[:lead]).all() and torch.isnan(buf[lead + total:]).all(), "wrote outside the batch"


@pytest.mark.parametrize("dtype", [F32, F16])
def test_packed_softmax_long_requests_take_a_workgroup_per_row(dtype):
    """Requests beyond one wavefront's registers (4096 binary32 / 8192 binary16 values per row) are served by a second
    launch over the same batch that gives every such row a workgroup; the shorter requests around them stay with the
    wavefront kernels.  max_len sizes the registers of that workgroup, so larger bounds run the same rows through
    every vectors-per-lane shape (2, 3, 4, 8)."""
    rng = np.random.Generator(np.random.Philox(35))
    wave_max = 4096 if dtype == F32 else 8192
    lengths, H = [wave_max + (404 if dtype == F32 else 108), 3] + ([wave_max + 1] if dtype == F32 else []) + [0, 77], 1
    lengths += [1100] * 23  # max_len may not exceed the token total: enough tokens for the largest bound
    total = H * sum(n * n for n in lengths)
    flat = (rng.standard_normal(total, dtype=np.float32) * 3).astype(dtype)
    orc.set_threads(gu.host_threads())
    want = orc.masked_softmax_packed(flat, lengths, H, 0.125)
    orc.set_threads(1)
    bounds = [max(lengths), 3 * 1024 * (4 if dtype == F32 else 8), 4 * 1024 * (4 if dtype == F32 else 8), 32768]
    for i, max_len in enumerate(sorted(set(bounds))):
        for mode in ({}, {"path": 0}) if i == 0 else ({},):
            with gu.overrides(**mode):
                got, buf = _run_packed(flat, lengths, H, 0.125, dtype, max_len=max_len, lead=3, tail=16)
            assert_parity(got, want, dtype, f"packed softmax, long requests, max_len={max_len} {mode}")
            assert torch.isnan(buf[:3]).all() and torch.isnan(buf[3 + total:]).all(), "wrote outside the batch"
    # a bound below the longest request: that request is left alone (or computed), everything else is computed
    got, _ = _run_packed(flat, lengths, H, 0.125, dtype, max_len=wave_max + 100, lead=0, tail=0)
    _, off = wl.packed_layout(lengths, H)
    assert_parity(got[off[1]:], want[off[1]:], dtype, "requests behind one that exceeds max_len")
    first = got[:off[1]]
    assert np.array_equal(first, flat[:off[1]]) or np.allclose(first, want[:off[1]], rtol=3e-3, atol=1e-6)


def test_packed_softmax_max_len_is_an_upper_bound_and_longer_requests_are_left_alone():
    rng = np.random.Generator(np.random.Philox(32))
    lengths, H = [40, 300, 9], 2
    total = H * sum(n * n for n in lengths)
    flat = rng.standard_normal(total, dtype=np.float32) * 3
    want = orc.masked_softmax_packed(flat, lengths, H, 0.5)
    got, _ = _run_packed(flat, lengths, H, 0.5, F32, max_len=349)       # any bound >= the longest request
    assert_parity(got, want, F32, "packed softmax with a loose max_len")
    got, _ = _run_packed(flat, lengths, H, 0.5, F32, max_len=256)       # request 1 does not fit 256 keys per row
    _, off = wl.packed_layout(lengths, H)
    np.testing.assert_array_equal(got[off[1]:off[2]], flat[off[1]:off[2]])
    assert_parity(got[:off[1]], want[:off[1]], F32, "request 0")
    assert_parity(got[off[2]:], want[off[2]:], F32, "request 2")


def test_packed_softmax_config_2_lengths_match_the_padded_length_aware_kernel():
    """Config 2's 32 requests, packed: the same numbers as the padded batch gives on its real part."""
    spec = wl.config_spec(2)
    lengths = [int(v) for v in spec.lengths]
    case = wl.softmax_case(spec)
    flat = np.concatenate([case.scores[b, :, :n, :n].reshape(-1) for b, n in enumerate(lengths)])
    got, _ = _run_packed(flat, lengths, spec.H, spec.scale, F32)
    _, off = wl.packed_layout(lengths, spec.H)
    for b in (0, 8, 23, 31):  # the oracle on a few whole requests (the longest, the shortest, two others)
        n = lengths[b]
        want = orc.masked_softmax_packed(flat[off[b]:off[b + 1]], [n], spec.H, spec.scale)
        assert_parity(got[off[b]:off[b + 1]], want, F32, f"packed config 2, request {b} of {n} tokens")
    sums = np.add.reduceat(got.astype(np.float64), np.concatenate(
        [off[b] + np.arange(spec.H * n) * n for b, n in enumerate(lengths)]))
    assert np.abs(sums - 1).max() < 1e-5


def test_packed_layernorm_is_the_plain_kernel_on_the_packed_tokens():
    rng = np.random.Generator(np.random.Philox(33))
    lengths, hidden = [17, 1, 300, 45], 768
    total = sum(lengths)
    case = wl.random_layernorm_case(34, total, hidden, eps=1e-5)
    assert_parity(_np(gu.run_layernorm(case)), gu.oracle_layernorm(case), F32, "LayerNorm over the packed tokens")


def test_packed_error_paths():
    # every call below must be rejected by the host-side validation: the pointers are not real
    L = tb.lib()
    fake = 0x10000
    f = L.turbo_masked_softmax_packed
    assert f(None, fake, fake, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_NULL
    assert f(fake, None, fake, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_NULL
    assert f(fake, fake, fake, 0, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_SHAPE
    assert f(fake, fake, fake, 1, 1, 4, 5, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_SHAPE     # max_len > total_tokens
    assert f(fake, fake, fake, 1, 1, 40000, 32769, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_SHAPE  # beyond one workgroup
    assert f(fake, fake, fake, 1, 1, 40000, 32769, 1.0, tb.TURBO_F16, None) == tb.TURBO_ERR_SHAPE
    assert f(fake, fake + 2, fake, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_ALIGN
    assert f(fake, fake, fake + 4, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_ALIGN
    assert f(fake, fake, fake, 1, 1, 4, 4, 1.0, 9, None) == tb.TURBO_ERR_DTYPE


# ------------------------------------------------------------------ causal variant

def _run_causal(scores, q_len, k_len, scale):
    s = gu.dev(scores)
    ql = None if q_len is None else torch.from_numpy(np.asarray(q_len, dtype=np.int32)).cuda()
    kl = None if k_len is None else torch.from_numpy(np.asarray(k_len, dtype=np.int32)).cuda()
    tb.turbo_masked_softmax_causal(s, ql, kl, scale)
    torch.cuda.synchronize()
    return s


@pytest.mark.parametrize("dtype", [F32, F16])
@pytest.mark.parametrize("path", [-1, tb.PATH_WAVE, tb.PATH_BLOCK, tb.PATH_STREAM])
def test_causal_softmax_shapes(dtype, path):
    """Keys above the diagonal are poisoned with NaN: they must be neither read into a result nor left in place."""
    rng = np.random.Generator(np.random.Philox(41))
    for B, H, Sq, Sk in [(1, 1, 1, 1), (2, 3, 7, 7), (2, 2, 16, 16), (3, 2, 33, 33), (2, 2, 64, 64), (2, 1, 100, 100), (2, 2, 128, 128),
                         (1, 2, 257, 257), (1, 1, 512, 512), (1, 1, 1000, 1000), (2, 1, 5, 133), (1, 2, 60, 493), (1, 1, 3, 4100),
                         (2, 1, 9, 4), (1, 1, 2100, 2100), (1, 1, 384, 384), (1, 1, 3, 640), (1, 1, 5, 768)]:
        scores = (rng.standard_normal((B, H, Sq, Sk), dtype=np.float32) * 3).astype(dtype)
        q_idx, k_idx = np.arange(Sq)[:, None], np.arange(Sk)[None, :]
        hidden = k_idx > q_idx + (Sk - Sq)
        poisoned = scores.copy()
        poisoned[:, :, hidden] = np.nan
        for use_lengths in (False, True):
            k_len = q_len = None
            if use_lengths:
                k_len = rng.integers(0, Sk + 1, size=B)
                q_len = rng.integers(0, Sq + 1, size=B)
                k_len[0], q_len[0] = Sk, Sq
            with gu.overrides(path=path):
                got = _np(_run_causal(poisoned, q_len, k_len, 0.125))
            want = orc.masked_softmax_causal(scores, q_len, k_len, 0.125)
            # rows the call leaves untouched keep their (poisoned) input; compare them bit for bit, the rest by value
            touched = np.ones((B, Sq), dtype=bool)
            visible = np.minimum(np.arange(Sq)[None, :] + (Sk - Sq) + 1, Sk if k_len is None else np.asarray(k_len)[:, None])
            touched &= np.broadcast_to(visible > 0, (B, Sq))
            if q_len is not None:
                touched &= np.arange(Sq)[None, :] < np.asarray(q_len)[:, None]
            what = f"causal softmax {B,H,Sq,Sk} path={path} lengths={use_lengths}"
            for b in range(B):
                live = touched[b]
                if live.any():
                    assert_parity(got[b][:, live], want[b][:, live], dtype, what)
                if (~live).any():
                    np.testing.assert_array_equal(got[b][:, ~live], poisoned[b][:, ~live])


def test_causal_softmax_on_config_4_matches_the_additive_mask_kernel():
    """GPT-2-medium scores [64,16,512,512] fp16: sampled rows against the oracle, and every element against what the
    additive 0 / -10000 mask kernel produces (the same exact zeros above the diagonal, fp16-close values below)."""
    spec = wl.config_spec(4)
    case = wl.softmax_case(spec)
    masked = gu.run_softmax(case)
    causal = _run_causal(case.scores, None, None, case.scale)
    B, H, Sq, Sk = case.shape
    rows = gu.sample_rows(B * H * Sq, 400, seed=44)
    got = _np(causal.view(-1, Sk)[torch.from_numpy(rows).cuda()])
    flat = case.scores.reshape(-1, Sk)[rows]
    for i, r in enumerate(rows[:200]):
        q = int(r % Sq)
        w = orc.masked_softmax(flat[i, :q + 1].reshape(1, 1, 1, q + 1), None, 0, 0, case.scale).reshape(-1)
        assert_parity(got[i, :q + 1], w, F16, f"causal config 4 row {r}")
        assert (got[i, q + 1:] == 0).all()
    diff = (causal.float() - masked.float()).abs().max().item()
    assert diff <= 2 ** -10, diff  # both round the same fp32 value to fp16, up to one ulp of values <= 1
    dead = torch.triu(torch.ones(Sq, Sk, dtype=torch.bool, device="cuda"), 1)
    assert (causal[:, :, dead] == 0).all()


def test_causal_error_paths():
    L = tb.lib()
    fake = 0x10000
    # every call below must be rejected by the host-side validation: the pointers are not real
    assert L.turbo_masked_softmax_causal(None, None, None, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_NULL
    assert L.turbo_masked_softmax_causal(fake, None, None, 1, 1, 0, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_SHAPE
    assert L.turbo_masked_softmax_causal(fake, fake + 2, None, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_ALIGN
    assert L.turbo_masked_softmax_causal(fake, None, None, 1, 1, 4, 4, 1.0, 3, None) == tb.TURBO_ERR_DTYPE


# ------------------------------------------------------------------ seeded random sweep over the length-aware entry points

import os


@pytest.mark.parametrize("chunk", range(int(os.environ.get("TURBO_TEST_SWEEP_CHUNKS", "4"))))
def test_randomized_length_aware_cases(chunk):
    rng = np.random.default_rng(7000 + chunk)
    special = [1, 2, 3, 4, 7, 8, 16, 17, 33, 64, 65, 96, 128, 160, 192, 257, 384, 493, 512, 640, 768, 1000, 1280, 2048, 4100]
    for case_no in range(40):
        dtype = F32 if rng.random() < 0.5 else F16
        kind = str(rng.choice(["varlen", "causal", "packed", "layernorm"]))
        path = int(rng.choice([-1, -1, tb.PATH_WAVE, tb.PATH_BLOCK, tb.PATH_STREAM]))
        cap = int(rng.choice([-1, -1, -1, 4, 8, 16]))
        if cap != -1 and cap < np.dtype(dtype).itemsize:
            cap = -1
        S = int(rng.choice(special)) if rng.random() < 0.7 else int(rng.integers(1, 1500))
        B, H = int(rng.integers(1, 5)), int(rng.integers(1, 4))
        what = f"chunk {chunk} case {case_no}: {kind} {np.dtype(dtype).name} B={B} H={H} S={S} path={path} cap={cap}"
        if kind in ("varlen", "causal"):
            Sq = S if rng.random() < 0.5 else int(rng.integers(1, max(2, min(S, 24) + 1)))
            Sq = min(Sq, max(1, 200000 // (S * B * H)))
            scores = (rng.standard_normal((B, H, Sq, S), dtype=np.float32) * 3).astype(dtype)
            k_len = rng.integers(0, S + 1, size=B)
            q_len = rng.integers(0, Sq + 1, size=B)
            use_q = rng.random() < 0.6
            with gu.overrides(path=path, max_vec_bytes=cap):
                if kind == "varlen":
                    got = _np(_run_softmax(scores, q_len if use_q else None, k_len, 0.125))
                    want = orc.masked_softmax_varlen(scores, q_len if use_q else None, k_len, 0.125)
                else:
                    use_k = rng.random() < 0.5
                    got = _np(_run_causal(scores, q_len if use_q else None, k_len if use_k else None, 0.125))
                    want = orc.masked_softmax_causal(scores, q_len if use_q else None, k_len if use_k else None, 0.125)
            assert_parity(got, want, dtype, what)
        elif kind == "packed":
            lengths = [int(v) for v in rng.integers(0, min(S, 600) + 1, size=B)]
            lengths[0] = max(1, min(S, 600))
            total = H * sum(n * n for n in lengths)
            flat = (rng.standard_normal(total, dtype=np.float32) * 3).astype(dtype)
            lead = int(rng.integers(0, 4))
            got, buf = _run_packed(flat, lengths, H, 0.125, dtype, max_len=max(lengths) + int(rng.integers(0, 50)) if sum(lengths) > max(lengths) + 50 else None, lead=lead, tail=8)
            assert_parity(got, orc.masked_softmax_packed(flat, lengths, H, 0.125), dtype, what + f" lengths={lengths}")
            assert torch.isnan(buf[:lead]).all() and torch.isnan(buf[lead + total:]).all(), what
        else:
            hidden = max(S, 8)
            Sq = max(1, min(int(rng.integers(1, 30)), 100000 // (hidden * B)))
            tdt = torch.float32 if dtype == F32 else torch.float16
            normal = lambda shape, std, mean=0.0: (rng.standard_normal(shape, dtype=np.float32) * np.float32(std) + np.float32(mean)).astype(dtype)
            x, res = normal((B, Sq, hidden), 1.0), normal((B, Sq, hidden), 1.0)
            bias, gamma, beta = normal((hidden,), 0.1), normal((hidden,), 0.1, 1.0), normal((hidden,), 0.1)
            lens = rng.integers(0, Sq + 1, size=B).astype(np.int32)
            out = torch.full((B, Sq, hidden), -7.25, dtype=tdt, device="cuda")
            with gu.overrides(path=path, max_vec_bytes=cap):
                tb.turbo_add_bias_layernorm_varlen(gu.dev(x), gu.dev(res), gu.dev(bias), gu.dev(gamma), gu.dev(beta), gu.dev(lens), 1e-5, out)
            torch.cuda.synchronize()
            want = orc.add_bias_layernorm_varlen(x, res, bias, gamma, beta, lens, 1e-5, np.full((B, Sq, hidden), -7.25))
            assert_parity(_np(out), want, dtype, what)
