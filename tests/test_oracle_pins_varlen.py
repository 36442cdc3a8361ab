"""Pins for the oracle's length-aware variants (zero-padded variable-length batches)."""
import numpy as np
import pytest
import torch

from oracle import turbo_oracle as orc
from paper_2010_05680_amd import workloads as wl


def test_varlen_softmax_by_hand():
    # one request, 4 keys of which 3 are real: the weights of logs of 1, 2, 3 and an exact zero; second query row is padding
    s = np.array([[0.0, 8 * np.log(2), 8 * np.log(3), 123.0], [5.0, 6.0, 7.0, 8.0]]).reshape(1, 1, 2, 4)
    y = orc.masked_softmax_varlen(s, [1], [3], 0.125)
    np.testing.assert_allclose(y[0, 0, 0], [1 / 6, 1 / 3, 1 / 2, 0.0], rtol=1e-14)
    assert y[0, 0, 0, 3] == 0.0
    np.testing.assert_array_equal(y[0, 0, 1], [5.0, 6.0, 7.0, 8.0])  # untouched
    # no query lengths: every row is computed
    y = orc.masked_softmax_varlen(s, None, [3], 0.125)
    assert y[0, 0, 1, 3] == 0.0 and y[0, 0, 1, :3].sum() == pytest.approx(1.0)
    # a request without keys is left alone
    np.testing.assert_array_equal(orc.masked_softmax_varlen(s, None, [0], 0.125), s)


def test_varlen_softmax_equals_library_softmax_on_the_real_part():
    rng = np.random.default_rng(0)
    B, H, S = 4, 3, 9
    s = rng.normal(size=(B, H, S, S)) * 3
    lens = np.array([9, 1, 5, 7])
    y = orc.masked_softmax_varlen(s, lens, lens, 0.3)
    for b, n in enumerate(lens):
        want = torch.softmax(torch.from_numpy(s[b, :, :n, :n]) * 0.3, -1).numpy()
        np.testing.assert_allclose(y[b, :, :n, :n], want, rtol=1e-13)
        assert (y[b, :, :n, n:] == 0).all()
        np.testing.assert_array_equal(y[b, :, n:, :], s[b, :, n:, :])


def test_varlen_softmax_agrees_with_the_padded_formulation_on_real_rows():
    """The additive 0 / -10000 key mask of the padded batch gives the same weights: exp underflows to the same zeros."""
    case = wl.random_softmax_case(5, 3, 2, 12, 12, mask_kind="key")
    padded = orc.masked_softmax(case.scores, case.mask, case.mask_stride_b, case.mask_stride_q, case.scale)
    y = orc.masked_softmax_varlen(case.scores, None, case.lengths, case.scale)
    np.testing.assert_allclose(y, padded, rtol=1e-13, atol=0)


def test_varlen_layernorm_touches_only_real_rows():
    rng = np.random.default_rng(1)
    B, S, hidden = 3, 6, 16
    x, r = rng.normal(size=(B, S, hidden)), rng.normal(size=(B, S, hidden))
    b, g, be = rng.normal(size=hidden), rng.normal(size=hidden), rng.normal(size=hidden)
    before = np.full((B, S, hidden), -7.25)
    lens = [6, 0, 2]
    y = orc.add_bias_layernorm_varlen(x, r, b, g, be, lens, 1e-5, before)
    T = torch.from_numpy
    want = torch.nn.functional.layer_norm(T(x) + T(b) + T(r), (hidden,), T(g), T(be), 1e-5).numpy()
    for bi, n in enumerate(lens):
        np.testing.assert_allclose(y[bi, :n], want[bi, :n], rtol=1e-11, atol=1e-13)
        assert (y[bi, n:] == -7.25).all()


# ------------------------------------------------------------------ row-packed layout (no padding in memory)

def _pack(blocks):
    return np.concatenate([b.reshape(-1) for b in blocks])


def test_packed_softmax_by_hand():
    # two requests, one head: lengths 3 and 1.  Scores 0, 8 ln 2, 8 ln 3 at scale 1/8 weigh 1 : 2 : 3.
    r0 = np.array([[0.0, 8 * np.log(2), 8 * np.log(3)], [1.0, 1.0, 1.0], [0.0, 8 * np.log(3), 0.0]])
    r1 = np.array([[42.0]])
    y = orc.masked_softmax_packed(_pack([r0, r1]), [3, 1], 1, 0.125)
    np.testing.assert_allclose(y[0:3], [1 / 6, 1 / 3, 1 / 2], rtol=1e-14)
    np.testing.assert_allclose(y[3:6], [1 / 3] * 3, rtol=1e-14)
    np.testing.assert_allclose(y[6:9], [1 / 5, 3 / 5, 1 / 5], rtol=1e-14)
    assert y[9] == 1.0 and y.size == 10


def test_packed_softmax_equals_library_softmax_per_request_and_skips_empty_requests():
    rng = np.random.default_rng(3)
    H, lens = 3, [4, 0, 1, 7, 2]
    blocks = [rng.normal(size=(H, n, n)) * 3 for n in lens]
    y = orc.masked_softmax_packed(_pack(blocks), lens, H, 0.25)
    pos = 0
    for n, blk in zip(lens, blocks):
        want = torch.softmax(torch.from_numpy(blk) * 0.25, -1).numpy()
        np.testing.assert_allclose(y[pos:pos + H * n * n].reshape(H, n, n), want, rtol=1e-13)
        pos += H * n * n
    assert pos == y.size
    with pytest.raises(ValueError):
        orc.masked_softmax_packed(np.zeros(5), [2], 1, 1.0)


def test_packed_softmax_is_the_padded_batch_without_its_padding():
    """Packing is a change of layout only: the real part of the zero-padded batch, computed by the length-aware
    oracle, is the packed result element for element."""
    rng = np.random.default_rng(4)
    B, H, S = 3, 2, 6
    lens = np.array([6, 2, 5])
    padded = rng.normal(size=(B, H, S, S)) * 2
    y_pad = orc.masked_softmax_varlen(padded, lens, lens, 0.5)
    y = orc.masked_softmax_packed(_pack([padded[b, :, :n, :n] for b, n in enumerate(lens)]), lens, H, 0.5)
    np.testing.assert_array_equal(y, _pack([y_pad[b, :, :n, :n] for b, n in enumerate(lens)]))


def test_packed_softmax_with_one_request_longer_than_a_wavefront_can_hold():
    """A request of 4500 keys beside short ones (rows of 4500 values need more than the 4096 binary32 values one
    wavefront's registers hold, so the HIP path serves it with a workgroup per row): the library softmax per request,
    a closed form, and the offsets of the requests behind the long one."""
    rng = np.random.default_rng(5)
    H, lens = 1, [3, 4500, 2]
    blocks = [rng.normal(size=(H, n, n)) * 3 for n in lens]
    # row 7 of the long request: a geometric progression, z_k = k ln(r) with r = 0.999: weights r^k (1 - r) / (1 - r^n)
    n, r = 4500, 0.999
    blocks[1][0, 7] = np.arange(n) * np.log(r) / 0.25
    y = orc.masked_softmax_packed(_pack(blocks), lens, H, 0.25)
    pos = 0
    for m, blk in zip(lens, blocks):
        want = torch.softmax(torch.from_numpy(blk) * 0.25, -1).numpy()
        np.testing.assert_allclose(y[pos:pos + H * m * m].reshape(H, m, m), want, rtol=1e-12, atol=1e-300)
        pos += H * m * m
    assert pos == y.size
    closed = r ** np.arange(n) * (1 - r) / (1 - r ** n)
    np.testing.assert_allclose(y[9 + 7 * n:9 + 8 * n], closed, rtol=1e-11)
    np.testing.assert_allclose(y[9:9 + n * n].reshape(n, n).sum(-1), 1.0, rtol=0, atol=1e-12)


# ------------------------------------------------------------------ causal variant

def test_causal_softmax_by_hand():
    # 3 queries over 3 keys: row q sees keys 0..q.  Scores 0, 8 ln 2, 8 ln 3 at scale 1/8 weigh 1 : 2 : 3.
    row = [0.0, 8 * np.log(2), 8 * np.log(3)]
    s = np.array([row, row, row]).reshape(1, 1, 3, 3)
    y = orc.masked_softmax_causal(s, None, None, 0.125)[0, 0]
    np.testing.assert_allclose(y[0], [1.0, 0.0, 0.0], rtol=1e-14)
    np.testing.assert_allclose(y[1], [1 / 3, 2 / 3, 0.0], rtol=1e-14)
    np.testing.assert_allclose(y[2], [1 / 6, 1 / 3, 1 / 2], rtol=1e-14)
    assert y[0, 1] == 0.0 and y[0, 2] == 0.0 and y[1, 2] == 0.0
    # more keys than queries (a cache of 2 earlier keys): the diagonal moves right by Sk - Sq, the last query sees all
    s = np.zeros((1, 1, 2, 4))
    y = orc.masked_softmax_causal(s, None, None, 1.0)[0, 0]
    np.testing.assert_allclose(y, [[1 / 3, 1 / 3, 1 / 3, 0.0], [0.25] * 4], rtol=1e-14)
    # more queries than keys: the first Sq - Sk queries see nothing and are left alone
    s = np.arange(6.0).reshape(1, 1, 3, 2)
    y = orc.masked_softmax_causal(s, None, None, 1.0)[0, 0]
    np.testing.assert_array_equal(y[0], s[0, 0, 0])
    np.testing.assert_allclose(y[1], [1.0, 0.0])
    assert y[2].sum() == pytest.approx(1.0) and (y[2] > 0).all()


@pytest.mark.parametrize("Sq,Sk", [(7, 7), (5, 9), (12, 12)])
def test_causal_softmax_equals_library_softmax_under_a_triangular_mask(Sq, Sk):
    rng = np.random.default_rng(Sq * 100 + Sk)
    B, H = 3, 2
    s = rng.normal(size=(B, H, Sq, Sk)) * 3
    y = orc.masked_softmax_causal(s, None, None, 0.3)
    keep = torch.ones(Sq, Sk, dtype=torch.bool).tril(diagonal=Sk - Sq)
    z = (torch.from_numpy(s) * 0.3).masked_fill(~keep, float("-inf"))
    np.testing.assert_allclose(y, torch.softmax(z, -1).numpy(), rtol=1e-13)
    assert (y[..., ~keep.numpy()] == 0).all()
    # the padded formulation with an additive 0 / -10000 mask above the diagonal gives the same weights (square case)
    if Sq == Sk:
        padded = orc.masked_softmax(s, wl.causal_mask(Sq, Sk, np.float64), 0, Sk, 0.3)
        np.testing.assert_allclose(y, padded, rtol=1e-12, atol=1e-300)


def test_causal_softmax_with_request_lengths():
    rng = np.random.default_rng(9)
    B, H, S = 3, 2, 8
    s = rng.normal(size=(B, H, S, S))
    k_len, q_len = np.array([8, 3, 5]), np.array([8, 8, 4])
    y = orc.masked_softmax_causal(s, q_len, k_len, 1.0)
    for b in range(B):
        for q in range(S):
            if q >= q_len[b]:
                np.testing.assert_array_equal(y[b, :, q], s[b, :, q])
                continue
            n = min(q + 1, k_len[b])
            want = torch.softmax(torch.from_numpy(s[b, :, q, :n]), -1).numpy()
            np.testing.assert_allclose(y[b, :, q, :n], want, rtol=1e-13)
            assert (y[b, :, q, n:] == 0).all()
