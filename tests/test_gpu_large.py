"""Tensors with more than 2^31 elements (more than 4 GiB): every row offset needs 64-bit arithmetic.

The tensors are built on the device from one seeded host block, repeated with a different power-of-two-friendly scale
per repetition (so a wrapped 32-bit offset would land on different data); the oracle sees exactly the rows that the
device holds: sampled rows are copied back before the kernel runs.  Samples sit at both ends and on both sides of
element 2^31 (= byte 2^32 for binary16).
"""
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
BLOCK_ROWS = 4096


def _np(t):
    return t.detach().cpu().numpy()


def _tiled(block: np.ndarray, n_rows: int) -> torch.Tensor:
    """[n_rows, L] device tensor: repetition i of the block is scaled by 1 + (i mod 13)/16 (exact in binary16)."""
    assert n_rows % BLOCK_ROWS == 0 and block.shape[0] == BLOCK_ROWS
    b = gu.dev(block)
    big = torch.empty((n_rows, block.shape[1]), dtype=b.dtype, device="cuda")
    view = big.view(n_rows // BLOCK_ROWS, BLOCK_ROWS, block.shape[1])
    for i in range(view.shape[0]):
        torch.mul(b, 1.0 + (i % 13) / 16.0, out=view[i])
    return big


def _rows_around_2_31(n_rows: int, row_len: int, seed: int) -> np.ndarray:
    assert n_rows * row_len > 2**31
    edge = 2**31 // row_len
    picks = set(np.random.default_rng(seed).integers(0, n_rows, size=200).tolist())
    picks.update(r for r in (0, 1, edge - 2, edge - 1, edge, edge + 1, edge + 2, n_rows - 2, n_rows - 1) if 0 <= r < n_rows)
    return np.array(sorted(picks), dtype=np.int64)


def _block(seed, row_len, dtype, std):
    rng = np.random.Generator(np.random.Philox(wl.SEED_BASE + seed))
    return (rng.standard_normal((BLOCK_ROWS, row_len), dtype=np.float32) * np.float32(std)).astype(dtype)


@pytest.mark.parametrize("B,H,Sq,Sk", [(3, 11, 8192, 8192), (130, 16, 8192, 128)], ids=["rows-of-8192", "rows-of-128"])
def test_softmax_beyond_2_31_elements(B, H, Sq, Sk):
    n_rows = B * H * Sq
    print(f"softmax {B,H,Sq,Sk} binary16, {n_rows * Sk / 2**31:.3f} x 2^31 elements", flush=True)
    scores = _tiled(_block(901, Sk, F16, 3.0), n_rows)
    lengths = np.array([max(1, (Sk * (3 + 2 * b)) // (3 + 2 * B)) for b in range(B)], dtype=np.int32)
    mask = wl.key_mask_from_lengths(lengths, Sk, F16)
    rows = _rows_around_2_31(n_rows, Sk, seed=1)
    before = _np(scores[torch.from_numpy(rows).cuda()])
    tb.turbo_masked_softmax_ex(scores.view(B, H, Sq, Sk), gu.dev(mask), Sk, 0, 0.125)
    torch.cuda.synchronize()
    got = _np(scores[torch.from_numpy(rows).cuda()])
    b_of_row = rows // (H * Sq)
    want = orc.masked_softmax(before.reshape(1, 1, len(rows), Sk), mask[b_of_row], len(rows) * Sk, Sk, 0.125)
    assert_parity(got, want.reshape(len(rows), Sk), F16, "softmax beyond 2^31 elements, sampled rows")
    # every row was rewritten: sums are 1 everywhere (checked in slabs to bound the temporary)
    worst = 0.0
    for r0 in range(0, n_rows, 1 << 16):
        worst = max(worst, (scores[r0:r0 + (1 << 16)].float().sum(-1) - 1).abs().max().item())
    assert worst < 3e-3, worst


def test_varlen_softmax_beyond_2_31_elements():
    B, H, Sq, Sk = 3, 11, 8192, 8192
    n_rows = B * H * Sq
    scores = _tiled(_block(902, Sk, F16, 3.0), n_rows)
    k_len = np.array([5000, 8192, 77], dtype=np.int32)
    q_len = np.array([8192, 6000, 8192], dtype=np.int32)
    rows = _rows_around_2_31(n_rows, Sk, seed=2)
    before = _np(scores[torch.from_numpy(rows).cuda()])
    tb.turbo_masked_softmax_varlen(scores.view(B, H, Sq, Sk), gu.dev(q_len), gu.dev(k_len), 0.125)
    torch.cuda.synchronize()
    got = _np(scores[torch.from_numpy(rows).cuda()])
    b_of_row, q_of_row = rows // (H * Sq), rows % Sq
    for i, (b, q) in enumerate(zip(b_of_row, q_of_row)):
        if q >= q_len[b]:
            np.testing.assert_array_equal(got[i], before[i])  # padding rows are left alone
            continue
        want = orc.masked_softmax(before[i, :k_len[b]].reshape(1, 1, 1, -1), None, 0, 0, 0.125).reshape(-1)
        assert_parity(got[i, :k_len[b]], want, F16, f"varlen softmax beyond 2^31 elements, row {rows[i]}")
        assert (got[i, k_len[b]:] == 0).all()


@pytest.mark.parametrize("n_rows,hidden,dtype", [(270336, 8192, F16), (2801664, 768, F32)], ids=["f16-8192", "f32-768"])
def test_layernorm_beyond_2_31_elements(n_rows, hidden, dtype):
    print(f"layernorm {n_rows}x{hidden} {np.dtype(dtype).name}, {n_rows * hidden / 2**31:.3f} x 2^31 elements", flush=True)
    x = _tiled(_block(903, hidden, dtype, 1.0), n_rows)
    res = _tiled(_block(904, hidden, dtype, 1.0), n_rows)
    rng = np.random.Generator(np.random.Philox(wl.SEED_BASE + 905))
    bias, beta = ((rng.standard_normal(hidden, dtype=np.float32) * np.float32(0.1)).astype(dtype) for _ in range(2))
    gamma = (1 + rng.standard_normal(hidden, dtype=np.float32) * np.float32(0.1)).astype(dtype)
    eps = 1e-5
    out = torch.full_like(x, float("nan"))
    tb.turbo_add_bias_layernorm_dt(x, res, gu.dev(bias), gu.dev(gamma), gu.dev(beta), eps, out)
    torch.cuda.synchronize()
    rows = _rows_around_2_31(n_rows, hidden, seed=3)
    sel = torch.from_numpy(rows).cuda()
    want = orc.add_bias_layernorm(_np(x[sel]), _np(res[sel]), bias, gamma, beta, eps)
    assert_parity(_np(out[sel]), want, dtype, "layernorm beyond 2^31 elements, sampled rows")
    for r0 in range(0, n_rows, 1 << 18):
        assert torch.isfinite(out[r0:r0 + (1 << 18)]).all(), "a row was not written"


def test_elementwise_beyond_2_31_elements():
    rows_n, hidden = 270336, 8192
    x = _tiled(_block(906, hidden, F16, 1.5), rows_n)
    rng = np.random.Generator(np.random.Philox(wl.SEED_BASE + 907))
    bias = (rng.standard_normal(hidden, dtype=np.float32) * np.float32(0.5)).astype(F16)
    out = torch.full_like(x, float("nan"))
    tb.turbo_add_bias_gelu(x, gu.dev(bias), False, out)
    torch.cuda.synchronize()
    rows = _rows_around_2_31(rows_n, hidden, seed=4)
    sel = torch.from_numpy(rows).cuda()
    assert_parity(_np(out[sel]), orc.add_bias_gelu(_np(x[sel]), bias), F16, "gelu beyond 2^31 elements, sampled rows")
    for r0 in range(0, rows_n, 1 << 16):
        assert torch.isfinite(out[r0:r0 + (1 << 16)]).all()
    del out
    # head split [B,S,3,H,D] -> [3,B,H,S,D] and merge back-to-front on the same storage size
    B, S, K, H, D = 88, 8192, 3, 16, 64
    assert B * S * K * H * D == rows_n * hidden
    x5 = x.view(B, S, K, H, D)
    hb = (rng.standard_normal((K, H, D), dtype=np.float32) * np.float32(0.3)).astype(F16)
    o5 = torch.full((K, B, H, S, D), float("nan"), dtype=torch.float16, device="cuda")
    tb.turbo_add_bias_split_heads(x5, gu.dev(hb), o5)
    torch.cuda.synchronize()
    for b in (0, B // 2 - 1, B // 2, B - 1):  # element 2^31 lies in the middle batch
        for s in (0, 4095, 8191):
            want = orc.add_bias_split_heads(_np(x5[b:b + 1, s:s + 1]), hb)
            assert_parity(_np(o5[:, b:b + 1, :, s:s + 1]), want, F16, f"split heads beyond 2^31 elements, b={b} s={s}")
    del x5, x
    m_in = o5.view(3 * B, H, S, D)  # the three parts as one batch of 3B: again more than 2^31 elements
    m_out = torch.full((3 * B, S, H, D), float("nan"), dtype=torch.float16, device="cuda")
    tb.turbo_merge_heads(m_in, m_out)
    torch.cuda.synchronize()
    for b in (0, 3 * B // 2, 3 * B - 1):
        np.testing.assert_array_equal(_np(m_out[b:b + 1]).astype(np.float64), orc.merge_heads(_np(m_in[b:b + 1])))
