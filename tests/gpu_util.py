"""Helpers for the GPU parity tests: upload a case, run the HIP path through the C ABI, fetch the result,
and evaluate the oracle on all rows or on a sample of rows."""
from __future__ import annotations

import contextlib

import numpy as np
import torch

from oracle import turbo_oracle as orc
from paper_2010_05680_amd import binding as tb


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


@contextlib.contextmanager
def overrides(path=-1, max_vec_bytes=-1, grid_waves=-1, block_waves=-1, grid_blocks=-1):
    tb.turbo_set_override(tb.TURBO_OVR_BLOCK_WAVES, block_waves)
    tb.turbo_set_override(tb.TURBO_OVR_GRID_BLOCKS, grid_blocks)
    tb.turbo_set_override(tb.TURBO_OVR_PATH, path)
    tb.turbo_set_override(tb.TURBO_OVR_MAX_VEC_BYTES, max_vec_bytes)
    tb.turbo_set_override(tb.TURBO_OVR_GRID_WAVES, grid_waves)
    try:
        yield
    finally:
        for k in (tb.TURBO_OVR_PATH, tb.TURBO_OVR_MAX_VEC_BYTES, tb.TURBO_OVR_GRID_WAVES, tb.TURBO_OVR_BLOCK_WAVES,
                  tb.TURBO_OVR_GRID_BLOCKS):
            tb.turbo_set_override(k, -1)


def run_softmax(case, stream=None) -> torch.Tensor:
    """HIP path on a SoftmaxCase; returns the device tensor holding the result."""
    s = dev(case.scores)
    m = None if case.mask is None else dev(case.mask)
    tb.turbo_masked_softmax_ex(s, m, case.mask_stride_b, case.mask_stride_q, case.scale, stream=stream)
    torch.cuda.synchronize()
    return s


def oracle_softmax(case) -> np.ndarray:
    return orc.masked_softmax(case.scores, case.mask, case.mask_stride_b, case.mask_stride_q, case.scale)


def oracle_softmax_rows(case, rows: np.ndarray) -> np.ndarray:
    """Oracle on selected rows of the flattened [B*H*Sq, Sk] view (rows are independent)."""
    B, H, Sq, Sk = case.scores.shape
    flat = case.scores.reshape(-1, Sk)
    sub = flat[rows].reshape(1, 1, len(rows), Sk)
    if case.mask is None:
        return orc.masked_softmax(sub, None, 0, 0, case.scale).reshape(len(rows), Sk)
    b = rows // (H * Sq)
    q = rows % Sq
    mflat = case.mask.reshape(-1)
    start = b * case.mask_stride_b + q * case.mask_stride_q
    mrows = np.stack([mflat[s0:s0 + Sk] for s0 in start])
    return orc.masked_softmax(sub, mrows, len(rows) * Sk, Sk, case.scale).reshape(len(rows), Sk)


def run_layernorm(case, out=None, stream=None, residual=True, bias=True):
    x = dev(case.x)
    r = dev(case.residual) if residual else None
    b = dev(case.bias) if bias else None
    g, be = dev(case.gamma), dev(case.beta)
    if out is None:
        out = torch.full_like(x, float("nan"))
    tb.turbo_add_bias_layernorm_dt(x, r, b, g, be, case.eps, out, stream=stream)
    torch.cuda.synchronize()
    return out


def oracle_layernorm(case, residual=True, bias=True, rows=None) -> np.ndarray:
    x = case.x if rows is None else case.x[rows]
    r = None if not residual else (case.residual if rows is None else case.residual[rows])
    return orc.add_bias_layernorm(x, r, case.bias if bias else None, case.gamma, case.beta, case.eps)


def sample_rows(n_rows: int, n: int, seed: int, tile: int = 512) -> np.ndarray:
    """Random rows plus the first/last rows and rows on both sides of tile boundaries."""
    rng = np.random.default_rng(seed)
    picks = set(rng.integers(0, n_rows, size=n).tolist())
    for r in (0, 1, tile - 1, tile, tile + 1, n_rows // 2, n_rows - tile - 1, n_rows - 2, n_rows - 1):
        if 0 <= r < n_rows:
            picks.add(int(r))
    return np.array(sorted(picks), dtype=np.int64)


# ---------------------------------------------------------------------------------------------------------------
# every element of a full-size tensor against the oracle, in slabs that keep the float64 temporaries small
# ---------------------------------------------------------------------------------------------------------------

FULL_CHUNK_ELEMS = 1 << 25  # elements per oracle call: four float64 temporaries of 256 MB each


def host_threads() -> int:
    """Host threads the oracle's row loop may use here (the GPU machine gives a one-GPU job 16)."""
    import os
    n = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    return max(1, min(16, n))


class ErrorStats:
    """Running maxima of what conftest.assert_parity returns, plus the element count."""

    def __init__(self):
        self.max_abs, self.max_rel, self.max_share, self.n = 0.0, 0.0, 0.0, 0

    def add(self, err, n):
        self.max_abs, self.max_rel = max(self.max_abs, err[0]), max(self.max_rel, err[1])
        self.max_share = max(self.max_share, err[2])
        self.n += int(n)

    def line(self, what):
        return (f"error report: {what} (all elements, {self.n}): max abs {self.max_abs:.3e}, max rel {self.max_rel:.3e}, "
                f"{100 * self.max_share:.0f} % of the bound")


def softmax_slabs(shape, part=0, n_parts=1):
    """(b, h0, h1) slabs of whole heads of one request, at most FULL_CHUNK_ELEMS elements each; the slabs are dealt
    round-robin to `n_parts` parts so that every part sees every region of the tensor."""
    B, H, Sq, Sk = shape
    hc = max(1, min(H, FULL_CHUNK_ELEMS // (Sq * Sk)))
    slabs = [(b, h0, min(H, h0 + hc)) for b in range(B) for h0 in range(0, H, hc)]
    return slabs[part::n_parts]


def oracle_softmax_slab(case, b, h0, h1) -> np.ndarray:
    """The additive-mask oracle on scores[b, h0:h1]: the mask of request b, shared by the heads."""
    sub = case.scores[b:b + 1, h0:h1]
    if case.mask is None:
        return orc.masked_softmax(sub, None, 0, 0, case.scale)[0]
    m = case.mask.reshape(-1)[b * case.mask_stride_b:]
    return orc.masked_softmax(sub, m, 0, case.mask_stride_q, case.scale)[0]


def row_ranges(n_rows, row_len, part=0, n_parts=1):
    step = max(1, FULL_CHUNK_ELEMS // row_len)
    ranges = [(r0, min(n_rows, r0 + step)) for r0 in range(0, n_rows, step)]
    return ranges[part::n_parts]
