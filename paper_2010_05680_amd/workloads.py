"""Seeded synthetic inputs for the two batch-reduction kernels.

This module only draws random tensors and describes shapes.  It contains none
of the arithmetic of softmax or LayerNorm, so both the CPU oracle's tests and
the HIP path's tests/bench may import it without sharing any method code.

The paper's own benchmark inputs are random tensors from a fixed seed, and its
variable-length workload draws request lengths uniformly from 5 to 500
(Section 6.2, variable-length experiment).  The five configurations below use
the same recipe: normal scores, additive 0/-10000 masks, zero-padded batches.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

SEED_BASE = 20100568
MASK_VALUE = -10000.0

# tensor indices used to derive per-tensor seeds
_T_SCORES, _T_LENGTHS, _T_X, _T_RES, _T_BIAS, _T_GAMMA, _T_BETA = range(7)


def _rng(cfg_index: int, tensor_index: int, seed_base: int = SEED_BASE) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(seed_base + 1000 * cfg_index + tensor_index))


def _normal(rng: np.random.Generator, shape, mean: float, std: float, dtype) -> np.ndarray:
    """N(mean, std^2) drawn in fp32, then rounded (nearest-even) to `dtype`."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    step = 1 << 24
    for lo in range(0, n, step):  # chunked so the temporary stays small
        hi = min(n, lo + step)
        blk = rng.standard_normal(hi - lo, dtype=np.float32)
        blk *= np.float32(std)
        if mean != 0.0:
            blk += np.float32(mean)
        out[lo:hi] = blk
    out = out.reshape(shape)
    return out if dtype == np.float32 else out.astype(dtype)


@dataclass
class SoftmaxCase:
    scores: np.ndarray                 # [B, H, Sq, Sk], contiguous, fp32 or fp16
    mask: Optional[np.ndarray]         # additive mask in the scores' dtype, or None
    mask_stride_b: int                 # element strides of the mask (0 = broadcast)
    mask_stride_q: int
    scale: float
    mask_kind: str                     # "none" | "key" | "causal" | "dense"
    lengths: Optional[np.ndarray] = None

    @property
    def shape(self):
        return self.scores.shape

    @property
    def algorithmic_bytes(self) -> int:
        s = self.scores.dtype.itemsize
        return 2 * s * self.scores.size + (0 if self.mask is None else self.mask.size * s)


@dataclass
class LayerNormCase:
    x: np.ndarray          # [rows, hidden]
    residual: np.ndarray   # [rows, hidden]
    bias: np.ndarray       # [hidden]
    gamma: np.ndarray      # [hidden]
    beta: np.ndarray       # [hidden]
    eps: float

    @property
    def shape(self):
        return self.x.shape

    @property
    def algorithmic_bytes(self) -> int:
        s = self.x.dtype.itemsize
        return 3 * s * self.x.size + 3 * s * self.x.shape[1]


@dataclass
class ConfigSpec:
    index: int
    name: str
    dtype: type
    B: int
    H: int
    Sq: int
    Sk: int
    score_std: float
    scale: float
    mask_kind: str
    rows: int
    hidden: int
    eps: float
    lengths: Optional[np.ndarray] = field(default=None, repr=False)


def variable_lengths(cfg_index: int = 2, n_requests: int = 32, lo: int = 5, hi: int = 500,
                     seed_base: int = SEED_BASE) -> np.ndarray:
    """Request lengths, uniform on the integers lo..hi (both inclusive)."""
    return _rng(cfg_index, _T_LENGTHS, seed_base).integers(lo, hi + 1, size=n_requests, dtype=np.int64)


def config_spec(index: int, seed_base: int = SEED_BASE) -> ConfigSpec:
    if index == 0:
        return ConfigSpec(0, "tiny-bert-base-fp32", np.float32, 1, 12, 16, 16, 3.0, 0.125, "key",
                          16, 768, 1e-12, lengths=np.array([12], dtype=np.int64))
    if index == 1:
        return ConfigSpec(1, "bert-base-serving-b20-s128-fp32", np.float32, 20, 12, 128, 128, 3.0, 0.125,
                          "none", 2560, 768, 1e-12)
    if index == 2:
        lengths = variable_lengths(2, seed_base=seed_base)
        smax = int(lengths.max())
        return ConfigSpec(2, "variable-length-b32-len5to500-fp32", np.float32, 32, 12, smax, smax, 3.0, 0.125,
                          "key", 32 * smax, 768, 1e-12, lengths=lengths)
    if index == 3:
        return ConfigSpec(3, "long-row-s4096-h4096-fp32", np.float32, 1, 16, 4096, 4096, 5.0, 0.125, "none",
                          4096, 4096, 1e-12)
    if index == 4:
        return ConfigSpec(4, "gpt2-medium-b64-s512-fp16", np.float16, 64, 16, 512, 512, 3.0, 0.125, "causal",
                          32768, 1024, 1e-5)
    raise ValueError(f"no such config: {index}")


def packed_layout(lengths, H: int):
    """Row-packed batch: (cu_seqlens int32 [B+1], score_offsets int64 [B+1]); request b's [H, len_b, len_b] scores
    start at element score_offsets[b], score_offsets[B] is the total."""
    n = np.asarray(lengths, dtype=np.int64)
    cu = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
    off = np.concatenate([[0], np.cumsum(int(H) * n * n)]).astype(np.int64)
    return cu, off


def key_mask_from_lengths(lengths: np.ndarray, Sk: int, dtype) -> np.ndarray:
    """[B, Sk] additive key mask: 0 for k < len_b, MASK_VALUE beyond."""
    k = np.arange(Sk)[None, :]
    return np.where(k < np.asarray(lengths)[:, None], 0.0, MASK_VALUE).astype(dtype)


def causal_mask(Sq: int, Sk: int, dtype) -> np.ndarray:
    """[Sq, Sk] additive mask: MASK_VALUE strictly above the diagonal (k > q)."""
    q = np.arange(Sq)[:, None]
    k = np.arange(Sk)[None, :]
    return np.where(k > q, MASK_VALUE, 0.0).astype(dtype)


def softmax_case(spec: ConfigSpec, seed_base: int = SEED_BASE) -> SoftmaxCase:
    scores = _normal(_rng(spec.index, _T_SCORES, seed_base), (spec.B, spec.H, spec.Sq, spec.Sk),
                     0.0, spec.score_std, spec.dtype)
    if spec.mask_kind == "none":
        return SoftmaxCase(scores, None, 0, 0, spec.scale, "none")
    if spec.mask_kind == "key":
        mask = key_mask_from_lengths(spec.lengths, spec.Sk, spec.dtype)
        return SoftmaxCase(scores, mask, spec.Sk, 0, spec.scale, "key", lengths=spec.lengths)
    if spec.mask_kind == "causal":
        return SoftmaxCase(scores, causal_mask(spec.Sq, spec.Sk, spec.dtype), 0, spec.Sk, spec.scale, "causal")
    raise ValueError(spec.mask_kind)


def layernorm_case(spec: ConfigSpec, seed_base: int = SEED_BASE) -> LayerNormCase:
    i = spec.index
    shape = (spec.rows, spec.hidden)
    return LayerNormCase(
        x=_normal(_rng(i, _T_X, seed_base), shape, 0.0, 1.0, spec.dtype),
        residual=_normal(_rng(i, _T_RES, seed_base), shape, 0.0, 1.0, spec.dtype),
        bias=_normal(_rng(i, _T_BIAS, seed_base), (spec.hidden,), 0.0, 0.1, spec.dtype),
        gamma=_normal(_rng(i, _T_GAMMA, seed_base), (spec.hidden,), 1.0, 0.1, spec.dtype),
        beta=_normal(_rng(i, _T_BETA, seed_base), (spec.hidden,), 0.0, 0.1, spec.dtype),
        eps=spec.eps,
    )


def random_softmax_case(seed: int, B: int, H: int, Sq: int, Sk: int, dtype=np.float32, mask_kind: str = "none",
                        score_std: float = 3.0, scale: float = 0.125) -> SoftmaxCase:
    """Free-form case for shape sweeps (the Table 2 grid, ragged tails, ...)."""
    rng = np.random.Generator(np.random.Philox(seed))
    scores = _normal(rng, (B, H, Sq, Sk), 0.0, score_std, dtype)
    if mask_kind == "none":
        return SoftmaxCase(scores, None, 0, 0, scale, "none")
    if mask_kind == "key":
        lengths = rng.integers(1, Sk + 1, size=B, dtype=np.int64)
        return SoftmaxCase(scores, key_mask_from_lengths(lengths, Sk, dtype), Sk, 0, scale, "key", lengths=lengths)
    if mask_kind == "causal":
        return SoftmaxCase(scores, causal_mask(Sq, Sk, dtype), 0, Sk, scale, "causal")
    if mask_kind == "dense":
        keep = rng.random((B, Sq, Sk)) < 0.7
        keep[..., 0] = True  # every row keeps at least one key
        mask = np.where(keep, 0.0, MASK_VALUE).astype(dtype)
        return SoftmaxCase(scores, mask, Sq * Sk, Sk, scale, "dense")
    raise ValueError(mask_kind)


def random_layernorm_case(seed: int, rows: int, hidden: int, dtype=np.float32, eps: float = 1e-12) -> LayerNormCase:
    rng = np.random.Generator(np.random.Philox(seed))
    shape = (rows, hidden)
    return LayerNormCase(
        x=_normal(rng, shape, 0.0, 1.0, dtype),
        residual=_normal(rng, shape, 0.0, 1.0, dtype),
        bias=_normal(rng, (hidden,), 0.0, 0.1, dtype),
        gamma=_normal(rng, (hidden,), 1.0, 0.1, dtype),
        beta=_normal(rng, (hidden,), 0.0, 0.1, dtype),
        eps=eps,
    )
