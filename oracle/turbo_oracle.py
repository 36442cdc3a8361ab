"""ctypes front end of the double-precision CPU oracle (oracle/turbo_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module.

Inputs of any float dtype are widened exactly to float64 before the call, so
for fp16 I/O the oracle sees the fp16-rounded values and returns float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "turbo_oracle.c")
_LIB = os.path.join(_HERE, "libturbo_oracle.so")
_lib = None

_dp = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2, OpenMP for the row loop)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        override = os.environ.get("TURBO_ORACLE_LIB")  # tests that plant a mistake in a copy of the oracle use this
        if override:
            lib = ctypes.CDLL(override)
        else:
            build()
            lib = ctypes.CDLL(_LIB)
        lib.oracle_set_threads.argtypes = [ctypes.c_int]
        lib.oracle_get_threads.restype = ctypes.c_int
        lib.oracle_masked_softmax.argtypes = [_dp, _dp, ctypes.c_longlong, ctypes.c_longlong, ctypes.c_int,
                                              ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, _dp]
        lib.oracle_masked_softmax.restype = None
        lib.oracle_add_bias_layernorm.argtypes = [_dp, _dp, _dp, _dp, _dp, ctypes.c_longlong, ctypes.c_int,
                                                  ctypes.c_double, _dp]
        lib.oracle_add_bias_layernorm.restype = None
        for name in ("oracle_variance_two_pass", "oracle_variance_sum_of_squares", "oracle_variance_welford"):
            f = getattr(lib, name)
            f.argtypes = [_dp, ctypes.c_int]
            f.restype = ctypes.c_double
        lib.oracle_welford_merge.argtypes = [ctypes.c_double] * 6 + [_dp] * 3
        lib.oracle_welford_merge.restype = None
        _ip = ctypes.POINTER(ctypes.c_int)
        lib.oracle_masked_softmax_varlen.argtypes = [_dp, _ip, _ip, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                     ctypes.c_int, ctypes.c_double, _dp]
        lib.oracle_masked_softmax_varlen.restype = None
        lib.oracle_masked_softmax_causal.argtypes = [_dp, _ip, _ip, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                     ctypes.c_int, ctypes.c_double, _dp]
        lib.oracle_masked_softmax_causal.restype = None
        lib.oracle_masked_softmax_packed.argtypes = [_dp, _ip, ctypes.c_int, ctypes.c_int, ctypes.c_double, _dp]
        lib.oracle_masked_softmax_packed.restype = None
        lib.oracle_add_bias_layernorm_varlen.argtypes = [_dp, _dp, _dp, _dp, _dp, _ip, ctypes.c_int, ctypes.c_int,
                                                         ctypes.c_int, ctypes.c_double, _dp, _dp]
        lib.oracle_add_bias_layernorm_varlen.restype = None
        lib.oracle_add_bias_gelu.argtypes = [_dp, _dp, ctypes.c_longlong, ctypes.c_int, ctypes.c_int, _dp]
        lib.oracle_add_bias_gelu.restype = None
        lib.oracle_add_bias_split_heads.argtypes = [_dp, _dp] + [ctypes.c_int] * 5 + [_dp]
        lib.oracle_add_bias_split_heads.restype = None
        lib.oracle_merge_heads.argtypes = [_dp] + [ctypes.c_int] * 4 + [_dp]
        lib.oracle_merge_heads.restype = None
        _lib = lib
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_dp)


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def get_threads() -> int:
    return int(_load().oracle_get_threads())


def masked_softmax(scores, mask=None, mask_stride_b: int = 0, mask_stride_q: int = 0, scale: float = 1.0) -> np.ndarray:
    """softmax_k(scale * scores + mask) over the last axis of a [B,H,Sq,Sk] array; float64 result.

    `mask` (any shape, flattened) is addressed as mask[b*mask_stride_b + q*mask_stride_q + k].
    """
    s = _f64(scores)
    if s.ndim != 4:
        raise ValueError("scores must be [B,H,Sq,Sk]")
    B, H, Sq, Sk = s.shape
    m = None
    if mask is not None:
        m = _f64(mask).reshape(-1)
        need = (B - 1) * mask_stride_b + (Sq - 1) * mask_stride_q + Sk
        if m.size < need:
            raise ValueError("mask too small for the given strides")
    out = np.empty_like(s)
    if s.size:
        _load().oracle_masked_softmax(_ptr(s), _ptr(m), int(mask_stride_b), int(mask_stride_q), B, H, Sq, Sk,
                                      float(scale), _ptr(out))
    return out


def add_bias_layernorm(x, residual, bias, gamma, beta, eps: float) -> np.ndarray:
    """LayerNorm(x + bias + residual) * gamma + beta over the last axis of [rows, hidden]; float64 result."""
    xx = _f64(x)
    if xx.ndim != 2:
        raise ValueError("x must be [rows, hidden]")
    rows, hidden = xx.shape
    rr = None if residual is None else _f64(residual)
    bb = None if bias is None else _f64(bias)
    gg, be = _f64(gamma), _f64(beta)
    if rr is not None and rr.shape != xx.shape:
        raise ValueError("residual shape")
    for v in (bb, gg, be):
        if v is not None and v.shape != (hidden,):
            raise ValueError("parameter vector shape")
    out = np.empty_like(xx)
    if xx.size:
        _load().oracle_add_bias_layernorm(_ptr(xx), _ptr(rr), _ptr(bb), _ptr(gg), _ptr(be), rows, hidden,
                                          float(eps), _ptr(out))
    return out


def variance_two_pass(x) -> float:
    v = _f64(x).reshape(-1)
    return float(_load().oracle_variance_two_pass(_ptr(v), v.size))


def variance_sum_of_squares(x) -> float:
    v = _f64(x).reshape(-1)
    return float(_load().oracle_variance_sum_of_squares(_ptr(v), v.size))


def variance_welford(x) -> float:
    v = _f64(x).reshape(-1)
    return float(_load().oracle_variance_welford(_ptr(v), v.size))


def welford_merge(a, b):
    """Merge two (count, mean, M2) triples."""
    n, mean, m2 = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    _load().oracle_welford_merge(*(float(v) for v in a), *(float(v) for v in b), ctypes.byref(n),
                                 ctypes.byref(mean), ctypes.byref(m2))
    return n.value, mean.value, m2.value


def add_bias_gelu(x, bias, approximate: bool = False) -> np.ndarray:
    """gelu(x + bias) over [rows, hidden]; erf form by default, tanh form with approximate=True; float64 result."""
    xx = _f64(x)
    if xx.ndim != 2:
        raise ValueError("x must be [rows, hidden]")
    rows, hidden = xx.shape
    bb = None if bias is None else _f64(bias)
    if bb is not None and bb.shape != (hidden,):
        raise ValueError("bias shape")
    out = np.empty_like(xx)
    if xx.size:
        _load().oracle_add_bias_gelu(_ptr(xx), _ptr(bb), rows, hidden, int(bool(approximate)), _ptr(out))
    return out


def add_bias_split_heads(x, bias) -> np.ndarray:
    """[B,S,n_split,H,D] (+ bias [n_split,H,D]) -> [n_split,B,H,S,D]; float64 result."""
    xx = _f64(x)
    if xx.ndim != 5:
        raise ValueError("x must be [B,S,n_split,H,D]")
    B, S, K, H, D = xx.shape
    bb = None if bias is None else _f64(bias)
    if bb is not None and bb.shape != (K, H, D):
        raise ValueError("bias must be [n_split,H,D]")
    out = np.empty((K, B, H, S, D), dtype=np.float64)
    if xx.size:
        _load().oracle_add_bias_split_heads(_ptr(xx), _ptr(bb), B, S, K, H, D, _ptr(out))
    return out


def merge_heads(x) -> np.ndarray:
    """[B,H,S,D] -> [B,S,H,D]; float64 result."""
    xx = _f64(x)
    if xx.ndim != 4:
        raise ValueError("x must be [B,H,S,D]")
    B, H, S, D = xx.shape
    out = np.empty((B, S, H, D), dtype=np.float64)
    if xx.size:
        _load().oracle_merge_heads(_ptr(xx), B, H, S, D, _ptr(out))
    return out


def _i32(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def _iptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_int))


def masked_softmax_varlen(scores, q_lengths, k_lengths, scale: float = 1.0) -> np.ndarray:
    """Length-aware softmax on [B,H,Sq,Sk]: rows q < q_lengths[b] are normalised over their first k_lengths[b]
    keys (exact zeros after); every other row is returned unchanged.  q_lengths may be None (all rows)."""
    s = _f64(scores)
    B, H, Sq, Sk = s.shape
    kl = _i32(k_lengths)
    ql = None if q_lengths is None else _i32(q_lengths)
    if kl.shape != (B,) or (ql is not None and ql.shape != (B,)):
        raise ValueError("lengths must be [B]")
    out = np.empty_like(s)
    if s.size:
        _load().oracle_masked_softmax_varlen(_ptr(s), _iptr(ql), _iptr(kl), B, H, Sq, Sk, float(scale), _ptr(out))
    return out


def masked_softmax_causal(scores, q_lengths, k_lengths, scale: float = 1.0) -> np.ndarray:
    """Causal softmax on [B,H,Sq,Sk]: query q sees keys k <= q + (Sk - Sq), and k < k_lengths[b] if given; rows
    q >= q_lengths[b] (if given) and rows without a visible key are returned unchanged."""
    s = _f64(scores)
    B, H, Sq, Sk = s.shape
    kl = None if k_lengths is None else _i32(k_lengths)
    ql = None if q_lengths is None else _i32(q_lengths)
    if (kl is not None and kl.shape != (B,)) or (ql is not None and ql.shape != (B,)):
        raise ValueError("lengths must be [B]")
    out = np.empty_like(s)
    if s.size:
        _load().oracle_masked_softmax_causal(_ptr(s), _iptr(ql), _iptr(kl), B, H, Sq, Sk, float(scale), _ptr(out))
    return out


def masked_softmax_packed(scores, lengths, H: int, scale: float = 1.0) -> np.ndarray:
    """Row-packed batch: `scores` is the flat concatenation of the requests' [H, len_b, len_b] blocks (no padding);
    every row of len_b keys becomes softmax(scale * row).  Returns the flat result."""
    s = _f64(scores).reshape(-1)
    ln = _i32(lengths)
    if ln.ndim != 1 or (ln < 0).any() or int(H) * int((ln.astype(np.int64) ** 2).sum()) != s.size:
        raise ValueError("scores must hold H * sum(len^2) values")
    out = np.empty_like(s)
    if s.size:
        _load().oracle_masked_softmax_packed(_ptr(s), _iptr(ln), len(ln), int(H), float(scale), _ptr(out))
    return out


def add_bias_layernorm_varlen(x, residual, bias, gamma, beta, lengths, eps: float, out_before) -> np.ndarray:
    """Length-aware add-bias-LayerNorm on [B,S,hidden]: rows s < lengths[b] are computed, the rest keep out_before."""
    xx = _f64(x)
    B, S, hidden = xx.shape
    rr = None if residual is None else _f64(residual)
    bb = None if bias is None else _f64(bias)
    gg, be = _f64(gamma), _f64(beta)
    ob = _f64(out_before)
    ln = _i32(lengths)
    if ob.shape != xx.shape or ln.shape != (B,):
        raise ValueError("shape")
    out = np.empty_like(xx)
    _load().oracle_add_bias_layernorm_varlen(_ptr(xx), _ptr(rr), _ptr(bb), _ptr(gg), _ptr(be), _iptr(ln), B, S, hidden,
                                             float(eps), _ptr(ob), _ptr(out))
    return out
