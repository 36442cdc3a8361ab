"""ctypes binding of libturbo_reduce.so: argument marshalling only.

Every function has the name and the argument order of its C entry point
(include/turbo_reduce.h); tensors stand in for (pointer, sizes, dtype).  All
arithmetic happens in the HIP kernels.  There is no CPU fallback: if the
library has not been built, loading fails with an error that says how to
build it.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# TURBO_REDUCE_LIB selects another build of the same library (e.g. one compiled with different tuning macros).
LIB_PATH = os.environ.get("TURBO_REDUCE_LIB") or os.path.join(_HERE, "libturbo_reduce.so")

TURBO_OK, TURBO_ERR_NULL, TURBO_ERR_SHAPE, TURBO_ERR_DTYPE, TURBO_ERR_ALIGN, TURBO_ERR_LAUNCH = range(6)
TURBO_F32, TURBO_F16 = 0, 1
TURBO_OVR_PATH, TURBO_OVR_MAX_VEC_BYTES, TURBO_OVR_GRID_WAVES, TURBO_OVR_BLOCK_WAVES, TURBO_OVR_GRID_BLOCKS = 0, 1, 2, 3, 4
PATH_WAVE, PATH_BLOCK, PATH_STREAM = 0, 1, 2

EXPORTED_SYMBOLS = (
    "turbo_masked_softmax", "turbo_masked_softmax_ex", "turbo_masked_softmax_varlen", "turbo_masked_softmax_packed", "turbo_masked_softmax_causal", "turbo_add_bias_layernorm",
    "turbo_add_bias_layernorm_dt", "turbo_add_bias_layernorm_varlen",
    "turbo_add_bias_gelu", "turbo_add_bias_split_heads", "turbo_merge_heads",
    "turbo_batch_schedule", "turbo_mem_plan", "turbo_cost_table_fill",
    "turbo_status_string", "turbo_set_override", "turbo_describe_plan", "turbo_debug_fastdiv",
    "turbo_stream_probe",
)

_lib = None


class TurboError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib() -> ctypes.CDLL:
    """The loaded C library (raw entry points, for callers that hold device pointers themselves)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2010_05680_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i, ll, f = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong, ctypes.c_float
        L.turbo_masked_softmax.argtypes = [vp, vp, i, i, i, i, f, i, vp]
        L.turbo_masked_softmax_ex.argtypes = [vp, vp, ll, ll, i, i, i, i, f, i, vp]
        L.turbo_masked_softmax_varlen.argtypes = [vp, vp, vp, i, i, i, i, f, i, vp]
        L.turbo_masked_softmax_varlen.restype = i
        L.turbo_add_bias_layernorm.argtypes = [vp, vp, vp, vp, vp, i, i, f, vp, vp]
        L.turbo_add_bias_layernorm_dt.argtypes = [vp, vp, vp, vp, vp, i, i, f, vp, i, vp]
        L.turbo_add_bias_layernorm_varlen.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, f, vp, i, vp]
        L.turbo_add_bias_layernorm_varlen.restype = i
        L.turbo_add_bias_gelu.argtypes = [vp, vp, i, i, i, vp, i, vp]
        L.turbo_add_bias_split_heads.argtypes = [vp, vp, i, i, i, i, i, vp, i, vp]
        L.turbo_merge_heads.argtypes = [vp, i, i, i, i, vp, i, vp]
        for name in ("turbo_masked_softmax", "turbo_masked_softmax_ex", "turbo_add_bias_layernorm",
                     "turbo_add_bias_layernorm_dt", "turbo_add_bias_layernorm_varlen", "turbo_set_override", "turbo_describe_plan",
                     "turbo_add_bias_gelu", "turbo_add_bias_split_heads", "turbo_merge_heads"):
            getattr(L, name).restype = i
        L.turbo_status_string.argtypes = [i]
        L.turbo_status_string.restype = ctypes.c_char_p
        L.turbo_set_override.argtypes = [i, i]
        L.turbo_describe_plan.argtypes = [i, i, i, i, i, ctypes.c_char_p, i]
        L.turbo_debug_fastdiv.argtypes = [ctypes.c_uint, ctypes.c_uint]
        L.turbo_debug_fastdiv.restype = ctypes.c_uint
        L.turbo_stream_probe.argtypes = [vp, vp, vp, ctypes.c_longlong, vp]
        L.turbo_masked_softmax_packed.argtypes = [vp, vp, vp, i, i, i, i, f, i, vp]
        L.turbo_masked_softmax_packed.restype = i
        L.turbo_masked_softmax_causal.argtypes = L.turbo_masked_softmax_varlen.argtypes
        L.turbo_masked_softmax_causal.restype = i
        L.turbo_stream_probe.restype = i
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().turbo_status_string(int(status)).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return TURBO_F32
    if t.dtype == torch.float16:
        return TURBO_F16
    raise TypeError(f"unsupported dtype {t.dtype}: the library stores binary32 or binary16")


def _dev_ptr(t: Optional[torch.Tensor], name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def _check(status: int, where: str) -> None:
    if status != TURBO_OK:
        raise TurboError(status, where)


def turbo_masked_softmax(scores: torch.Tensor, mask: Optional[torch.Tensor], scale: float, stream=None) -> torch.Tensor:
    """In-place softmax_k(scale*scores + mask) on [B,H,Sq,Sk]; mask is dense [B,Sq,Sk] or None."""
    B, H, Sq, Sk = scores.shape
    _dtype_code(scores)
    if mask is not None:
        if mask.dtype != scores.dtype or tuple(mask.shape) != (B, Sq, Sk):
            raise ValueError("mask must be [B,Sq,Sk] in the scores' dtype")
    _check(lib().turbo_masked_softmax(_dev_ptr(scores, "scores"), _dev_ptr(mask, "mask"), B, H, Sq, Sk, float(scale),
                                      _dtype_code(scores), _stream_ptr(stream)), "turbo_masked_softmax")
    return scores


def turbo_masked_softmax_ex(scores: torch.Tensor, mask: Optional[torch.Tensor], mask_stride_b: int, mask_stride_q: int,
                            scale: float, stream=None) -> torch.Tensor:
    """In-place softmax with mask element (b,q,k) at mask[b*mask_stride_b + q*mask_stride_q + k]."""
    B, H, Sq, Sk = scores.shape
    _dtype_code(scores)
    if mask is not None:
        if mask.dtype != scores.dtype:
            raise ValueError("mask must have the scores' dtype")
        need = (B - 1) * mask_stride_b + (Sq - 1) * mask_stride_q + Sk
        if mask_stride_b >= 0 and mask_stride_q >= 0 and mask.numel() < need:
            raise ValueError("mask is smaller than its strides imply")
    _check(lib().turbo_masked_softmax_ex(_dev_ptr(scores, "scores"), _dev_ptr(mask, "mask"), int(mask_stride_b),
                                         int(mask_stride_q), B, H, Sq, Sk, float(scale), _dtype_code(scores),
                                         _stream_ptr(stream)), "turbo_masked_softmax_ex")
    return scores


def _lengths_ptr(t: Optional[torch.Tensor], B: int, name: str) -> Optional[int]:
    if t is None:
        return None
    if t.dtype != torch.int32 or tuple(t.shape) != (B,):
        raise ValueError(f"{name} must be an int32 tensor of shape [B]")
    return _dev_ptr(t, name)


def turbo_masked_softmax_varlen(scores: torch.Tensor, q_lengths: Optional[torch.Tensor], k_lengths: torch.Tensor,
                                scale: float, stream=None) -> torch.Tensor:
    """In-place length-aware softmax: keys beyond k_lengths[b] get weight 0 unread, rows beyond q_lengths[b] are skipped."""
    B, H, Sq, Sk = scores.shape
    dt = _dtype_code(scores)
    _check(lib().turbo_masked_softmax_varlen(_dev_ptr(scores, "scores"), _lengths_ptr(q_lengths, B, "q_lengths"),
                                             _lengths_ptr(k_lengths, B, "k_lengths"), B, H, Sq, Sk, float(scale), dt,
                                             _stream_ptr(stream)), "turbo_masked_softmax_varlen")
    return scores


def turbo_masked_softmax_causal(scores: torch.Tensor, q_lengths: Optional[torch.Tensor], k_lengths: Optional[torch.Tensor],
                                scale: float, stream=None) -> torch.Tensor:
    """In-place causal softmax: query q sees keys k <= q + (Sk - Sq), further limited by the optional lengths; the
    other keys get weight 0 unread."""
    B, H, Sq, Sk = scores.shape
    dt = _dtype_code(scores)
    _check(lib().turbo_masked_softmax_causal(_dev_ptr(scores, "scores"), _lengths_ptr(q_lengths, B, "q_lengths"),
                                             _lengths_ptr(k_lengths, B, "k_lengths"), B, H, Sq, Sk, float(scale), dt,
                                             _stream_ptr(stream)), "turbo_masked_softmax_causal")
    return scores


def _layernorm_args(x, residual, bias, gamma, beta, out):
    rows, hidden = x.shape
    _dtype_code(x)
    for name, t, shape in (("residual", residual, (rows, hidden)), ("out", out, (rows, hidden)),
                           ("bias", bias, (hidden,)), ("gamma", gamma, (hidden,)), ("beta", beta, (hidden,))):
        if t is not None and (tuple(t.shape) != shape or t.dtype != x.dtype):
            raise ValueError(f"{name} must be {shape} in x's dtype")
    return rows, hidden


def turbo_masked_softmax_packed(scores: torch.Tensor, cu_seqlens: torch.Tensor, score_offsets: torch.Tensor, H: int,
                                total_tokens: int, max_len: int, scale: float, stream=None) -> torch.Tensor:
    """In-place softmax over a row-packed batch: `scores` is flat, request b's [H, len_b, len_b] block starts at
    score_offsets[b]; cu_seqlens (int32 [B+1]) and score_offsets (int64 [B+1]) live on the device."""
    dt = _dtype_code(scores)
    if cu_seqlens.dtype != torch.int32 or score_offsets.dtype != torch.int64 or cu_seqlens.numel() != score_offsets.numel():
        raise ValueError("cu_seqlens must be int32 [B+1] and score_offsets int64 [B+1]")
    B = cu_seqlens.numel() - 1
    _check(lib().turbo_masked_softmax_packed(_dev_ptr(scores, "scores"), _dev_ptr(cu_seqlens, "cu_seqlens"),
                                             _dev_ptr(score_offsets, "score_offsets"), B, int(H), int(total_tokens),
                                             int(max_len), float(scale), dt, _stream_ptr(stream)),
           "turbo_masked_softmax_packed")
    return scores


def turbo_add_bias_layernorm(x, residual, bias, gamma, beta, eps: float, out: torch.Tensor, stream=None) -> torch.Tensor:
    """out = LayerNorm(x + bias + residual) * gamma + beta, binary32 tensors."""
    if x.dtype != torch.float32:
        raise TypeError("turbo_add_bias_layernorm is the binary32 entry point; use turbo_add_bias_layernorm_dt")
    rows, hidden = _layernorm_args(x, residual, bias, gamma, beta, out)
    _check(lib().turbo_add_bias_layernorm(_dev_ptr(x, "x"), _dev_ptr(residual, "residual"), _dev_ptr(bias, "bias"),
                                          _dev_ptr(gamma, "gamma"), _dev_ptr(beta, "beta"), rows, hidden, float(eps),
                                          _dev_ptr(out, "out"), _stream_ptr(stream)), "turbo_add_bias_layernorm")
    return out


def turbo_add_bias_layernorm_dt(x, residual, bias, gamma, beta, eps: float, out: torch.Tensor, stream=None) -> torch.Tensor:
    """The same with all tensors in x's dtype (binary32 or binary16 storage)."""
    rows, hidden = _layernorm_args(x, residual, bias, gamma, beta, out)
    _check(lib().turbo_add_bias_layernorm_dt(_dev_ptr(x, "x"), _dev_ptr(residual, "residual"), _dev_ptr(bias, "bias"),
                                             _dev_ptr(gamma, "gamma"), _dev_ptr(beta, "beta"), rows, hidden,
                                             float(eps), _dev_ptr(out, "out"), _dtype_code(x), _stream_ptr(stream)),
           "turbo_add_bias_layernorm_dt")
    return out


def turbo_add_bias_layernorm_varlen(x, residual, bias, gamma, beta, lengths: torch.Tensor, eps: float, out: torch.Tensor,
                                    stream=None) -> torch.Tensor:
    """x, residual, out [B,S,hidden]; token rows s >= lengths[b] are padding: neither read nor written."""
    B, S, hidden = x.shape
    _layernorm_args(x.view(B * S, hidden), None if residual is None else residual.view(B * S, hidden), bias, gamma, beta,
                    out.view(B * S, hidden))
    _check(lib().turbo_add_bias_layernorm_varlen(_dev_ptr(x, "x"), _dev_ptr(residual, "residual"), _dev_ptr(bias, "bias"),
                                                 _dev_ptr(gamma, "gamma"), _dev_ptr(beta, "beta"),
                                                 _lengths_ptr(lengths, B, "lengths"), B, S, hidden, float(eps),
                                                 _dev_ptr(out, "out"), _dtype_code(x), _stream_ptr(stream)),
           "turbo_add_bias_layernorm_varlen")
    return out


def turbo_add_bias_gelu(x: torch.Tensor, bias: Optional[torch.Tensor], approximate: bool, out: torch.Tensor,
                        stream=None) -> torch.Tensor:
    """out = gelu(x + bias) on [rows, hidden]; erf form, or the tanh form with approximate=True."""
    rows, hidden = x.shape
    dt = _dtype_code(x)
    if out.shape != x.shape or out.dtype != x.dtype or (bias is not None and (tuple(bias.shape) != (hidden,) or bias.dtype != x.dtype)):
        raise ValueError("out must match x; bias must be [hidden] in x's dtype")
    _check(lib().turbo_add_bias_gelu(_dev_ptr(x, "x"), _dev_ptr(bias, "bias"), rows, hidden, int(bool(approximate)),
                                     _dev_ptr(out, "out"), dt, _stream_ptr(stream)), "turbo_add_bias_gelu")
    return out


def turbo_add_bias_split_heads(x: torch.Tensor, bias: Optional[torch.Tensor], out: torch.Tensor, stream=None) -> torch.Tensor:
    """x [B,S,n_split,H,D] (+ bias [n_split,H,D]) -> out [n_split,B,H,S,D]."""
    B, S, K, H, D = x.shape
    dt = _dtype_code(x)
    if tuple(out.shape) != (K, B, H, S, D) or out.dtype != x.dtype:
        raise ValueError("out must be [n_split,B,H,S,D] in x's dtype")
    if bias is not None and (tuple(bias.shape) != (K, H, D) or bias.dtype != x.dtype):
        raise ValueError("bias must be [n_split,H,D] in x's dtype")
    _check(lib().turbo_add_bias_split_heads(_dev_ptr(x, "x"), _dev_ptr(bias, "bias"), B, S, K, H, D, _dev_ptr(out, "out"),
                                            dt, _stream_ptr(stream)), "turbo_add_bias_split_heads")
    return out


def turbo_merge_heads(x: torch.Tensor, out: torch.Tensor, stream=None) -> torch.Tensor:
    """x [B,H,S,D] -> out [B,S,H,D]."""
    B, H, S, D = x.shape
    dt = _dtype_code(x)
    if tuple(out.shape) != (B, S, H, D) or out.dtype != x.dtype:
        raise ValueError("out must be [B,S,H,D] in x's dtype")
    _check(lib().turbo_merge_heads(_dev_ptr(x, "x"), B, H, S, D, _dev_ptr(out, "out"), dt, _stream_ptr(stream)),
           "turbo_merge_heads")
    return out


def turbo_stream_probe(in0: torch.Tensor, in1: Optional[torch.Tensor], out: torch.Tensor, stream=None) -> torch.Tensor:
    """Measurement aid: out = in0 (+ in1) over the tensors' raw bytes taken as binary32 (same byte counts required)."""
    n_bytes = in0.numel() * in0.element_size()
    if out.numel() * out.element_size() != n_bytes or (in1 is not None and in1.numel() * in1.element_size() != n_bytes):
        raise ValueError("all buffers must hold the same number of bytes")
    _check(lib().turbo_stream_probe(_dev_ptr(in0, "in0"), _dev_ptr(in1, "in1"), _dev_ptr(out, "out"), n_bytes,
                                    _stream_ptr(stream)), "turbo_stream_probe")
    return out


def turbo_set_override(key: int, value: int) -> None:
    _check(lib().turbo_set_override(int(key), int(value)), "turbo_set_override")


def turbo_describe_plan(op: int, rows: int, row_len: int, dtype: int, aligned16: bool = True) -> str:
    buf = ctypes.create_string_buffer(128)
    _check(lib().turbo_describe_plan(int(op), int(rows), int(row_len), int(dtype), int(bool(aligned16)), buf, 128),
           "turbo_describe_plan")
    return buf.value.decode()
