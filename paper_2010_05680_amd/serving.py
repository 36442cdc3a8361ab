"""ctypes binding of the host-side planning routines (include/turbo_serving.h): marshalling only."""
from __future__ import annotations

import ctypes
from typing import List, Sequence, Tuple

import numpy as np

from . import binding as _b

_ready = False


def _lib():
    global _ready
    L = _b.lib()
    if not _ready:
        ip, dp, lp = ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_longlong)
        L.turbo_batch_schedule.argtypes = [ip, ctypes.c_int, dp, ctypes.c_int, ctypes.c_int, ip, ip, ip, dp]
        L.turbo_batch_schedule.restype = ctypes.c_int
        L.turbo_mem_plan.argtypes = [ip, ip, lp, ctypes.c_int, lp, ip, ctypes.c_int, ctypes.c_longlong, ctypes.c_double,
                                     ip, lp]
        L.turbo_mem_plan.restype = ctypes.c_int
        L.turbo_cost_table_fill.argtypes = [ip, ctypes.c_int, ip, ctypes.c_int, dp, ctypes.c_int, ctypes.c_int, dp]
        L.turbo_cost_table_fill.restype = ctypes.c_int
        _ready = True
    return L


def _ints(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def turbo_batch_schedule(lengths: Sequence[int], cached_cost: np.ndarray, max_batch: int) -> Tuple[List[List[int]], float]:
    """cached_cost: [max_len+1, max_batch+1] per-request costs.  Returns (batches of request indices, total cost)."""
    lens = _ints(lengths)
    table = np.ascontiguousarray(cached_cost, dtype=np.float64)
    max_len = table.shape[0] - 1
    if table.ndim != 2 or table.shape[1] != max_batch + 1:
        raise ValueError("cached_cost must be [max_len+1, max_batch+1]")
    n = len(lens)
    order = np.zeros(max(n, 1), np.int32)
    ends = np.zeros(max(n, 1), np.int32)
    nb = ctypes.c_int(0)
    total = ctypes.c_double(0.0)
    ip, dp = ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_double)
    st = _lib().turbo_batch_schedule(lens.ctypes.data_as(ip), n, table.ctypes.data_as(dp), max_len, max_batch,
                                     order.ctypes.data_as(ip), ends.ctypes.data_as(ip), ctypes.byref(nb),
                                     ctypes.byref(total))
    _b._check(st, "turbo_batch_schedule")
    batches, begin = [], 0
    for k in range(nb.value):
        batches.append([int(v) for v in order[begin:ends[k]]])
        begin = int(ends[k])
    return batches, total.value


def turbo_cost_table_fill(sample_len: Sequence[int], sample_batch: Sequence[int], sample_cost: np.ndarray, max_len: int,
                          max_batch: int) -> np.ndarray:
    """sample_cost [len(sample_len), len(sample_batch)] per-request costs -> dense table [max_len+1, max_batch+1]."""
    sl, sb = _ints(sample_len), _ints(sample_batch)
    sc = np.ascontiguousarray(sample_cost, dtype=np.float64)
    if sc.shape != (len(sl), len(sb)):
        raise ValueError("sample_cost must be [len(sample_len), len(sample_batch)]")
    table = np.zeros((max(max_len, 0) + 1, max(max_batch, 0) + 1), np.float64)
    ip, dp = ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_double)
    st = _lib().turbo_cost_table_fill(sl.ctypes.data_as(ip), len(sl), sb.ctypes.data_as(ip), len(sb), sc.ctypes.data_as(dp),
                                      int(max_len), int(max_batch), table.ctypes.data_as(dp))
    _b._check(st, "turbo_cost_table_fill")
    return table


def turbo_mem_plan(first_op, last_op, size, chunk_sizes: Sequence[int], default_chunk_size: int = 2 << 20,
                   k_scale: float = 1.2, max_chunks: int = 0):
    """Returns (assigned_chunk, assigned_offset, chunk sizes in use afterwards)."""
    f, l = _ints(first_op), _ints(last_op)
    s = np.ascontiguousarray(size, dtype=np.int64)
    n = len(s)
    cap = max_chunks or (len(chunk_sizes) + n + 1)
    chunks = np.zeros(cap, np.int64)
    chunks[:len(chunk_sizes)] = chunk_sizes
    nc = ctypes.c_int(len(chunk_sizes))
    ac = np.zeros(max(n, 1), np.int32)
    ao = np.zeros(max(n, 1), np.int64)
    ip, lp = ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_longlong)
    st = _lib().turbo_mem_plan(f.ctypes.data_as(ip), l.ctypes.data_as(ip), s.ctypes.data_as(lp), n,
                               chunks.ctypes.data_as(lp), ctypes.byref(nc), cap, int(default_chunk_size), float(k_scale),
                               ac.ctypes.data_as(ip), ao.ctypes.data_as(lp))
    _b._check(st, "turbo_mem_plan")
    return [int(v) for v in ac[:n]], [int(v) for v in ao[:n]], [int(v) for v in chunks[:nc.value]]
