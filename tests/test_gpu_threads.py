"""Concurrent host threads, each on its own stream, call the library at once.

The entry points keep no state beyond two per-device caches (compute-unit count, resident workgroups of the LayerNorm
block family) that are filled on first use; calls from several threads must neither corrupt them nor each other's
launches.  Every thread's results are compared with the oracle, element by element.
"""
import threading

import numpy as np
import pytest
import torch

from oracle import turbo_oracle as orc
from paper_2010_05680_amd import binding as tb

from conftest import assert_parity

pytestmark = pytest.mark.gpu

N_THREADS = 4
ROUNDS = 6

# (kind, shape): softmax [B,H,Sq,Sk] with a key mask / LayerNorm [rows, hidden]; one per kernel family and more
WORK = [
    ("softmax", (2, 3, 40, 77)), ("softmax", (1, 2, 9, 4096)), ("softmax", (1, 1, 3, 40000)), ("softmax", (2, 2, 64, 128)),
    ("layernorm", (70, 768)), ("layernorm", (33, 4096)), ("layernorm", (5, 40000)), ("layernorm", (64, 1001)),
]


def _inputs(kind, shape, dtype, seed):
    rng = np.random.default_rng(seed)
    if kind == "softmax":
        B, H, Sq, Sk = shape
        scores = (rng.standard_normal(shape) * 3).astype(dtype)
        mask = np.zeros((B, Sk), dtype=dtype)
        mask[:, Sk - Sk // 5:] = -10000
        return scores, mask
    rows, hidden = shape
    x, res = (rng.standard_normal(shape).astype(dtype) for _ in range(2))
    bias, beta = (0.1 * rng.standard_normal(hidden)).astype(dtype), (0.1 * rng.standard_normal(hidden)).astype(dtype)
    gamma = (1 + 0.1 * rng.standard_normal(hidden)).astype(dtype)
    return x, res, bias, gamma, beta


def _worker(tid, results, errors, barrier):
    try:
        torch.cuda.set_device(0)
        stream = torch.cuda.Stream()
        barrier.wait()  # all threads make their first call together
        with torch.cuda.stream(stream):
            for rnd in range(ROUNDS):
                for w, (kind, shape) in enumerate(WORK):
                    if (w + rnd) % N_THREADS != tid:
                        continue
                    dtype = np.float32 if (w + rnd) % 2 == 0 else np.float16
                    inp = _inputs(kind, shape, dtype, seed=1000 * rnd + w)
                    dev = [torch.from_numpy(a).cuda() for a in inp]
                    if kind == "softmax":
                        tb.turbo_masked_softmax_ex(dev[0], dev[1], shape[3], 0, 0.125, stream=stream)
                        got = dev[0]
                    else:
                        got = torch.full_like(dev[0], float("nan"))
                        tb.turbo_add_bias_layernorm_dt(dev[0], dev[1], dev[2], dev[3], dev[4], 1e-5, got, stream=stream)
                    stream.synchronize()
                    results.append((kind, shape, dtype, inp, got.cpu().numpy()))
    except Exception as exc:  # surfaced by the main thread
        errors.append((tid, repr(exc)))


def test_concurrent_callers_on_their_own_streams():
    results, errors = [], []
    barrier = threading.Barrier(N_THREADS)
    threads = [threading.Thread(target=_worker, args=(t, results, errors, barrier)) for t in range(N_THREADS)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=240)
    assert not any(t.is_alive() for t in threads), "a worker thread did not finish"
    assert not errors, errors
    assert len(results) == ROUNDS * len(WORK)
    for kind, shape, dtype, inp, got in results:
        if kind == "softmax":
            want = orc.masked_softmax(inp[0], inp[1], shape[3], 0, 0.125)
        else:
            want = orc.add_bias_layernorm(*inp, 1e-5)
        assert_parity(got, want, dtype, f"{kind} {shape} {np.dtype(dtype).name} from a worker thread")
