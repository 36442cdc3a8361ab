#!/usr/bin/env python3
"""Benchmark of the batch-reduction hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch: the in-place masked softmax over the
attention scores followed by the fused add-bias-LayerNorm, both launched through the C ABI on one
HIP stream.  The headline workload is the benchmark's configs[3] (rows of 4096 fp32 values), the largest
configuration that fits one GPU; configs[1] (BERT-base serving batch), the smallest timed one and the stated worst
case, is reported with every other configuration under "per_config".

Timing is "cold": every timing loop cycles through enough independent buffer sets (at least 640 MB of streamed
tensors in total, more than twice the 256 MB last-level cache) that every launch streams its operands from HBM.  Inputs are resident
in HBM before the timed region starts.  The metric is achieved HBM GB/s over the algorithmic bytes
(softmax 2*s*N + mask, LayerNorm 3*s*M + 3*s*hidden), reported against the 8 TB/s peak.

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per launch measured with rocprofv3 counters (FETCH_SIZE / WRITE_SIZE, each scaled by what the same
# counter reads for a plain copy of known size); written from the counter runs described beside it.
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "hbm_traffic_pmc_configs1-4.json")
COLD_BYTES = 640 << 20       # rotate over at least this many bytes of operands
MAX_SETS = 48                # config 1's softmax tensor is 15.7 MB: 41 sets reach COLD_BYTES


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, help="BASELINE.json config index of the headline workload")
    ap.add_argument("--seed", type=int, default=0, help="offset added to the seed of the device-side input generator")
    ap.add_argument("--dtype", choices=["config", "f32", "f16"], default="config",
                    help="storage type of the headline workload's tensors (default: the configuration's own)")
    ap.add_argument("--per-config", type=int, default=1, help="also time every config's two kernels (0/1)")
    ap.add_argument("--cpu-baseline", type=int, default=1, help="time the CPU oracle on a bounded sample (0/1)")
    ap.add_argument("--launch", choices=["auto", "graph", "eager"], default="auto",
                    help="graph replay, eager stream launches, or (auto) graph for microsecond kernels and the faster "
                         "of the two for kernels long enough to hide the host's launch cost")
    ap.add_argument("--kernel-iters", type=int, default=100, help="launches per kernel timing loop")
    ap.add_argument("--traffic-probe", type=int, default=0,
                    help="run only: one plain copy of a known size, then N cold launches of each kernel of --config and "
                         "of the plain streams over the same buffers; meant to run under `rocprofv3 --pmc <counters>`")
    ap.add_argument("--probe-warm", type=int, default=0, help="with --traffic-probe: 1 = reuse one buffer set (cache-resident)")
    return ap.parse_args()


class KernelSets:
    """Independent operand sets for one config, generated on the device from a fixed seed."""

    def __init__(self, spec, torch, tb, wl, max_sets=MAX_SETS, cold_bytes=COLD_BYTES, seed=0):
        self.spec, self.torch, self.tb = spec, torch, tb
        tdt = torch.float32 if spec.dtype == np.float32 else torch.float16
        es = 4 if spec.dtype == np.float32 else 2
        self.es = es
        gen = torch.Generator(device="cuda")
        gen.manual_seed(wl.SEED_BASE + 1000 * spec.index + seed)
        n_sm = spec.B * spec.H * spec.Sq * spec.Sk
        n_ln = spec.rows * spec.hidden
        # masks (shared by all sets: they are read-only and tiny)
        self.mask, self.msb, self.msq = None, 0, 0
        if spec.mask_kind == "key":
            self.mask = torch.from_numpy(wl.key_mask_from_lengths(spec.lengths, spec.Sk, spec.dtype)).cuda()
            self.msb, self.msq = spec.Sk, 0
        elif spec.mask_kind == "causal":
            self.mask = torch.from_numpy(wl.causal_mask(spec.Sq, spec.Sk, spec.dtype)).cuda()
            self.msb, self.msq = 0, spec.Sk
        mask_bytes = 0 if self.mask is None else self.mask.numel() * es
        self.softmax_bytes = 2 * es * n_sm + mask_bytes
        self.layernorm_bytes = 3 * es * n_ln + 3 * es * spec.hidden
        self.softmax_rows = spec.B * spec.H * spec.Sq

        def n_sets(per_set):
            return int(max(2, min(max_sets, -(-cold_bytes // per_set))))

        self.n_sm_sets = n_sets(es * n_sm)
        self.n_ln_sets = n_sets(3 * es * n_ln)
        self.scores = []
        for _ in range(self.n_sm_sets):
            t = torch.randn((spec.B, spec.H, spec.Sq, spec.Sk), generator=gen, device="cuda", dtype=torch.float32)
            self.scores.append((t * spec.score_std).to(tdt))
        self.x, self.res, self.out = [], [], []
        for _ in range(self.n_ln_sets):
            self.x.append(torch.randn((spec.rows, spec.hidden), generator=gen, device="cuda", dtype=torch.float32).to(tdt))
            self.res.append(torch.randn((spec.rows, spec.hidden), generator=gen, device="cuda", dtype=torch.float32).to(tdt))
            self.out.append(torch.empty((spec.rows, spec.hidden), device="cuda", dtype=tdt))
        p = lambda mean, std: (torch.randn((spec.hidden,), generator=gen, device="cuda") * std + mean).to(tdt)
        self.bias, self.gamma, self.beta = p(0, 0.1), p(1, 0.1), p(0, 0.1)

    def softmax(self, i, stream):
        self.tb.turbo_masked_softmax_ex(self.scores[i % self.n_sm_sets], self.mask, self.msb, self.msq, self.spec.scale,
                                        stream=stream)

    def layernorm(self, i, stream):
        j = i % self.n_ln_sets
        self.tb.turbo_add_bias_layernorm_dt(self.x[j], self.res[j], self.bias, self.gamma, self.beta, self.spec.eps,
                                            self.out[j], stream=stream)

    def step(self, i, stream):
        self.softmax(i, stream)
        self.layernorm(i, stream)


AUTO_EAGER_FROM_MS = 0.015  # kernels at least this long hide the host's cost of an eager launch
HEADLINE_REPS = 5  # repetitions of the K-step headline measurement; the median one is reported
TIMING_LOOPS = 3  # every figure is the MEDIAN of this many timing loops (each loop averages all its launches)


class Timing:
    """ms: median over the timing loops of the per-launch average; ms_min: the fastest loop; n: launches per loop."""

    def __init__(self, loops_ms, n, mode):
        self.loops_ms = sorted(loops_ms)
        self.ms = float(np.median(self.loops_ms))
        self.ms_min = self.loops_ms[0]
        self.n, self.mode = n, mode


def time_launches(torch, stream, fn, iters, period, launch):
    """Per-launch duration of fn(i) over `iters` launches on `stream`, by HIP events on that stream.

    With launch == "graph", `period` consecutive launches (one full rotation over the buffer sets) are
    captured into a HIP graph that is replayed; this removes host launch cost from kernels that run
    for a few microseconds.  Kernels of tens of microseconds hide that cost by themselves, and a graph's
    kernel nodes then cost more per launch than plain stream launches (about 1.5 us each, measured; the
    profiler's per-dispatch durations agree with the eager figure), so "auto" times such kernels both
    ways and keeps the mode whose median is lower.  Returns a Timing."""
    if launch == "auto":
        best = _time_launches(torch, stream, fn, iters, period, "graph")
        if best.ms >= AUTO_EAGER_FROM_MS:
            eager = _time_launches(torch, stream, fn, iters, period, "eager")
            best = min(best, eager, key=lambda r: r.ms)
        return best
    return _time_launches(torch, stream, fn, iters, period, launch)


def time_ms(*args):
    return time_launches(*args).ms


def _time_launches(torch, stream, fn, iters, period, launch):
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(stream):
        for i in range(max(3, min(period, 10))):
            fn(i)
        stream.synchronize()
        mode = "eager"
        graph = None
        if launch == "graph":
            try:
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=stream):
                    for i in range(period):
                        fn(i)
                mode = "graph"
            except Exception as exc:  # capture not possible: fall back to eager launches, say so
                print(f"[bench] graph capture failed ({exc!r}); eager launches", file=sys.stderr)
                graph = None
        loops = []
        for _ in range(TIMING_LOOPS):
            if graph is not None:
                reps = max(1, -(-iters // period))
                graph.replay()
                stream.synchronize()
                start.record(stream)
                for _ in range(reps):
                    graph.replay()
                stop.record(stream)
                stream.synchronize()
                n = reps * period
            else:
                start.record(stream)
                for i in range(iters):
                    fn(i)
                stop.record(stream)
                stream.synchronize()
                n = iters
            loops.append(start.elapsed_time(stop) / n)
    return Timing(loops, n, mode)


COPY_PROBE_BYTES = 256 << 20


def traffic_probe(torch, tb, ks, stream, n, warm):
    """Calibration copy, then n launches each of: the softmax, the LayerNorm, and the plain streams of the same bytes
    and buffers (in-place copy, two-input add); eager, on one stream, for rocprofv3 counter runs.

    The copy is torch's elementwise copy kernel over COPY_PROBE_BYTES (reads that many bytes, writes that
    many): the ratio counter/known-bytes it yields scales the byte counters of the other kernels.  With `warm`
    every launch uses buffer set 0 (what a cache-resident tensor costs); otherwise the sets rotate (cold)."""
    src = torch.randn(COPY_PROBE_BYTES // 4, device="cuda")
    dst = torch.empty_like(src)
    pick = (lambda i: 0) if warm else (lambda i: i)
    with torch.cuda.stream(stream):
        for _ in range(3):
            dst.copy_(src)
        for i in range(n):
            ks.softmax(pick(i), stream)
        for i in range(n):
            ks.layernorm(pick(i), stream)
        for i in range(n):
            t = ks.scores[pick(i) % ks.n_sm_sets]
            tb.turbo_stream_probe(t, None, t, stream=stream)
        for i in range(n):
            j = pick(i) % ks.n_ln_sets
            tb.turbo_stream_probe(ks.x[j], ks.res[j], ks.out[j], stream=stream)
        stream.synchronize()
    print(json.dumps({"traffic_probe": True, "copy_bytes_each_way": COPY_PROBE_BYTES, "regime": "warm" if warm else "cold",
                      "softmax_bytes": ks.softmax_bytes, "layernorm_bytes": ks.layernorm_bytes, "launches": n,
                      "order": ["3 x calibration copy", "softmax", "layernorm", "stream_probe in place (softmax's bytes)",
                                "stream_probe two inputs (LayerNorm's tensors)"]}))


def elementwise_table(torch, tb, stream, launch, iters):
    """Cold timings of the element-wise fused kernels on the shapes that go with configs 1 and 4:
    feed-forward activation [B*S, 4*hidden], Q/K/V head split [B,S,3,H,64] and head merge [B,H,S,64]."""
    rows = []
    for label, tdt, es, B, S, H, D in (("config 1 model (BERT-base, f32)", torch.float32, 4, 20, 128, 12, 64),
                                       ("config 4 model (GPT-2-medium, f16)", torch.float16, 2, 64, 512, 16, 64)):
        hidden = H * D
        gen = torch.Generator(device="cuda")
        gen.manual_seed(20100568 + es)

        def sets(shape, per_set_bytes):
            n = int(max(2, min(MAX_SETS, -(-COLD_BYTES // per_set_bytes))))
            return [torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).to(tdt) for _ in range(n)], n

        entry = {"model": label}
        # bias + GELU on [B*S, 4*hidden]
        n_el = B * S * 4 * hidden
        xs, n = sets((B * S, 4 * hidden), 2 * es * n_el)
        outs = [torch.empty_like(x) for x in xs]
        bias = torch.randn((4 * hidden,), generator=gen, device="cuda").to(tdt)
        for approx, name in ((False, "add_bias_gelu_erf"), (True, "add_bias_gelu_tanh")):
            ms = time_ms(torch, stream, lambda i: tb.turbo_add_bias_gelu(xs[i % n], bias, approx, outs[i % n],
                                                                                  stream=stream), iters, n, launch)
            nbytes = 2 * es * n_el + es * 4 * hidden
            entry[name] = {"shape": [B * S, 4 * hidden], "bytes": nbytes, "cold_us": round(ms * 1e3, 2),
                           "cold_GBs": round(nbytes / ms / 1e6, 1), "cold_frac_of_8TBs": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)}
        del xs, outs
        # Q/K/V head split with bias, then head merge
        n_el = B * S * 3 * hidden
        xs, n = sets((B, S, 3, H, D), 2 * es * n_el)
        outs = [torch.empty((3, B, H, S, D), device="cuda", dtype=tdt) for _ in xs]
        b3 = torch.randn((3, H, D), generator=gen, device="cuda").to(tdt)
        ms = time_ms(torch, stream, lambda i: tb.turbo_add_bias_split_heads(xs[i % n], b3, outs[i % n],
                                                                                     stream=stream), iters, n, launch)
        nbytes = 2 * es * n_el + es * 3 * hidden
        entry["add_bias_split_heads"] = {"shape": [B, S, 3, H, D], "bytes": nbytes, "cold_us": round(ms * 1e3, 2),
                                         "cold_GBs": round(nbytes / ms / 1e6, 1),
                                         "cold_frac_of_8TBs": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)}
        ys = [o[0] for o in outs]  # [B,H,S,D], contiguous
        ms_out = [torch.empty((B, S, H, D), device="cuda", dtype=tdt) for _ in ys]
        ms = time_ms(torch, stream, lambda i: tb.turbo_merge_heads(ys[i % n], ms_out[i % n], stream=stream),
                                 iters, n, launch)
        nbytes = 2 * es * B * S * hidden
        entry["merge_heads"] = {"shape": [B, H, S, D], "bytes": nbytes, "cold_us": round(ms * 1e3, 2),
                                "cold_GBs": round(nbytes / ms / 1e6, 1),
                                "cold_frac_of_8TBs": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)}
        del xs, outs, ys, ms_out
        torch.cuda.empty_cache()
        rows.append(entry)
    return rows


def varlen_table(torch, tb, wl, stream, launch, iters):
    """Config 2 (zero-padded variable-length batch) through the length-aware entry points: the same tensors, but
    padding is neither read nor written.  Bytes are the ones actually moved: per head, a request of length n reads
    n*n scores and writes n*Smax; LayerNorm touches n of the Smax token rows."""
    spec = wl.config_spec(2)
    ks = KernelSets(spec, torch, tb, wl)
    lens = torch.from_numpy(spec.lengths.astype(np.int32)).cuda()
    B, S, H, hid, es = spec.B, spec.Sk, spec.H, spec.hidden, 4
    sm_bytes = int(sum(es * H * (n * n + n * S) for n in spec.lengths)) + 4 * B
    ln_bytes = int(sum(3 * es * n * hid for n in spec.lengths)) + 3 * es * hid + 4 * B
    view = lambda t: t.view(B, S, hid)
    rows = {}
    for name, fn, per, nbytes, padded_bytes in (
            ("softmax", lambda i: tb.turbo_masked_softmax_varlen(ks.scores[i % ks.n_sm_sets], lens, lens, spec.scale,
                                                                stream=stream), ks.n_sm_sets, sm_bytes, ks.softmax_bytes),
            ("layernorm", lambda i: tb.turbo_add_bias_layernorm_varlen(
                view(ks.x[i % ks.n_ln_sets]), view(ks.res[i % ks.n_ln_sets]), ks.bias, ks.gamma, ks.beta, lens, spec.eps,
                view(ks.out[i % ks.n_ln_sets]), stream=stream), ks.n_ln_sets, ln_bytes, ks.layernorm_bytes)):
        ms = time_ms(torch, stream, fn, iters, per, launch)
        rows[name] = {"cold_us": round(ms * 1e3, 2), "bytes_moved": nbytes, "GBs_of_bytes_moved": round(nbytes / ms / 1e6, 1),
                      "padded_bytes": padded_bytes, "real_fraction_of_padded_bytes": round(nbytes / padded_bytes, 3)}
    # the same requests with no padding in memory at all (row-packed): softmax blocks [H, n, n] one after the other,
    # LayerNorm over the [sum n, hidden] token rows with the ordinary entry point
    cu, off = wl.packed_layout(spec.lengths, H)
    total_tokens, n_scores = int(cu[-1]), int(off[-1])
    n_sets = int(max(2, min(MAX_SETS, -(-COLD_BYTES // (es * n_scores)))))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(wl.SEED_BASE + 2002)
    packed = [torch.randn(n_scores, generator=gen, device="cuda") * spec.score_std for _ in range(n_sets)]
    cu_d, off_d = torch.from_numpy(cu).cuda(), torch.from_numpy(off).cuda()
    max_len = int(spec.lengths.max())
    ms = time_ms(torch, stream, lambda i: tb.turbo_masked_softmax_packed(
        packed[i % n_sets], cu_d, off_d, H, total_tokens, max_len, spec.scale, stream=stream), iters, n_sets, launch)
    nbytes = 2 * es * n_scores + 12 * (B + 1)
    rows["softmax_packed"] = {"cold_us": round(ms * 1e3, 2), "bytes_moved": nbytes, "GBs_of_bytes_moved": round(nbytes / ms / 1e6, 1)}
    del packed
    n_sets = int(max(2, min(MAX_SETS, -(-COLD_BYTES // (3 * es * total_tokens * hid)))))
    xs, rs = ([torch.randn((total_tokens, hid), generator=gen, device="cuda") for _ in range(n_sets)] for _ in range(2))
    outs = [torch.empty_like(x) for x in xs]
    ms = time_ms(torch, stream, lambda i: tb.turbo_add_bias_layernorm_dt(
        xs[i % n_sets], rs[i % n_sets], ks.bias, ks.gamma, ks.beta, spec.eps, outs[i % n_sets], stream=stream), iters, n_sets, launch)
    nbytes = 3 * es * total_tokens * hid + 3 * es * hid
    rows["layernorm_packed"] = {"cold_us": round(ms * 1e3, 2), "bytes_moved": nbytes, "GBs_of_bytes_moved": round(nbytes / ms / 1e6, 1)}
    rows["lengths"] = [int(v) for v in spec.lengths]
    del ks, xs, rs, outs
    torch.cuda.empty_cache()
    # config 4 (GPT-2-medium, fp16) through the causal entry point: no mask tensor, keys above the diagonal unread
    spec4 = wl.config_spec(4)
    k4 = KernelSets(spec4, torch, tb, wl)
    ms = time_ms(torch, stream, lambda i: tb.turbo_masked_softmax_causal(k4.scores[i % k4.n_sm_sets], None, None,
                                                                                  spec4.scale, stream=stream),
                             iters, k4.n_sm_sets, launch)
    n_rows, Sq, Sk = spec4.B * spec4.H * spec4.Sq, spec4.Sq, spec4.Sk
    read_elems = spec4.B * spec4.H * sum(min(Sk, -(-(q + 1 + Sk - Sq) // 8) * 8) for q in range(Sq))  # whole 16-byte vectors
    nbytes = 2 * (read_elems + n_rows * Sk)
    rows["causal_config4"] = {"cold_us": round(ms * 1e3, 2), "bytes_moved": nbytes, "GBs_of_bytes_moved": round(nbytes / ms / 1e6, 1),
                              "additive_mask_bytes": k4.softmax_bytes}
    return rows


def scheduler_table(torch, tb, wl, stream, launch, iters):
    """The DP batch scheduler (Algorithm 2) fed with this build's own kernel times.

    The step (softmax [b,12,L,L] with a key mask + add-bias-LayerNorm [b*L,768], fp32, cold) is timed on a grid of
    lengths and batch sizes; turbo_cost_table_fill interpolates the per-request cost table; turbo_batch_schedule
    splits config 2's 32 requests; each batch of the schedule is then timed at its own padded shape.  The cost is
    that of the two kernels only (no GEMMs), so the schedule says what padding costs these kernels, nothing more."""
    from paper_2010_05680_amd import serving as sv
    base = wl.config_spec(2)
    lengths = [int(v) for v in base.lengths]

    def step_ms(b, L):
        spec = wl.ConfigSpec(2, f"b{b}-len{L}", np.float32, b, base.H, L, L, base.score_std, base.scale, "key",
                             b * L, base.hidden, base.eps, lengths=np.full(b, L, dtype=np.int64))
        k = KernelSets(spec, torch, tb, wl, max_sets=8)
        ms = time_ms(torch, stream, lambda i: k.step(i, stream), iters, max(k.n_sm_sets, k.n_ln_sets), launch)
        del k
        return ms

    sample_len, sample_batch = [16, 64, 128, 256, 384, 500], [1, 2, 4, 8, 16, 32]
    per_request = np.array([[step_ms(b, L) / b for b in sample_batch] for L in sample_len])
    torch.cuda.empty_cache()
    table = sv.turbo_cost_table_fill(sample_len, sample_batch, per_request, 500, 32)
    batches, predicted = sv.turbo_batch_schedule(lengths, table, 32)
    shapes = [(len(b), max(lengths[i] for i in b)) for b in batches]
    measured = sum(step_ms(b, L) for b, L in shapes)
    padded = step_ms(len(lengths), max(lengths))
    torch.cuda.empty_cache()
    return {
        "sampled_lengths": sample_len, "sampled_batch_sizes": sample_batch,
        "per_request_us": [[round(v * 1e3, 3) for v in row] for row in per_request],
        "schedule": [{"requests": b, "padded_to": L} for b, L in shapes],
        "predicted_us": round(predicted * 1e3, 2), "measured_us": round(measured * 1e3, 2),
        "one_padded_batch_us": round(padded * 1e3, 2),
        "one_request_at_a_time_predicted_us": round(sum(table[n, 1] for n in lengths) * 1e3, 2),
    }


def cpu_baseline(spec, wl, torch, tb, budget_s=16.0):
    """The oracle as it stands, on a bounded sample of the headline workload, on the host cores of this machine; the HIP
    path runs on the same sample and its largest deviation from the oracle is reported beside the timing."""
    from oracle import turbo_oracle as orc
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    cores = max(1, min(16, cores))
    # bound the sample: about 16M elements of each tensor (whole rows, from the start of the tensor)
    n_rows_sm = spec.B * spec.H * spec.Sq
    take_sm = min(n_rows_sm, max(1, (16 << 20) // spec.Sk))
    take_ln = min(spec.rows, max(1, (16 << 20) // spec.hidden))
    whole_sm, whole_ln = take_sm == n_rows_sm, take_ln == spec.rows
    # the sample is drawn with the workload's distributions at the sample's own shape (the tensors of the full
    # workload are gigabytes on the host); rows are independent, so a sample of rows is the same work per row
    sample = wl.ConfigSpec(spec.index, spec.name + "-sample", spec.dtype, 1, 1, take_sm, spec.Sk, spec.score_std, spec.scale,
                           "none", take_ln, spec.hidden, spec.eps)
    sc, lc = wl.softmax_case(sample), wl.layernorm_case(sample)
    s64 = sc.scores.astype(np.float64)
    x, r = lc.x.astype(np.float64), lc.residual.astype(np.float64)
    b, g, be = (v.astype(np.float64) for v in (lc.bias, lc.gamma, lc.beta))
    es = sc.scores.dtype.itemsize
    bytes_per_pass = 2 * es * take_sm * spec.Sk + 3 * es * take_ln * spec.hidden

    def one_pass():
        return orc.masked_softmax(s64, None, 0, 0, sc.scale), orc.add_bias_layernorm(x, r, b, g, be, lc.eps)

    out = {}
    for label, threads in (("all", cores), ("one", 1)):
        orc.set_threads(threads)
        want = one_pass()
        t0 = time.perf_counter()
        n = 0
        while True:
            one_pass()
            n += 1
            if time.perf_counter() - t0 > budget_s / 2:
                break
        dt = time.perf_counter() - t0
        out[label] = bytes_per_pass * n / dt / 1e9
    orc.set_threads(1)

    # the HIP path on the same sample, against the oracle's output
    s_dev = torch.from_numpy(sc.scores).cuda()
    tb.turbo_masked_softmax_ex(s_dev, None, 0, 0, sc.scale)
    o_dev = torch.empty((take_ln, spec.hidden), device="cuda", dtype=s_dev.dtype)
    tb.turbo_add_bias_layernorm_dt(*(torch.from_numpy(v).cuda() for v in (lc.x, lc.residual, lc.bias, lc.gamma, lc.beta)),
                                   lc.eps, o_dev)
    torch.cuda.synchronize()
    errs = {}
    for name, got, ref in (("softmax", s_dev.cpu().numpy().astype(np.float64), want[0]),
                           ("layernorm", o_dev.cpu().numpy().astype(np.float64), want[1])):
        err = np.abs(got - ref)
        big = np.abs(ref) >= 0.1  # where the relative error is the meaningful one
        errs[name] = {"max_abs_err": float(err.max()),
                      "max_rel_err_where_ref_ge_0.1": float((err[big] / np.abs(ref[big])).max()) if big.any() else None}
    return {
        "value": round(out["all"], 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
        "sample": (f"{'all' if whole_sm else 'the first'} {take_sm} of {n_rows_sm} softmax rows x {spec.Sk} and "
                   f"{'all' if whole_ln else 'the first'} {take_ln} of {spec.rows} LayerNorm rows x {spec.hidden} of the "
                   f"headline workload's shape and distributions, fp64 oracle incl. its output writes, repeated for "
                   f"{budget_s / 2:.0f} s per thread count; bytes counted as for the GPU (storage type); mask omitted"),
        "one_core_value": round(out["one"], 3),
        "hip_path_vs_oracle_on_the_sample": errs,
    }


def roofline_entry(name, nbytes, t, period, traffic):
    achieved = nbytes / (t.ms * 1e-3) / 1e9
    entry = {
        "bound": "hbm", "kernel": name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
        "algorithmic_bytes_per_launch": nbytes, "avg_launch_us": round(t.ms * 1e3, 3),
        "fastest_loop_us": round(t.ms_min * 1e3, 3), "launches": t.n,
        "timing": f"one HIP event pair around {t.n} back-to-back {t.mode} launches on the launch stream, median of "
                  f"{TIMING_LOOPS} such loops, cold (rotating {period} buffer sets)",
    }
    if traffic and traffic.get("algorithmic_bytes") == nbytes:
        entry["traffic"] = traffic["traffic_bytes"]
        entry["traffic_measured_in_this_run"] = False
        entry["traffic_source"] = ("rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script (--traffic-probe), "
                                   "summarised in profiles/; not re-measured by this run")
    return entry


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; rows are independent, so the path would shard by rows "
              "with no communication, but no multi-GPU figure is produced. Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2010_05680_amd import binding as tb
    from paper_2010_05680_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    tb.lib()  # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()

    spec = wl.config_spec(args.config)
    if args.dtype != "config":
        import dataclasses
        spec = dataclasses.replace(spec, dtype=np.float32 if args.dtype == "f32" else np.float16)
    ks = KernelSets(spec, torch, tb, wl, seed=args.seed)
    if args.traffic_probe:
        traffic_probe(torch, tb, ks, stream, args.traffic_probe, args.probe_warm)
        return
    period = max(ks.n_sm_sets, ks.n_ln_sets)
    step_bytes = ks.softmax_bytes + ks.layernorm_bytes

    # ---- headline: exactly K whole steps per repetition, wall clock bracketed by synchronisation ----
    steps = args.steps
    with torch.cuda.stream(stream):
        graph, graph_rem, mode = None, None, "eager"
        for i in range(args.warmup):
            ks.step(i, stream)
        stream.synchronize()
        reps, rem = divmod(steps, period)
        # auto: a step of >= 100 MB runs for tens of microseconds and hides the host's launch cost; below that, graph
        headline_launch = args.launch if args.launch != "auto" else ("eager" if step_bytes >= (100 << 20) else "graph")
        if headline_launch == "graph":
            try:  # one graph holds a full rotation over the buffer sets; a second one the remainder of K
                if reps:
                    graph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(graph, stream=stream):
                        for i in range(period):
                            ks.step(i, stream)
                if rem:
                    graph_rem = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(graph_rem, stream=stream):
                        for i in range(rem):
                            ks.step(i, stream)
                mode = "graph"
                for g in (graph, graph_rem):
                    if g is not None:
                        g.replay()
                stream.synchronize()
            except Exception as exc:
                print(f"[bench] graph capture failed ({exc!r}); eager launches", file=sys.stderr)
                graph, graph_rem, mode = None, None, "eager"

        def k_steps():
            """Exactly K steps: wall clock between two device synchronisations, and a HIP event pair on the stream."""
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ev0.record(stream)
            if mode == "graph":
                for _ in range(reps):
                    graph.replay()
                if graph_rem is not None:
                    graph_rem.replay()
            else:
                for i in range(steps):
                    ks.step(i, stream)
            ev1.record(stream)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / steps, ev0.elapsed_time(ev1) / steps

        # a K of 20 is a few milliseconds of work: the K steps are timed HEADLINE_REPS times and the median
        # repetition is reported, so one slow host wake-up cannot decide the figure
        runs = sorted(k_steps() for _ in range(HEADLINE_REPS))
    ms_per_step, ms_per_step_events = runs[len(runs) // 2]
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- both kernels of the headline workload: live HIP-event timing on the launch stream ----
    traffic = {}
    try:
        with open(TRAFFIC_JSON) as fh:
            traffic = json.load(fh)
    except (OSError, ValueError):
        pass
    t_sm = time_launches(torch, stream, lambda i: ks.softmax(i, stream), args.kernel_iters * 2, ks.n_sm_sets, args.launch)
    t_ln = time_launches(torch, stream, lambda i: ks.layernorm(i, stream), args.kernel_iters * 2, ks.n_ln_sets, args.launch)
    roof = {"softmax": roofline_entry("softmax", ks.softmax_bytes, t_sm, ks.n_sm_sets, traffic.get(f"cfg{spec.index}_softmax")),
            "layernorm": roofline_entry("layernorm", ks.layernorm_bytes, t_ln, ks.n_ln_sets,
                                        traffic.get(f"cfg{spec.index}_layernorm"))}
    dom = "softmax" if ks.softmax_bytes >= ks.layernorm_bytes else "layernorm"
    other = "layernorm" if dom == "softmax" else "softmax"

    # ---- every config, both kernels, cold and warm, beside the plain stream of the same bytes ----
    per_config = []
    empty_launch_us = None
    if args.per_config:
        # a launch that moves 16 bytes: what one dispatch costs when launches run back to back
        tiny = torch.zeros(4, device="cuda")
        t_empty = time_launches(torch, stream, lambda i: tb.turbo_stream_probe(tiny, None, tiny, stream=stream),
                                args.kernel_iters * 4, 40, "graph")
        empty_launch_us = round(t_empty.ms * 1e3, 3)
        for idx in range(5):
            sp = wl.config_spec(idx)
            k = ks if (idx == args.config and args.dtype == "config") else KernelSets(sp, torch, tb, wl, seed=args.seed)
            row = {"config": idx, "name": sp.name, "dtype": "f32" if sp.dtype == np.float32 else "f16"}
            for name, fn, per, nbytes, nrows, streamed in (
                    ("softmax", lambda i, k=k: k.softmax(i, stream), k.n_sm_sets, k.softmax_bytes, k.softmax_rows,
                     k.es * sp.B * sp.H * sp.Sq * sp.Sk),
                    ("layernorm", lambda i, k=k: k.layernorm(i, stream), k.n_ln_sets, k.layernorm_bytes, sp.rows,
                     3 * k.es * sp.rows * sp.hidden)):
                iters = args.kernel_iters if nbytes < (256 << 20) else max(10, args.kernel_iters // 4)
                t_cold = time_launches(torch, stream, fn, iters, per, args.launch)
                t_warm = time_launches(torch, stream, lambda i, fn=fn: fn(0), iters, 4, args.launch)
                # the plain stream of the same bytes, mix and buffers: in-place copy for softmax, out = x + residual
                # for LayerNorm (turbo_stream_probe, same access shape as the library's element-wise kernels)
                if name == "softmax":
                    probe = lambda i, k=k: tb.turbo_stream_probe(k.scores[i % k.n_sm_sets], None, k.scores[i % k.n_sm_sets],
                                                                 stream=stream)
                else:
                    probe = lambda i, k=k: tb.turbo_stream_probe(k.x[i % k.n_ln_sets], k.res[i % k.n_ln_sets],
                                                                 k.out[i % k.n_ln_sets], stream=stream)
                t_plain = time_launches(torch, stream, probe, iters, per, args.launch)
                rotated = per * streamed
                row[name] = {
                    "bytes": nbytes, "rows": nrows,
                    "cold_us": round(t_cold.ms * 1e3, 2), "cold_us_fastest_loop": round(t_cold.ms_min * 1e3, 2),
                    "cold_GBs": round(nbytes / t_cold.ms / 1e6, 1),
                    "cold_frac_of_8TBs": round(nbytes / t_cold.ms / 1e6 / HBM_PEAK_GBS, 4),
                    "cold_rows_per_s": round(nrows / (t_cold.ms * 1e-3), 1),
                    "warm_us": round(t_warm.ms * 1e3, 2), "warm_GBs": round(nbytes / t_warm.ms / 1e6, 1),
                    "plain_stream_us": round(t_plain.ms * 1e3, 2), "speed_vs_plain_stream": round(t_plain.ms / t_cold.ms, 3),
                    "launch": t_cold.mode, "plain_stream_launch": t_plain.mode, "buffer_sets": per,
                    "rotation_bytes": rotated,
                    "regime": "cold (rotation exceeds twice the 256 MB last-level cache)" if rotated >= (512 << 20)
                              else "cache-resident: the tensors are too small to rotate out of the last-level cache",
                }
            per_config.append(row)
            if k is not ks:
                del k
                torch.cuda.empty_cache()

    result = {
        "metric": "achieved HBM GB/s (fraction of peak) for softmax + add-bias-LayerNorm",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if spec.dtype == np.float32 else "f16", "data": "synthetic",
        "config": {
            "workload": f"configs[{spec.index}] {spec.name}: softmax [{spec.B},{spec.H},{spec.Sq},{spec.Sk}] in place + "
                        f"add-bias-LayerNorm [{spec.rows},{spec.hidden}]",
            "bytes_per_step": step_bytes, "launch": mode, "regime": f"cold, rotating {period} buffer sets",
            "frac_of_8TBs": round(value / HBM_PEAK_GBS, 4), "seed": args.seed,
            "timing": f"wall clock between device synchronisations around exactly {steps} steps; median of {HEADLINE_REPS} "
                      f"such repetitions",
            "ms_per_step_by_hip_events": round(ms_per_step_events, 6),
            "ms_per_step_all_repetitions": [round(r[0], 6) for r in runs],
        },
        "roofline": roof[dom],
        "roofline_other_kernel": roof[other],
    }
    if args.cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(spec, wl, torch, tb)
    if per_config:
        result["empty_launch_us"] = empty_launch_us
        result["per_config"] = per_config
        result["elementwise"] = elementwise_table(torch, tb, stream, args.launch, max(20, args.kernel_iters // 2))
        result["length_aware_config2"] = varlen_table(torch, tb, wl, stream, args.launch, max(20, args.kernel_iters // 2))
        result["scheduler_on_measured_costs"] = scheduler_table(torch, tb, wl, stream, args.launch, max(20, args.kernel_iters // 2))
    print(json.dumps(result))


if __name__ == "__main__":
    main()
