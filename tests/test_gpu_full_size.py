"""Every element of configurations 2, 3 and 4 against the CPU oracle, at the configurations' full sizes and in the
launch configuration the benchmark times (the library's own plan, no overrides).

The oracle runs slab by slab on all host threads; each test covers one part of one tensor so that it ends within
seconds, and the parts of a tensor together cover all of it (slabs are dealt round-robin to the parts).  The GPU
result of a configuration is computed once and kept on the device for its parts.
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

SOFTMAX_PARTS = {2: 2, 3: 4, 4: 4}
_cache = {}


def _cached(key, make):
    """One entry at a time: the tensors of a configuration are gigabytes on the host."""
    if key not in _cache:
        _cache.clear()
        torch.cuda.empty_cache()
        _cache[key] = make()
    return _cache[key]


@pytest.fixture(autouse=True)
def _oracle_on_all_threads():
    orc.set_threads(gu.host_threads())
    yield
    orc.set_threads(1)


def _lengths_dev(v):
    return torch.from_numpy(np.asarray(v, dtype=np.int32)).cuda()


# ------------------------------------------------------------------ additive-mask softmax, as benchmarked

def _softmax_run(idx):
    case = wl.softmax_case(wl.config_spec(idx))
    return case, gu.run_softmax(case)


@pytest.mark.parametrize("idx,part", [(i, p) for i in (2, 3, 4) for p in range(SOFTMAX_PARTS[i])])
def test_softmax_every_element_of_the_full_size_configs(idx, part):
    case, out = _cached(("softmax", idx), lambda: _softmax_run(idx))
    stats = gu.ErrorStats()
    for b, h0, h1 in gu.softmax_slabs(case.shape, part, SOFTMAX_PARTS[idx]):
        got = out[b, h0:h1].cpu().numpy()
        want = gu.oracle_softmax_slab(case, b, h0, h1)
        stats.add(assert_parity(got, want, case.scores.dtype, f"softmax cfg{idx} request {b} heads {h0}..{h1 - 1}"), got.size)
    print(stats.line(f"softmax cfg{idx} part {part + 1}/{SOFTMAX_PARTS[idx]}"), flush=True)
    assert stats.n > 0


# ------------------------------------------------------------------ add-bias-LayerNorm, as benchmarked

def _layernorm_run(idx):
    case = wl.layernorm_case(wl.config_spec(idx))
    return case, gu.run_layernorm(case)


@pytest.mark.parametrize("idx", [2, 3, 4])
def test_layernorm_every_element_of_the_full_size_configs(idx):
    case, out = _cached(("layernorm", idx), lambda: _layernorm_run(idx))
    rows, hidden = case.shape
    stats = gu.ErrorStats()
    for r0, r1 in gu.row_ranges(rows, hidden):
        got = out[r0:r1].cpu().numpy()
        want = orc.add_bias_layernorm(case.x[r0:r1], case.residual[r0:r1], case.bias, case.gamma, case.beta, case.eps)
        stats.add(assert_parity(got, want, case.x.dtype, f"layernorm cfg{idx} rows {r0}..{r1 - 1}"), got.size)
    print(stats.line(f"layernorm cfg{idx}"), flush=True)
    assert stats.n == rows * hidden


# ------------------------------------------------------------------ length-aware and causal entry points

def _varlen_softmax_run():
    spec = wl.config_spec(2)
    case = wl.softmax_case(spec)
    poisoned = case.scores.copy()
    for b, n in enumerate(spec.lengths):  # what lies beyond the lengths must be neither read nor written
        poisoned[b, :, :, n:] = np.nan
        poisoned[b, :, n:, :] = np.nan
    s = gu.dev(poisoned)
    lens = _lengths_dev(spec.lengths)
    tb.turbo_masked_softmax_varlen(s, lens, lens, case.scale)
    torch.cuda.synchronize()
    return spec, case, s


@pytest.mark.parametrize("part", range(2))
def test_varlen_softmax_every_element_of_config_2(part):
    spec, case, out = _cached(("varlen softmax", 2), _varlen_softmax_run)
    B, H, Sq, Sk = case.shape
    stats = gu.ErrorStats()
    for b in range(part, B, 2):
        n = int(spec.lengths[b])
        got = out[b].cpu().numpy()
        want = orc.masked_softmax_varlen(case.scores[b:b + 1], [n], [n], case.scale)[0]
        stats.add(assert_parity(got[:, :n, :n], want[:, :n, :n], F32, f"varlen softmax cfg2 request {b} ({n} tokens)"),
                  H * n * n)
        assert (got[:, :n, n:] == 0).all(), f"request {b}: keys beyond the length must be exact zeros"
        assert np.isnan(got[:, n:, :]).all(), f"request {b}: padding rows must stay untouched"
    print(stats.line(f"varlen softmax cfg2 part {part + 1}/2, real rows and keys"), flush=True)


def test_varlen_layernorm_every_element_of_config_2():
    spec = wl.config_spec(2)
    case = wl.layernorm_case(spec)
    B, S, hidden = spec.B, spec.Sk, spec.hidden
    x, r = case.x.reshape(B, S, hidden).copy(), case.residual.reshape(B, S, hidden).copy()
    for b, n in enumerate(spec.lengths):
        x[b, n:] = np.nan
        r[b, n:] = np.nan
    out = torch.full((B, S, hidden), float("nan"), dtype=torch.float32, device="cuda")
    tb.turbo_add_bias_layernorm_varlen(gu.dev(x), gu.dev(r), gu.dev(case.bias), gu.dev(case.gamma), gu.dev(case.beta),
                                       _lengths_dev(spec.lengths), case.eps, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = orc.add_bias_layernorm(case.x, case.residual, case.bias, case.gamma, case.beta, case.eps).reshape(B, S, hidden)
    stats = gu.ErrorStats()
    for b, n in enumerate(spec.lengths):
        stats.add(assert_parity(got[b, :n], want[b, :n], F32, f"varlen layernorm cfg2 request {b}"), n * hidden)
        assert np.isnan(got[b, n:]).all(), f"request {b}: padding rows must stay untouched"
    print(stats.line("varlen layernorm cfg2, real rows"), flush=True)


def _causal_run():
    spec = wl.config_spec(4)
    case = wl.softmax_case(spec)
    Sq, Sk = spec.Sq, spec.Sk
    poisoned = case.scores.copy()
    poisoned[:, :, np.triu(np.ones((Sq, Sk), dtype=bool), 1)] = np.nan  # keys above the diagonal must not be read
    s = gu.dev(poisoned)
    tb.turbo_masked_softmax_causal(s, None, None, case.scale)
    torch.cuda.synchronize()
    return case, s


@pytest.mark.parametrize("part", range(4))
def test_causal_softmax_every_element_of_config_4(part):
    case, out = _cached(("causal softmax", 4), _causal_run)
    B, H, Sq, Sk = case.shape
    stats = gu.ErrorStats()
    for b, h0, h1 in gu.softmax_slabs(case.shape, part, 4):
        got = out[b, h0:h1].cpu().numpy()
        want = orc.masked_softmax_causal(case.scores[b:b + 1, h0:h1], None, None, case.scale)[0]
        stats.add(assert_parity(got, want, F16, f"causal softmax cfg4 request {b} heads {h0}..{h1 - 1}"), got.size)
    print(stats.line(f"causal softmax cfg4 part {part + 1}/4"), flush=True)


def test_packed_softmax_every_element_of_config_2():
    """Config 2's 32 requests without any padding in memory: every request against the oracle."""
    spec = wl.config_spec(2)
    lengths = [int(v) for v in spec.lengths]
    case = wl.softmax_case(spec)
    flat = np.concatenate([case.scores[b, :, :n, :n].reshape(-1) for b, n in enumerate(lengths)])
    cu, off = wl.packed_layout(lengths, spec.H)
    s = gu.dev(flat)
    tb.turbo_masked_softmax_packed(s, torch.from_numpy(cu).cuda(), torch.from_numpy(off).cuda(), spec.H, int(cu[-1]),
                                   max(lengths), spec.scale)
    torch.cuda.synchronize()
    got = s.cpu().numpy()
    want = orc.masked_softmax_packed(flat, lengths, spec.H, spec.scale)
    stats = gu.ErrorStats()
    stats.add(assert_parity(got, want, F32, "packed softmax cfg2"), got.size)
    print(stats.line("packed softmax cfg2"), flush=True)
