"""Host-side planning routines (DP batch scheduler, sequence-length-aware allocator): the oracles against their pins,
and the C++ implementation against them (the scheduler against exhaustive search; the allocator against its contract,
hand cases and, on tiny instances, a byte-map brute force).  CPU only."""
import math

import numpy as np
import pytest

from oracle import serving_oracle as so
from paper_2010_05680_amd import binding as tb
from paper_2010_05680_amd import serving as sv


def _table(cost, max_len, max_batch):
    t = np.zeros((max_len + 1, max_batch + 1))
    for L in range(1, max_len + 1):
        for b in range(1, max_batch + 1):
            t[L, b] = cost(L, b)
    return t


# ------------------------------------------------------------------ scheduler: oracle pins

def test_scheduler_oracle_two_requests_by_hand():
    cost = lambda L, b: {(3, 1): 5.0, (9, 1): 7.0, (9, 2): 4.0}[(L, b)]
    assert so.batch_schedule_exhaustive([9, 3], cost, 2) == (8.0, [2])        # 2*4 < 5+7
    cost2 = lambda L, b: {(3, 1): 5.0, (9, 1): 7.0, (9, 2): 6.5}[(L, b)]
    assert so.batch_schedule_exhaustive([9, 3], cost2, 2) == (12.0, [1, 1])   # 13 > 5+7


def test_scheduler_oracle_closed_forms():
    lengths = [40, 7, 19, 8, 63, 22]  # distinct, so that padding always costs something
    # no benefit from batching (per-request cost ignores the batch size): serving one by one is optimal
    c, sizes = so.batch_schedule_exhaustive(lengths, lambda L, b: 0.5 * L + 1.0, 6)
    assert sizes == [1] * 6 and c == pytest.approx(sum(0.5 * L + 1.0 for L in lengths))
    # a batch costs the same whatever it holds: one batch of everything, unless the cap forbids it
    assert so.batch_schedule_exhaustive(lengths, lambda L, b: 10.0 / b, 6) == (10.0, [6])
    c, sizes = so.batch_schedule_exhaustive(lengths, lambda L, b: 10.0 / b, 4)
    assert c == 20.0 and len(sizes) == 2 and max(sizes) <= 4


def test_scheduler_paper_example_under_an_affine_cost_model():
    """Section 5's example: lengths 17, 18, 52, 63, 77; one batch of five is worse than no batching and three
    batches are optimal.  The paper's cost table is not printed; with batch time = a + c*len*b this is exactly
    the regime 11c < a < 28c (derivation in the test body), where the optimum is {17,18} {52,63} {77}."""
    lengths = [17, 18, 52, 63, 77]
    a, c = 20.0, 1.0
    cost = lambda L, b: (a + c * L * b) / b
    best, sizes = so.batch_schedule_exhaustive(lengths, cost, 5)
    assert sizes == [2, 2, 1] and best == pytest.approx(3 * a + c * (36 + 126 + 77))
    no_batching = sum(cost(L, 1) for L in lengths)
    one_batch = cost(77, 5) * 5
    assert one_batch > no_batching > best


# ------------------------------------------------------------------ scheduler: C++ against the oracle

@pytest.mark.parametrize("seed", range(12))
def test_scheduler_matches_exhaustive_search(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 13))
    max_len = 60
    max_batch = int(rng.integers(1, n + 2))
    lengths = rng.integers(1, max_len + 1, size=n)
    kind = seed % 3
    if kind == 0:    # fixed overhead + work
        a, c = rng.uniform(1, 50), rng.uniform(0.1, 2)
        cost = lambda L, b: (a + c * L * b) / b
    elif kind == 1:  # arbitrary table
        tab = rng.uniform(0.1, 10, size=(max_len + 1, max_batch + 1))
        cost = lambda L, b: float(tab[L, b])
    else:            # saturating batching benefit
        cost = lambda L, b: L * (1.0 + 3.0 / b) + 2.0
    table = _table(cost, max_len, max_batch)
    batches, total = sv.turbo_batch_schedule(lengths, table, max_batch)
    want_cost, _ = so.batch_schedule_exhaustive(list(lengths), lambda L, b: float(table[L, b]), max_batch)
    assert total == pytest.approx(want_cost, rel=1e-12)
    # the schedule itself: a partition of the requests, sorted by length, batches within the cap, cost as claimed
    flat = [i for b in batches for i in b]
    assert sorted(flat) == list(range(n))
    assert [lengths[i] for i in flat] == sorted(lengths)
    assert all(1 <= len(b) <= max_batch for b in batches)
    assert sum(table[max(lengths[i] for i in b), len(b)] * len(b) for b in batches) == pytest.approx(total, rel=1e-12)


def test_scheduler_paper_example_and_ties():
    lengths = [77, 17, 63, 18, 52]
    table = _table(lambda L, b: (20.0 + L * b) / b, 80, 5)
    batches, total = sv.turbo_batch_schedule(lengths, table, 5)
    assert [[lengths[i] for i in b] for b in batches] == [[17, 18], [52, 63], [77]]
    assert total == pytest.approx(299.0)
    # equal lengths keep their arrival order; on equal cost the strict comparison keeps the smaller last batch
    batches, total = sv.turbo_batch_schedule([5, 5, 5], _table(lambda L, b: 1.0, 5, 3), 3)
    assert batches == [[0], [1], [2]] and total == 3.0


def test_scheduler_rejects_bad_input():
    L = sv._lib()
    one = np.zeros(4)
    with pytest.raises(tb.TurboError):
        sv.turbo_batch_schedule([0, 3], _table(lambda L, b: 1.0, 5, 2), 2)   # length 0
    with pytest.raises(tb.TurboError):
        sv.turbo_batch_schedule([9], _table(lambda L, b: 1.0, 5, 2), 2)      # beyond the table
    assert L.turbo_batch_schedule(None, 1, None, 1, 1, None, None, None, None) == tb.TURBO_ERR_NULL


# ------------------------------------------------------------------ cost table from samples

SAMPLE_LEN, SAMPLE_BATCH = [8, 64, 200, 500], [1, 4, 16]


def test_cost_table_oracle_reproduces_samples_and_bilinear_models_exactly():
    """Pins: equality at the sample points; a cost of the form a + b*len + c*batch + d*len*batch is reproduced
    everywhere, inside and outside the grid (closed form); one sampled length or batch size means constant along
    that axis; continued lines that would go negative stop at zero."""
    model = lambda L, b: 3.0 + 0.25 * L + 1.5 * b + 0.01 * L * b
    samples = [[model(L, b) for b in SAMPLE_BATCH] for L in SAMPLE_LEN]
    table = so.cost_table_from_samples(SAMPLE_LEN, SAMPLE_BATCH, samples, 600, 20)
    for L in range(1, 601):
        for b in range(1, 21):
            assert table[L][b] == pytest.approx(model(L, b), rel=1e-12)
    bumpy = [[math.sin(L) + 0.1 * b * b + 5 for b in SAMPLE_BATCH] for L in SAMPLE_LEN]
    table = so.cost_table_from_samples(SAMPLE_LEN, SAMPLE_BATCH, bumpy, 500, 16)
    for i, L in enumerate(SAMPLE_LEN):
        for j, b in enumerate(SAMPLE_BATCH):
            assert table[L][b] == pytest.approx(bumpy[i][j], rel=1e-12)
    assert all(table[0][b] == 0 for b in range(17)) and all(table[L][0] == 0 for L in range(501))
    flat = so.cost_table_from_samples([100], [2], [[7.0]], 300, 8)
    assert all(flat[L][b] == 7.0 for L in range(1, 301) for b in range(1, 9))
    falling = so.cost_table_from_samples([10, 20], [1], [[10.0], [1.0]], 40, 1)
    assert falling[30][1] == 0.0 and falling[15][1] == pytest.approx(5.5)


def test_cost_table_oracle_matches_library_interpolation_inside_the_grid():
    from scipy.interpolate import RegularGridInterpolator
    rng = np.random.default_rng(5)
    samples = rng.uniform(1, 9, size=(len(SAMPLE_LEN), len(SAMPLE_BATCH)))
    table = np.array(so.cost_table_from_samples(SAMPLE_LEN, SAMPLE_BATCH, samples.tolist(), 500, 16))
    f = RegularGridInterpolator((SAMPLE_LEN, SAMPLE_BATCH), samples, method="linear")
    pts = np.array([(L, b) for L in range(8, 501) for b in range(1, 17)], dtype=float)
    np.testing.assert_allclose(table[8:501, 1:17].reshape(-1), f(pts), rtol=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_cost_table_matches_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    n_len, n_batch = int(rng.integers(1, 6)), int(rng.integers(1, 5))
    sl = np.sort(rng.choice(np.arange(1, 300), size=n_len, replace=False)).tolist()
    sb = np.sort(rng.choice(np.arange(1, 33), size=n_batch, replace=False)).tolist()
    sc = rng.uniform(0.5, 20, size=(n_len, n_batch))
    got = sv.turbo_cost_table_fill(sl, sb, sc, 320, 40)
    want = np.array(so.cost_table_from_samples(sl, sb, sc.tolist(), 320, 40))
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    for i, L in enumerate(sl):
        for j, b in enumerate(sb):
            assert got[L, b] == pytest.approx(sc[i, j], rel=1e-13)


def test_cost_table_feeds_the_scheduler_and_rejects_bad_grids():
    # samples of the affine model behind the paper's example, taken at a few lengths and batch sizes only
    model = lambda L, b: (20.0 + L * b) / b
    sl, sb = [10, 40, 80], [1, 2, 5]
    table = sv.turbo_cost_table_fill(sl, sb, np.array([[model(L, b) for b in sb] for L in sl]), 80, 5)
    lengths = [77, 17, 63, 18, 52]
    batches, _ = sv.turbo_batch_schedule(lengths, table, 5)
    assert [[lengths[i] for i in b] for b in batches] == [[17, 18], [52, 63], [77]]
    with pytest.raises(tb.TurboError):
        sv.turbo_cost_table_fill([10, 10], [1], np.ones((2, 1)), 20, 2)   # grid not strictly increasing
    with pytest.raises(tb.TurboError):
        sv.turbo_cost_table_fill([0, 10], [1], np.ones((2, 1)), 20, 2)    # length 0
    with pytest.raises(tb.TurboError):
        sv.turbo_cost_table_fill([5], [1], np.ones((1, 1)), 0, 2)
    assert sv._lib().turbo_cost_table_fill(None, 1, None, 1, None, 1, 1, None) == tb.TURBO_ERR_NULL


# ------------------------------------------------------------------ allocator: hand cases and the contract
#
# A plan of this greedy heuristic is not unique in general, so there is no "expected output" to transcribe.  What is
# fixed: the contract every plan must meet (so.plan_violations, so.chunk_size_violations, the peak of live bytes as a
# lower bound), hand cases small enough to place by eye, and, on instances of a few dozen bytes, the greedy choice
# itself, found by brute force on a byte map (so.greedy_plan_by_byte_map).  The hand cases pin the brute force too.

def _plans(first, last, size, held, default, k_scale=1.2):
    """The C++ planner's plan and the byte-map brute force's, for cases small enough for the latter."""
    return (sv.turbo_mem_plan(first, last, size, held, default, k_scale),
            so.greedy_plan_by_byte_map(first, last, size, held, default, k_scale))


def test_allocator_reuses_the_bytes_of_dead_tensors():
    # two tensors that never live together share offset 0; a third that lives with both goes behind the larger
    first, last, size = [0, 3, 0], [2, 5, 5], [100, 80, 50]
    for chunk, offset, chunks in _plans(first, last, size, [], 256):
        assert chunk == [0, 0, 0] and offset == [0, 0, 100] and chunks == [256]
        assert so.plan_violations(first, last, size, chunk, offset, chunks) == []


def test_allocator_takes_the_tightest_hole_that_holds_the_tensor():
    """Placed largest first: A(100)@0, D(60)@100, X(45)@160, B(40)@205, Y(25)@245, Z(22)@270, all alive from the start.
    X and Y die at operator 3, which leaves holes of 45 bytes at 160 and of 25 bytes at 245 for a tensor born at 5."""
    first = [0, 0, 0, 0, 0, 0, 5]
    last = [9, 9, 3, 9, 3, 9, 9]
    base = [100, 60, 45, 40, 25, 22]
    for newcomer, want_offset in ((20, 245),    # placed last; fits both holes: the 25-byte one is tighter
                                  (25, 160),    # as large as Y, so placed before Z: behind B there is only open room
                                  (30, 160)):   # placed before Y and Z; only the 45-byte hole holds it
        size = base + [newcomer]
        for chunk, offset, chunks in _plans(first, last, size, [], 400):
            assert offset[:6] == [0, 100, 160, 205, 245, 270] and chunk == [0] * 7 and chunks == [400]
            assert offset[6] == want_offset, (newcomer, offset)
            assert so.plan_violations(first, last, size, chunk, offset, chunks) == []
    # a newcomer of 50 bytes is placed third, behind D; X, which it never meets, then shares its first bytes, and
    # everything smaller moves up: B behind the newcomer, Y behind B (the 5 bytes between X and B hold nothing), Z last
    size = base + [50]
    for chunk, offset, chunks in _plans(first, last, size, [], 400):
        assert offset == [0, 100, 160, 210, 250, 275, 160] and chunks == [400]
    # in a chunk of 280 bytes Z no longer fits behind Y: a second chunk of max(default, ceil(1.2 * 22)) bytes
    for chunk, offset, chunks in _plans(first, last, size, [], 280):
        assert chunk == [0, 0, 0, 0, 0, 1, 0] and offset[5] == 0 and chunks == [280, 280]
    # a hole between two residents wins over open room behind them even when the open room is the tighter fit
    first, last, size = [0, 0, 0, 4], [9, 2, 9, 9], [50, 30, 20, 10]
    for chunk, offset, chunks in _plans(first, last, size, [], 112):
        # A(50)@0, X(30)@50 dies at 2, Z(20)@80; the newcomer (10, born at 4) sees a hole of 30 at 50 and 12 bytes of
        # open room at 100
        assert offset == [0, 50, 80, 50] and chunks == [112]


def test_allocator_opens_chunks_by_the_size_rule_and_gives_back_unused_ones():
    first, last = [0, 0], [1, 1]
    # a tensor larger than the default chunk gets ceil(1.2 * size); the small one fits behind it
    for chunk, offset, chunks in _plans(first, last, [1000, 10], [], 512):
        assert chunks == [1200] and chunk == [0, 0] and offset == [0, 1000]
    # chunks left over from a longer request are given back when a short one does not need them
    for chunk, offset, chunks in _plans([0], [0], [100], [512, 2048, 512], 512):
        assert chunks == [512] and chunk == [0]
    # ... and the one that is used keeps its size even if it is not the first
    for chunk, offset, chunks in _plans([0], [0], [1000], [512, 2048, 512], 512):
        assert chunks == [2048] and chunk == [0] and offset == [0]
    # the first chunk with room wins, not the one with the tightest hole
    for chunk, offset, chunks in _plans([0], [0], [100], [2048, 128], 512):
        assert chunks == [2048] and chunk == [0]
    # ceil, not floor: 1.2 * 1001 = 1201.2
    for chunk, offset, chunks in _plans([0], [0], [1001], [], 512):
        assert chunks == [1202]


def _bert_like_records(seq, rng=None):
    """Life times and sizes shaped like one encoder layer's intermediates for a request of `seq` tokens."""
    h, heads = 768, 12
    recs = [(0, 1, 3 * seq * h), (1, 4, seq * h), (1, 2, seq * h), (1, 4, seq * h), (2, 3, heads * seq * seq),
            (3, 4, heads * seq * seq), (4, 5, seq * h), (5, 6, seq * h), (6, 7, seq * h), (7, 8, 4 * seq * h),
            (8, 9, 4 * seq * h), (9, 10, seq * h)]
    first, last, size = zip(*recs)
    return list(first), list(last), [4 * s for s in size]


@pytest.mark.parametrize("seq", [5, 40, 128, 200, 240, 500])
def test_allocator_plan_is_valid_and_not_wasteful(seq):
    first, last, size = _bert_like_records(seq)
    chunk, offset, chunks = sv.turbo_mem_plan(first, last, size, [])
    assert so.plan_violations(first, last, size, chunk, offset, chunks) == []
    assert so.chunk_size_violations(size, chunk, offset, chunks, [], 2 << 20, 1.2) == []
    peak = so.peak_live_bytes(first, last, size)
    assert sum(chunks) >= peak
    assert sum(chunks) <= max(2 << 20, 1.2 * peak) + len(chunks) * (2 << 20)


def test_plan_checkers_notice_a_bad_plan():
    first, last, size = [0, 0], [1, 1], [10, 10]
    assert so.plan_violations(first, last, size, [0, 0], [0, 5], [100]) != []      # overlapping bytes
    assert so.plan_violations(first, last, size, [0, 0], [0, 95], [100]) != []     # leaves the chunk
    assert so.plan_violations(first, last, size, [0, 1], [0, 0], [100]) != []      # missing chunk
    assert so.plan_violations(first, last, size, [0, 0], [0, 10], [100]) == []
    assert so.chunk_size_violations(size, [0, 0], [0, 10], [100], [], 100, 1.2) == []
    assert so.chunk_size_violations(size, [0, 0], [0, 10], [101], [], 100, 1.2) != []    # not the rule's size
    assert so.chunk_size_violations(size, [0, 0], [5, 15], [100], [], 100, 1.2) != []    # nothing at offset 0
    assert so.chunk_size_violations(size, [0, 0], [0, 10], [100, 64], [64], 100, 1.2) != []  # an empty chunk is kept
    assert so.peak_live_bytes([0, 2, 1], [1, 3, 2], [10, 20, 5]) == 25


# ------------------------------------------------------------------ allocator: C++ against brute force and contract

@pytest.mark.parametrize("seed", range(40))
def test_allocator_makes_the_greedy_choice_on_instances_small_enough_for_brute_force(seed):
    """A few tensors of a few bytes each: the byte-map brute force fixes the plan of the greedy rule, and the C++
    planner must produce exactly it (equal sizes, holes of equal length and exact fits occur often at this scale)."""
    rng = np.random.default_rng(300 + seed)
    n = int(rng.integers(1, 14))
    n_ops = int(rng.integers(1, 9))
    first = [int(v) for v in rng.integers(0, n_ops, size=n)]
    last = [min(n_ops - 1, f + int(d)) for f, d in zip(first, rng.integers(0, 4, size=n))]
    size = [int(v) for v in rng.integers(1, 13, size=n)]
    held = [int(v) for v in rng.integers(4, 40, size=int(rng.integers(0, 4)))]
    default = int(rng.choice([8, 16, 48]))
    k_scale = float(rng.choice([1.0, 1.2, 2.0]))
    got = sv.turbo_mem_plan(first, last, size, held, default, k_scale)
    want = so.greedy_plan_by_byte_map(first, last, size, held, default, k_scale)
    assert got == want, (first, last, size, held, default, k_scale)
    assert so.plan_violations(first, last, size, *got) == []
    assert so.chunk_size_violations(size, *got, held, default, k_scale) == []


@pytest.mark.parametrize("seed", range(20))
def test_allocator_meets_its_contract_on_large_random_instances(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(1, 40))
    n_ops = int(rng.integers(1, 25))
    first = rng.integers(0, n_ops, size=n)
    last = np.minimum(n_ops - 1, first + rng.integers(0, 6, size=n))
    size = rng.integers(1, 5000, size=n) * int(rng.choice([1, 64, 1024]))
    held = [int(v) for v in rng.integers(1, 4, size=int(rng.integers(0, 4))) * 4096]
    default = int(rng.choice([1024, 4096, 2 << 20]))
    chunk, offset, chunks = sv.turbo_mem_plan(first, last, size, held, default, 1.2)
    assert so.plan_violations(first, last, size, chunk, offset, chunks) == []
    assert so.chunk_size_violations([int(v) for v in size], chunk, offset, chunks, held, default, 1.2) == []
    assert sum(chunks) >= so.peak_live_bytes(first, last, size)
    # largest first: nothing larger than a chunk's resident at offset 0 can sit in a chunk this plan opened
    assert len(chunks) <= len(held) + n


@pytest.mark.parametrize("seqs", [[200, 240], [500, 5, 128], [40, 40, 41]])
def test_allocator_across_consecutive_requests(seqs):
    """Chunks carry over from one inference to the next, as in the paper's Figure 6 scenario (length 200 then 240)."""
    held = []
    counts = []
    for seq in seqs:
        first, last, size = _bert_like_records(seq)
        before = list(held)
        chunk, offset, held = sv.turbo_mem_plan(first, last, size, held)
        assert so.plan_violations(first, last, size, chunk, offset, held) == []
        assert so.chunk_size_violations(size, chunk, offset, held, before, 2 << 20, 1.2) == []
        assert sum(held) >= so.peak_live_bytes(first, last, size)
        counts.append(len(held))
    if seqs == [200, 240]:
        assert counts[1] >= counts[0]  # the longer request keeps the chunks and may add to them
    if seqs == [40, 40, 41]:
        assert counts[0] == counts[1]  # the same request again needs nothing new


@pytest.mark.parametrize("seq", [17, 128, 493])
def test_one_layer_plan_is_reused_by_every_repeated_layer(seq):
    """Section 6.2.2's way to keep the O(#tensor^2) planner cheap: plan the tensors of ONE of the repeated layers
    and use the same offsets in all of them.  What makes that valid is the record given to the tensor that crosses
    the layer boundary (a layer's output is the next layer's input and residual): it lives for the whole layer in
    the one-layer plan.  Checked by unrolling 12 layers with the one-layer offsets and running the plan checker
    over all 12 * 12 + 1 tensors with their true life times."""
    ops = 12  # operators per layer
    first, last, size = _bert_like_records(seq)
    carried = 4 * seq * 768
    f1, l1, s1 = first + [0], last + [ops - 1], size + [carried]
    chunk, offset, chunks = sv.turbo_mem_plan(f1, l1, s1, [])
    assert so.plan_violations(f1, l1, s1, chunk, offset, chunks) == []
    layers = 12
    uf, ul, us, uc, uo = [], [], [], [], []
    for k in range(layers):
        for t in range(len(first)):
            uf.append(first[t] + k * ops)
            ul.append(last[t] + k * ops)
            us.append(size[t]); uc.append(chunk[t]); uo.append(offset[t])
    # boundary tensors: the model input feeds layer 0; layer k's output (written by its last operator) is read by
    # layer k+1 up to its residual add (operator 7)
    uf.append(0); ul.append(7); us.append(carried); uc.append(chunk[-1]); uo.append(offset[-1])
    for k in range(layers):
        uf.append(k * ops + ops - 1)
        ul.append(min((k + 1) * ops + 7, layers * ops - 1))
        us.append(carried); uc.append(chunk[-1]); uo.append(offset[-1])
    assert so.plan_violations(uf, ul, us, uc, uo, chunks) == []
    # and the footprint is that of one layer, not of twelve
    assert sum(chunks) <= max(2 << 20, 1.2 * so.peak_live_bytes(f1, l1, s1)) + len(chunks) * (2 << 20)


def test_allocator_rejects_bad_input():
    with pytest.raises(tb.TurboError):
        sv.turbo_mem_plan([2], [1], [10], [])          # last before first
    with pytest.raises(tb.TurboError):
        sv.turbo_mem_plan([0], [1], [0], [])           # empty tensor
    with pytest.raises(tb.TurboError):
        sv.turbo_mem_plan([0], [1], [10], [], k_scale=0.5)
    with pytest.raises(tb.TurboError):
        sv.turbo_mem_plan([0, 0], [1, 1], [10, 10], [], default_chunk_size=10, k_scale=1.0, max_chunks=1)


def test_host_routines_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """Compiles the host-side C++ with -fsanitize=address,undefined into a small driver (tests/native/) that runs
    random instances, rejected ones included, with output arrays of exactly the documented sizes."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = tmp_path / "host_sanitize"
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-static-libasan", "-static-libubsan",  # the runtimes inside the program: no load-order demands
                           os.path.join(root, "tests", "native", "host_sanitize.cpp"),
                           os.path.join(root, "paper_2010_05680_amd", "csrc", "serving_host.cpp"), "-o", str(exe)])
    res = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0 and res.stdout.strip() == "ok", res.stdout + res.stderr
