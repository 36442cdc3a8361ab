"""CPU oracle for the two host-side planning routines of the paper (test infrastructure only).

* batch scheduling (Section 5, Equation 2): the DEFINITION the dynamic program solves, written out as an
  exhaustive search: sort the requests by length, try every way of cutting the sorted list into consecutive
  batches of at most `max_batch` requests, keep the cheapest.  A batch of b requests whose longest has length L
  costs cached_cost[L][b] * b.
* memory planning (Section 4.2, Algorithm 1): not a definition but a greedy heuristic, so the oracle takes the
  algorithm's steps in the paper's order and notation (FindGapFromChunk, MemAllocate), in plain Python, plus a
  checker of the property the plan must have: tensors whose life times overlap never share bytes.
* cost table from samples (Section 6.3): bilinear weights over a sample grid, continued outside it.

Pinned by tests/test_serving_host.py (hand cases, closed forms, invariants).  Shares nothing with the C++ code.
"""
from __future__ import annotations

import bisect
import itertools
import math
from typing import Callable, List, Sequence, Tuple


# ---------------------------------------------------------------- batch scheduling

def schedule_cost(sorted_lengths: Sequence[int], cuts: Sequence[int], cost: Callable[[int, int], float]) -> float:
    """Total cost of cutting the sorted list at the given (exclusive) end positions."""
    total, begin = 0.0, 0
    for end in cuts:
        b = end - begin
        total += cost(sorted_lengths[end - 1], b) * b
        begin = end
    return total


def batch_schedule_exhaustive(lengths: Sequence[int], cost: Callable[[int, int], float], max_batch: int):
    """(minimal total cost, list of batch sizes of one optimal schedule) over all consecutive partitions."""
    s = sorted(lengths)
    n = len(s)
    best = (math.inf, None)
    for k in range(n):  # number of interior cut points
        for interior in itertools.combinations(range(1, n), k):
            cuts = list(interior) + [n]
            sizes = [e - b for b, e in zip([0] + cuts[:-1], cuts)]
            if max(sizes) > max_batch:
                continue
            c = schedule_cost(s, cuts, cost)
            if c < best[0]:
                best = (c, sizes)
    return best


def _axis_weights(grid: Sequence[int], v: int):
    """Two grid indices and their weights for linear inter-/extrapolation of position v on an increasing grid."""
    if len(grid) == 1:
        return 0, 0, 1.0, 0.0
    hi = bisect.bisect_right(list(grid), v)          # first line beyond v
    hi = min(max(hi, 1), len(grid) - 1)              # outside the grid: the outermost pair of lines
    lo = hi - 1
    t = (v - grid[lo]) / (grid[hi] - grid[lo])
    return lo, hi, 1.0 - t, t


def cost_table_from_samples(sample_len: Sequence[int], sample_batch: Sequence[int], sample_cost, max_len: int,
                            max_batch: int):
    """Dense per-request cost table [max_len+1][max_batch+1] from samples on a grid (Section 6.3, second strategy).

    Reading (the paper only says "interpolation"): weighted sum of the four surrounding samples with the product of the
    two axes' linear weights; outside the grid the weights of the outermost pair of lines are continued; negative
    results become 0; row 0 and column 0 are 0."""
    table = [[0.0] * (max_batch + 1) for _ in range(max_len + 1)]
    for length in range(1, max_len + 1):
        i0, i1, a0, a1 = _axis_weights(sample_len, length)
        for b in range(1, max_batch + 1):
            j0, j1, b0, b1 = _axis_weights(sample_batch, b)
            v = (a0 * b0 * sample_cost[i0][j0] + a0 * b1 * sample_cost[i0][j1] +
                 a1 * b0 * sample_cost[i1][j0] + a1 * b1 * sample_cost[i1][j1])
            table[length][b] = max(v, 0.0)
    return table


# ---------------------------------------------------------------- memory planning (Algorithm 1)

INVALID = None


def find_gap_from_chunk(t: int, chunk: List[Tuple[int, int]], chunk_size: int, first_op, last_op, size):
    """chunk: records (tensor_id, offset) in increasing offset order.  Returns an offset or INVALID."""
    smallest_gap = math.inf
    prev_offset = 0
    best_offset = INVALID
    for x, offset_x in chunk:
        max_first_op = max(first_op[t], first_op[x])
        min_last_op = min(last_op[t], last_op[x])
        if max_first_op <= min_last_op:
            gap = offset_x - prev_offset
            if gap >= size[t] and gap < smallest_gap:
                smallest_gap = gap
                best_offset = prev_offset
            prev_offset = max(prev_offset, offset_x + size[x])
    if best_offset is INVALID and chunk_size - prev_offset >= size[t]:
        best_offset = prev_offset
    return best_offset


def mem_allocate(first_op, last_op, size, chunk_sizes: Sequence[int], default_chunk_size: int = 2 << 20,
                 k_scale: float = 1.2):
    """Returns (assigned_chunk, assigned_offset, chunk sizes in use afterwards)."""
    n = len(size)
    order = sorted(range(n), key=lambda i: -size[i])  # non-increasing size, stable
    sizes = list(chunk_sizes)
    chunks: List[List[Tuple[int, int]]] = [[] for _ in sizes]
    assigned_chunk = [None] * n
    assigned_offset = [None] * n
    for t in order:
        is_assigned = False
        for chunk_id, chunk in enumerate(chunks):
            offset = find_gap_from_chunk(t, chunk, sizes[chunk_id], first_op, last_op, size)
            if offset is not INVALID:
                assigned_chunk[t], assigned_offset[t] = chunk_id, offset
                chunk.append((t, offset))
                chunk.sort(key=lambda r: r[1])
                is_assigned = True
                break
        if not is_assigned:
            new_chunk_size = max(default_chunk_size, math.ceil(size[t] * k_scale))
            assigned_chunk[t], assigned_offset[t] = len(chunks), 0
            sizes.append(new_chunk_size)
            chunks.append([(t, 0)])
    used = [c for c in range(len(chunks)) if chunks[c]]
    renumber = {c: i for i, c in enumerate(used)}
    return [renumber[c] for c in assigned_chunk], assigned_offset, [sizes[c] for c in used]


def plan_violations(first_op, last_op, size, assigned_chunk, assigned_offset, chunk_sizes) -> List[str]:
    """Every way in which a plan breaks its contract (empty list = valid)."""
    bad = []
    n = len(size)
    for t in range(n):
        c = assigned_chunk[t]
        if not (0 <= c < len(chunk_sizes)):
            bad.append(f"tensor {t}: chunk {c} does not exist")
            continue
        if assigned_offset[t] < 0 or assigned_offset[t] + size[t] > chunk_sizes[c]:
            bad.append(f"tensor {t}: [{assigned_offset[t]}, {assigned_offset[t] + size[t]}) leaves chunk {c}")
    for a in range(n):
        for b in range(a + 1, n):
            if assigned_chunk[a] != assigned_chunk[b]:
                continue
            alive_together = max(first_op[a], first_op[b]) <= min(last_op[a], last_op[b])
            share_bytes = (assigned_offset[a] < assigned_offset[b] + size[b]
                           and assigned_offset[b] < assigned_offset[a] + size[a])
            if alive_together and share_bytes:
                bad.append(f"tensors {a} and {b} are alive together and overlap in chunk {assigned_chunk[a]}")
    return bad


def peak_live_bytes(first_op, last_op, size) -> int:
    """Largest sum of sizes alive at one operator: a lower bound on the bytes any plan needs."""
    ops = sorted(set(first_op) | set(last_op))
    return max(sum(s for f, l, s in zip(first_op, last_op, size) if f <= op <= l) for op in ops)
