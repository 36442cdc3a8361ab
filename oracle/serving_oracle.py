"""CPU oracle for the two host-side planning routines of the paper (test infrastructure only).

* batch scheduling (Section 5, Equation 2): the DEFINITION the dynamic program solves, written out as an
  exhaustive search: sort the requests by length, try every way of cutting the sorted list into consecutive
  batches of at most `max_batch` requests, keep the cheapest.  A batch of b requests whose longest has length L
  costs cached_cost[L][b] * b.
* memory planning (Section 4.2, Algorithm 1): a greedy heuristic whose result is not unique, so what is checked is
  the contract a plan must meet -- tensors whose life times overlap never share bytes and stay inside their chunk,
  a new chunk has max(default, ceil(k * size)) bytes, the footprint is bounded below by the peak of live bytes --
  and, on instances of a few dozen bytes, the greedy choice itself by brute force over a byte map of every chunk
  (largest tensor first, first chunk with room, tightest hole, a new chunk only when nothing has room).
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

def _alive_together(first_op, last_op, a: int, b: int) -> bool:
    return first_op[a] <= last_op[b] and first_op[b] <= last_op[a]


def greedy_plan_by_byte_map(first_op, last_op, size, held_chunks: Sequence[int], default_chunk_size: int,
                            k_scale: float):
    """The plan the greedy rule fixes, found by brute force on a byte map (only for instances of a few dozen bytes).

    Tensors are taken largest first (equal sizes in input order).  For every chunk, in order, the bytes that some
    tensor alive together with the new one occupies are marked in a list of booleans, and the maximal runs of free
    bytes are read off it.  A run that ends at an occupied byte is a hole; the run that reaches the chunk's end is
    the open room.  The first chunk with a hole or open room that is long enough takes the tensor: at the start of
    the shortest sufficient hole (the lowest one among equals), else at the start of the open room.  If no chunk has
    room a chunk of max(default, ceil(k * size)) bytes is added.  Chunks that end up empty are dropped and the rest
    renumbered.  Returns (assigned_chunk, assigned_offset, chunk sizes in use)."""
    n = len(size)
    order = sorted(range(n), key=lambda t: (-size[t], t))
    capacities = [int(c) for c in held_chunks]
    members: List[List[int]] = [[] for _ in capacities]
    where = [None] * n  # (chunk, offset)
    for t in order:
        target = None
        for c, cap in enumerate(capacities):
            taken = [False] * cap
            for r in members[c]:
                if _alive_together(first_op, last_op, t, r):
                    for byte in range(where[r][1], where[r][1] + size[r]):
                        taken[byte] = True
            runs = []  # (start, length, reaches_the_end)
            byte = 0
            while byte < cap:
                if taken[byte]:
                    byte += 1
                    continue
                begin = byte
                while byte < cap and not taken[byte]:
                    byte += 1
                runs.append((begin, byte - begin, byte == cap))
            holes = [(length, begin) for begin, length, open_end in runs if not open_end and length >= size[t]]
            room = [begin for begin, length, open_end in runs if open_end and length >= size[t]]
            if holes:
                target = (c, min(holes)[1])
            elif room:
                target = (c, room[0])
            if target is not None:
                break
        if target is None:
            capacities.append(max(int(default_chunk_size), math.ceil(size[t] * k_scale)))
            members.append([])
            target = (len(capacities) - 1, 0)
        members[target[0]].append(t)
        where[t] = target
    used = [c for c in range(len(capacities)) if members[c]]
    new_index = {c: i for i, c in enumerate(used)}
    return [new_index[where[t][0]] for t in range(n)], [where[t][1] for t in range(n)], [capacities[c] for c in used]


def chunk_size_violations(size, assigned_chunk, assigned_offset, chunk_sizes, held_chunks: Sequence[int],
                          default_chunk_size: int, k_scale: float) -> List[str]:
    """The sizes of the chunks in use: the chunks kept from earlier inferences appear in their old order with their old
    sizes (those that ended up empty are dropped), then the chunks opened by this plan, each of
    max(default, ceil(k * size of the tensor that opened it)) bytes; that tensor sits at offset 0 and is the largest
    of its chunk, because tensors are placed largest first."""
    bad = []
    held = list(held_chunks)
    pos = 0
    kept = 0
    for c, cap in enumerate(chunk_sizes):
        while pos < len(held) and held[pos] != cap:  # dropped chunks
            pos += 1
        if pos < len(held):
            pos += 1
            kept += 1
            continue
        # not one of the held chunks: must follow the size rule for its largest tensor, which starts at offset 0
        inside = [t for t in range(len(size)) if assigned_chunk[t] == c]
        if not inside:
            bad.append(f"chunk {c} is in the list but holds no tensor")
            continue
        opener = max(inside, key=lambda t: size[t])
        want = max(int(default_chunk_size), math.ceil(size[opener] * k_scale))
        if cap != want:
            bad.append(f"new chunk {c} has {cap} bytes, the rule gives {want}")
        if not any(assigned_offset[t] == 0 and size[t] == size[opener] for t in inside):
            bad.append(f"new chunk {c}: no largest tensor at offset 0")
    for c in range(len(chunk_sizes)):
        if not any(assigned_chunk[t] == c for t in range(len(size))):
            bad.append(f"chunk {c} is kept although it holds no tensor")
    return bad


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
