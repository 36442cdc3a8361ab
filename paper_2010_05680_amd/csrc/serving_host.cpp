// Host-side planning routines: the DP batch scheduler (Algorithm 2 / Equation 2) and the sequence-length-aware
// allocator (Algorithm 1) of the paper.  Plain C++, no GPU work.
#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <vector>

#include "../../include/turbo_reduce.h"
#include "../../include/turbo_serving.h"

extern "C" int turbo_batch_schedule(const int* lengths, int n, const double* cached_cost, int max_len, int max_batch,
                                    int* order, int* batch_end, int* n_batches, double* total_cost) {
    if (!lengths || !cached_cost || !order || !batch_end || !n_batches || !total_cost) return TURBO_ERR_NULL;
    if (n <= 0 || max_len <= 0 || max_batch <= 0) return TURBO_ERR_SHAPE;
    for (int i = 0; i < n; ++i)
        if (lengths[i] < 1 || lengths[i] > max_len) return TURBO_ERR_SHAPE;

    std::iota(order, order + n, 0);
    std::stable_sort(order, order + n, [&](int a, int b) { return lengths[a] < lengths[b]; });

    const long long stride = (long long)max_batch + 1;
    // states[i]: least cost of serving the first i sorted requests; start[i]: where their last batch begins
    std::vector<double> states(n + 1, 0.0);
    std::vector<int> start(n + 1, 0);
    for (int i = 1; i <= n; ++i) {
        const int cur_len = lengths[order[i - 1]];  // longest request of any batch that ends here
        double best = std::numeric_limits<double>::infinity();
        int best_start = i - 1;
        for (int j = i - 1; j >= 0 && i - j <= max_batch; --j) {  // batch = sorted requests j .. i-1
            const int b = i - j;
            const double cost = states[j] + cached_cost[cur_len * stride + b] * b;
            if (cost < best) {
                best = cost;
                best_start = j;
            }
        }
        states[i] = best;
        start[i] = best_start;
    }
    // walk back from the end to list the batches, then reverse
    int count = 0;
    for (int i = n; i > 0; i = start[i]) batch_end[count++] = i;
    std::reverse(batch_end, batch_end + count);
    *n_batches = count;
    *total_cost = states[n];
    return TURBO_OK;
}

namespace {

// Position of v on a strictly increasing grid g[0..n): the cell index i (0 <= i <= n-2) whose two lines bracket v,
// or the outermost cell when v lies outside the grid, and the weight w of line i+1 (outside the grid w < 0 or > 1:
// the cell's line is continued).  A grid of one line gives cell 0 with weight 0.
void grid_cell(const int* g, int n, int v, int* cell, double* w) {
    if (n == 1) {
        *cell = 0;
        *w = 0.0;
        return;
    }
    int i = 0;
    while (i < n - 2 && v >= g[i + 1]) ++i;
    *cell = i;
    *w = (double)(v - g[i]) / (double)(g[i + 1] - g[i]);
}

}  // namespace

extern "C" int turbo_cost_table_fill(const int* sample_len, int n_len, const int* sample_batch, int n_batch,
                                     const double* sample_cost, int max_len, int max_batch, double* cached_cost) {
    if (!sample_len || !sample_batch || !sample_cost || !cached_cost) return TURBO_ERR_NULL;
    if (n_len <= 0 || n_batch <= 0 || max_len <= 0 || max_batch <= 0) return TURBO_ERR_SHAPE;
    for (int i = 0; i < n_len; ++i)
        if (sample_len[i] < 1 || (i > 0 && sample_len[i] <= sample_len[i - 1])) return TURBO_ERR_SHAPE;
    for (int j = 0; j < n_batch; ++j)
        if (sample_batch[j] < 1 || (j > 0 && sample_batch[j] <= sample_batch[j - 1])) return TURBO_ERR_SHAPE;
    const long long stride = (long long)max_batch + 1;
    for (int len = 0; len <= max_len; ++len) {
        int ci;
        double wi;
        grid_cell(sample_len, n_len, len, &ci, &wi);
        const int ci1 = n_len > 1 ? ci + 1 : ci;
        for (int b = 0; b <= max_batch; ++b) {
            if (len == 0 || b == 0) {
                cached_cost[len * stride + b] = 0.0;
                continue;
            }
            int cj;
            double wj;
            grid_cell(sample_batch, n_batch, b, &cj, &wj);
            const int cj1 = n_batch > 1 ? cj + 1 : cj;
            const double c00 = sample_cost[(long long)ci * n_batch + cj], c01 = sample_cost[(long long)ci * n_batch + cj1];
            const double c10 = sample_cost[(long long)ci1 * n_batch + cj], c11 = sample_cost[(long long)ci1 * n_batch + cj1];
            const double lo = c00 + (c01 - c00) * wj, hi = c10 + (c11 - c10) * wj;
            const double v = lo + (hi - lo) * wi;
            cached_cost[len * stride + b] = v > 0.0 ? v : 0.0;  // a continued line may cross zero: costs do not
        }
    }
    return TURBO_OK;
}

namespace {

// The planner's contract (Section 4.2): tensors whose life times overlap never share bytes; tensors are placed
// largest first; a tensor goes into the first chunk that has room for it, into the tightest hole that holds it, and
// a new chunk is opened only when no chunk has room.  The paper's Algorithm 1 is one way to meet it; what follows is
// written from that contract: per chunk, the bytes that are busy while the tensor lives are swept once in address
// order and the holes between them are the candidates.

struct Span {  // bytes [begin, end) of a chunk
    long long begin, end;
};

struct Chunk {
    long long capacity;
    std::vector<int> residents;  // tensors placed in this chunk so far, in no particular order
};

struct Lifetimes {
    const int* first_op;
    const int* last_op;
    bool overlap(int a, int b) const { return first_op[a] <= last_op[b] && first_op[b] <= last_op[a]; }
};

// Offset for `need` bytes of tensor t in `chunk`, or -1 when the chunk has no room while t lives.
// `busy` is scratch storage reused between calls.
long long place_in_chunk(const Chunk& chunk, int t, long long need, const Lifetimes& life, const long long* size,
                         const long long* offset_of, std::vector<Span>& busy) {
    busy.clear();
    for (int r : chunk.residents)
        if (life.overlap(t, r)) busy.push_back(Span{offset_of[r], offset_of[r] + size[r]});
    std::sort(busy.begin(), busy.end(), [](const Span& a, const Span& b) { return a.begin < b.begin; });

    long long frontier = 0;    // everything below is covered by the spans seen so far, or is a hole already examined
    long long tightest = -1;   // begin of the smallest hole that holds the tensor
    long long tightest_len = std::numeric_limits<long long>::max();
    for (const Span& sp : busy) {
        const long long hole = sp.begin - frontier;  // <= 0 when the span starts inside covered bytes
        if (hole >= need && hole < tightest_len) {
            tightest = frontier;
            tightest_len = hole;
        }
        frontier = std::max(frontier, sp.end);
    }
    if (tightest >= 0) return tightest;                       // a hole between residents is preferred ...
    return chunk.capacity - frontier >= need ? frontier : -1;  // ... to the open room behind the last of them
}

}  // namespace

extern "C" int turbo_mem_plan(const int* first_op, const int* last_op, const long long* size, int n,
                              long long* chunk_sizes, int* n_chunks, int max_chunks, long long default_chunk_size,
                              double k_scale, int* assigned_chunk, long long* assigned_offset) {
    if (!first_op || !last_op || !size || !chunk_sizes || !n_chunks || !assigned_chunk || !assigned_offset)
        return TURBO_ERR_NULL;
    if (n <= 0 || max_chunks <= 0 || *n_chunks < 0 || *n_chunks > max_chunks || default_chunk_size <= 0 ||
        !(k_scale >= 1.0))
        return TURBO_ERR_SHAPE;
    for (int i = 0; i < n; ++i)
        if (size[i] <= 0 || first_op[i] > last_op[i]) return TURBO_ERR_SHAPE;
    for (int c = 0; c < *n_chunks; ++c)
        if (chunk_sizes[c] <= 0) return TURBO_ERR_SHAPE;

    // largest first; equal sizes keep their input order
    std::vector<int> placement_order(n);
    std::iota(placement_order.begin(), placement_order.end(), 0);
    std::stable_sort(placement_order.begin(), placement_order.end(), [&](int a, int b) { return size[a] > size[b]; });

    std::vector<Chunk> chunks(*n_chunks);
    for (int c = 0; c < *n_chunks; ++c) chunks[c].capacity = chunk_sizes[c];  // kept from earlier inferences, empty
    const Lifetimes life{first_op, last_op};
    std::vector<Span> busy;
    for (int t : placement_order) {
        int home = -1;
        long long at = -1;
        for (size_t c = 0; c < chunks.size() && home < 0; ++c) {
            at = place_in_chunk(chunks[c], t, size[t], life, size, assigned_offset, busy);
            if (at >= 0) home = (int)c;
        }
        if (home < 0) {  // nothing fits: a chunk of its own, with head room for somewhat longer requests
            const long long with_head_room = (long long)std::ceil((double)size[t] * k_scale);
            chunks.push_back(Chunk{std::max(default_chunk_size, with_head_room), {}});
            home = (int)chunks.size() - 1;
            at = 0;
        }
        chunks[home].residents.push_back(t);
        assigned_chunk[t] = home;
        assigned_offset[t] = at;
    }

    // chunks without a resident are given back; the others close ranks and the tensors follow
    std::vector<int> renumbered(chunks.size(), -1);
    int in_use = 0;
    for (size_t c = 0; c < chunks.size(); ++c)
        if (!chunks[c].residents.empty()) renumbered[c] = in_use++;
    if (in_use > max_chunks) return TURBO_ERR_SHAPE;
    for (size_t c = 0; c < chunks.size(); ++c)
        if (renumbered[c] >= 0) chunk_sizes[renumbered[c]] = chunks[c].capacity;
    for (int t = 0; t < n; ++t) assigned_chunk[t] = renumbered[assigned_chunk[t]];
    *n_chunks = in_use;
    return TURBO_OK;
}
