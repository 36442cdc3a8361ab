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

struct Placed {
    int tensor;
    long long offset;
};

// Smallest gap of `chunk` that can hold tensor t among the tensors alive at the same time, or -1.
long long find_gap(const std::vector<Placed>& chunk, long long chunk_size, int t, const int* first_op,
                   const int* last_op, const long long* size) {
    long long smallest_gap = std::numeric_limits<long long>::max();
    long long prev_offset = 0;
    long long best_offset = -1;
    for (const Placed& x : chunk) {  // kept in increasing offset order
        const int max_first = std::max(first_op[t], first_op[x.tensor]);
        const int min_last = std::min(last_op[t], last_op[x.tensor]);
        if (max_first <= min_last) {  // life times overlap
            const long long gap = x.offset - prev_offset;
            if (gap >= size[t] && gap < smallest_gap) {
                smallest_gap = gap;
                best_offset = prev_offset;
            }
            prev_offset = std::max(prev_offset, x.offset + size[x.tensor]);
        }
    }
    if (best_offset < 0 && chunk_size - prev_offset >= size[t]) best_offset = prev_offset;
    return best_offset;
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

    std::vector<int> by_size(n);
    std::iota(by_size.begin(), by_size.end(), 0);
    std::stable_sort(by_size.begin(), by_size.end(), [&](int a, int b) { return size[a] > size[b]; });

    std::vector<long long> sizes(chunk_sizes, chunk_sizes + *n_chunks);
    std::vector<std::vector<Placed>> chunks(sizes.size());
    for (int t : by_size) {
        bool assigned = false;
        for (size_t c = 0; c < chunks.size() && !assigned; ++c) {
            const long long off = find_gap(chunks[c], sizes[c], t, first_op, last_op, size);
            if (off >= 0) {
                assigned_chunk[t] = (int)c;
                assigned_offset[t] = off;
                auto pos = std::upper_bound(chunks[c].begin(), chunks[c].end(), off,
                                            [](long long o, const Placed& p) { return o < p.offset; });
                chunks[c].insert(pos, Placed{t, off});
                assigned = true;
            }
        }
        if (!assigned) {
            const long long scaled = (long long)std::ceil((double)size[t] * k_scale);
            sizes.push_back(std::max(default_chunk_size, scaled));
            chunks.push_back({Placed{t, 0}});
            assigned_chunk[t] = (int)chunks.size() - 1;
            assigned_offset[t] = 0;
        }
    }
    // release the chunks this inference does not use and renumber the rest
    std::vector<int> new_index(chunks.size(), -1);
    int kept = 0;
    for (size_t c = 0; c < chunks.size(); ++c)
        if (!chunks[c].empty()) new_index[c] = kept++;
    if (kept > max_chunks) return TURBO_ERR_SHAPE;
    for (size_t c = 0; c < chunks.size(); ++c)
        if (new_index[c] >= 0) chunk_sizes[new_index[c]] = sizes[c];
    for (int t = 0; t < n; ++t) assigned_chunk[t] = new_index[assigned_chunk[t]];
    *n_chunks = kept;
    return TURBO_OK;
}
