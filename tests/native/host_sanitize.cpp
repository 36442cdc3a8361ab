// Host-side planning routines under AddressSanitizer and UBSan: random instances, including ones that must be
// rejected, with the output arrays sized exactly as the header says.  Prints "ok" when every call returned and the
// plans satisfy their contract; any out-of-bounds access aborts the program through the sanitizers.
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "../../include/turbo_reduce.h"
#include "../../include/turbo_serving.h"

static int fail(const char* what) {
    std::printf("FAILED: %s\n", what);
    return 1;
}

int main() {
    std::mt19937 rng(20100568);
    auto uni = [&](int lo, int hi) { return std::uniform_int_distribution<int>(lo, hi)(rng); };

    for (int it = 0; it < 300; ++it) {  // cost table + scheduler
        const int n_len = uni(1, 5), n_batch = uni(1, 4), max_len = uni(1, 120), max_batch = uni(1, 12);
        std::vector<int> sl(n_len), sb(n_batch);
        int v = 0;
        for (int& x : sl) x = (v += uni(1, 40));
        v = 0;
        for (int& x : sb) x = (v += uni(1, 5));
        std::vector<double> samples((size_t)n_len * n_batch);
        for (double& c : samples) c = 0.5 + uni(0, 1000) / 100.0;
        std::vector<double> table((size_t)(max_len + 1) * (max_batch + 1), -1.0);
        if (turbo_cost_table_fill(sl.data(), n_len, sb.data(), n_batch, samples.data(), max_len, max_batch, table.data()) != TURBO_OK)
            return fail("cost table");
        for (double c : table)
            if (!(c >= 0.0)) return fail("cost table entry");
        const int n = uni(1, 40);
        std::vector<int> lengths(n), order(n), ends(n);
        for (int& x : lengths) x = uni(1, max_len);
        int nb = 0;
        double total = 0;
        if (turbo_batch_schedule(lengths.data(), n, table.data(), max_len, max_batch, order.data(), ends.data(), &nb, &total) != TURBO_OK)
            return fail("schedule");
        if (nb < 1 || nb > n || ends[nb - 1] != n) return fail("schedule shape");
        for (int k = 0, begin = 0; k < nb; begin = ends[k++])
            if (ends[k] <= begin || ends[k] - begin > max_batch) return fail("batch size");
        lengths[uni(0, n - 1)] = max_len + 1;  // must be rejected, not read past the table
        if (turbo_batch_schedule(lengths.data(), n, table.data(), max_len, max_batch, order.data(), ends.data(), &nb, &total) != TURBO_ERR_SHAPE)
            return fail("schedule accepted a length beyond the table");
    }

    for (int it = 0; it < 300; ++it) {  // allocator
        const int n = uni(1, 60), n_ops = uni(1, 30);
        std::vector<int> first(n), last(n), chunk(n);
        std::vector<long long> size(n), offset(n);
        for (int i = 0; i < n; ++i) {
            first[i] = uni(0, n_ops - 1);
            last[i] = std::min(n_ops - 1, first[i] + uni(0, 6));
            size[i] = (long long)uni(1, 5000) * (uni(0, 2) == 0 ? 1024 : 1);
        }
        const int held = uni(0, 3);
        const int max_chunks = held + uni(0, n + 1);  // sometimes too few: the call must say so, not overrun chunk_sizes
        std::vector<long long> chunks(max_chunks > 0 ? max_chunks : 1);
        for (int c = 0; c < held && c < max_chunks; ++c) chunks[c] = (long long)uni(1, 4) * 4096;
        int n_chunks = std::min(held, max_chunks);
        const int st = turbo_mem_plan(first.data(), last.data(), size.data(), n, chunks.data(), &n_chunks, max_chunks,
                                      uni(0, 1) ? 4096 : (2 << 20), 1.2, chunk.data(), offset.data());
        if (st == TURBO_ERR_SHAPE) continue;  // not enough room for the chunks this instance needs
        if (st != TURBO_OK) return fail("mem plan status");
        if (n_chunks < 0 || n_chunks > max_chunks) return fail("chunk count");
        for (int i = 0; i < n; ++i) {
            if (chunk[i] < 0 || chunk[i] >= n_chunks || offset[i] < 0 || offset[i] + size[i] > chunks[chunk[i]])
                return fail("tensor outside its chunk");
            for (int j = 0; j < i; ++j) {
                const bool alive_together = std::max(first[i], first[j]) <= std::min(last[i], last[j]);
                const bool share_bytes = chunk[i] == chunk[j] && offset[i] < offset[j] + size[j] && offset[j] < offset[i] + size[i];
                if (alive_together && share_bytes) return fail("tensors alive together share bytes");
            }
        }
    }
    std::printf("ok\n");
    return 0;
}
