// The kernel planner (csrc/plan.h, host code only) under UBSan and AddressSanitizer: row lengths up to INT_MAX,
// every element size, alignment and override.  Checks the invariants the kernels rely on: the chosen shape is one
// that is compiled and it covers the row.  Prints "ok".
#include <climits>
#include <cstdio>
#include <random>

#include "../../paper_2010_05680_amd/csrc/plan.h"

using namespace turbo;

static int check(int row_len, int es, long long align, long long rows, const OpLimits& lim, const Overrides& ovr) {
    const Plan p = make_plan(row_len, es, align, rows, lim, ovr);
    char text[128];
    describe_plan(p, text, sizeof text);
    auto bad = [&](const char* what) {
        std::printf("FAILED (%s): row_len=%d es=%d align=%lld rows=%lld -> %s\n", what, row_len, es, align, rows, text);
        return 1;
    };
    if (p.vec < 1 || p.vec * es > 16 || (p.vec & (p.vec - 1))) return bad("vector width");
    if (p.under_aligned) {
        if (p.vec * es != 16 || row_len < p.vec) return bad("under-aligned mode");
    } else if (row_len % p.vec != 0 || align % p.vec != 0) {
        return bad("aligned mode on an unaligned row");
    }
    const long long nvec = ((long long)row_len + p.vec - 1) / p.vec;
    if (p.path == kPathWave) {
        if ((long long)p.lanes * p.nv < nvec || round_up_nv(p.nv) != p.nv || !wave_shape_supported(p.lanes, p.nv)) return bad("wave shape");
        // lane groups narrower than a wavefront hold several vectors per lane only in the mode without bounds checks
        if (p.lanes < 64 && p.nv > 1 && !p.full) return bad("narrow lane group with several vectors outside the exact-tiling mode");
        if (p.nv * p.vec > lim.wave_max_epl) return bad("wave registers");
    } else if (p.path == kPathBlock) {
        if (64ll * p.waves * p.nv < nvec || round_up_nv(p.nv) != p.nv || p.waves < 2 || p.waves > kBlockMaxWaves) return bad("block shape");
        {   // the register budget that decides which shapes are compiled
            const int budget = (es == 2 && p.vec * es >= 16) ? lim.block_max_epl_2byte : lim.block_max_epl;
            if (p.nv * p.vec > budget && p.nv != 1) return bad("block registers");
            if (p.vec * es < 16 && p.nv > lim.block_max_nv_narrow) return bad("narrow vectors per lane");
        }
        // shapes the softmax launcher leaves out because the planner never asks for them
        if (&lim == &kSoftmaxLimits && p.vec <= 2 && (p.nv == 5 || p.nv == 6 || p.nv == 8)) return bad("softmax block shape that is not compiled");
    } else if (p.path != kPathStream) {
        return bad("family");
    }
    if (p.full && (p.under_aligned || (p.path == kPathWave ? (long long)p.lanes * p.nv * p.vec : 64ll * p.waves * p.nv * p.vec) != row_len))
        return bad("exact tiling claimed");
    return 0;
}

int main() {
    std::mt19937_64 rng(5680);
    const int edge[] = {1, 2, 3, 4, 5, 7, 8, 63, 64, 65, 511, 512, 513, 4095, 4096, 4097, 32767, 32768, 32769, 65535, 65536,
                        1 << 20, (1 << 30) - 1, 1 << 30, INT_MAX - 16, INT_MAX - 1, INT_MAX};
    const OpLimits* limits[] = {&kSoftmaxLimits, &kLayerNormLimits};
    long long n = 0;
    for (const OpLimits* lim : limits)
        for (int es : {4, 2})
            for (long long align : {1ll, 2ll, 4ll, 8ll, 16ll})
                for (int path : {-1, 0, 1, 2})
                    for (int cap : {-1, 2, 4, 8, 16})
                    for (int block_waves : {-1, 2, 3, 5, 7, 8, 11, 16}) {
                        Overrides ovr;
                        ovr.path = path;
                        ovr.max_vec_bytes = cap;
                        ovr.block_waves = block_waves;
                        for (int no_full : {0, 1}) {
                            ovr.no_full = no_full;
                            for (int len : edge)
                                for (long long rows : {1ll, 4096ll, 2000000000ll}) {
                                    if (check(len, es, align, rows, *lim, ovr)) return 1;
                                    ++n;
                                }
                            for (int i = 0; i < 60; ++i) {
                                const int len = 1 + (int)(rng() % (i % 2 ? 70000u : 3000u));
                                if (check(len, es, align, 1 + (long long)(rng() % 100000), *lim, ovr)) return 1;
                                ++n;
                            }
                        }
                    }
    std::printf("ok %lld plans\n", n);
    return 0;
}
