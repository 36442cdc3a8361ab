// Host-side choice of kernel variant from row length, element size and alignment.
// Plain C++ (no HIP), shared by the launchers and by turbo_describe_plan().
//
// Three families, chosen by row length (the paper assigns rows to thread blocks
// and splits a block's work over warps, Section 4.1.2; here the split is chosen
// per call because the row length is shared by the whole batch):
//   wave   : an aligned group of G lanes (4..64) owns a row and keeps it in
//            registers; a wavefront works on R * (64/G) rows at once.
//   block  : a workgroup of W wavefronts owns a row; per-wavefront partial
//            results are combined through LDS with one barrier.
//   stream : a workgroup owns a row too long for registers and makes two sweeps over it; the row's first
//            128 KB wait in LDS in between, the rest is read twice.
#pragma once
#include <cstdio>

namespace turbo {

enum PathKind { kPathWave = 0, kPathBlock = 1, kPathStream = 2 };

// How a kernel treats the end of a row.
//   kModeFull   : the lanes tile the row exactly; no bounds checks at all.
//   kModeRagged : aligned vectors, lanes past the row end are masked.
//   kModeUnder  : element-aligned wide vectors; the last one overlaps its neighbour.
enum RowMode { kModeFull = 0, kModeRagged = 1, kModeUnder = 2 };

constexpr int kMaxNV = 16;                 // most vectors a lane keeps in registers
constexpr int kWaveMaxVecs = 64 * kMaxNV;  // longest row (in vectors) a single wavefront may own
constexpr int kBlockMaxWaves = 16;
#ifndef TURBO_WAVE_FAMILY_WAVES
#define TURBO_WAVE_FAMILY_WAVES 4
#endif
constexpr int kWaveFamilyWaves = TURBO_WAVE_FAMILY_WAVES;  // wavefronts per workgroup in the wave family
constexpr int kStreamThreads = 1024;

// Register budgets, in row elements held per lane, that bound each family.
struct OpLimits {
    int target_elems;    // wave: rows in flight are chosen so a lane holds about this many values
    int wave_max_epl;    // wave: most elements of one row per lane
    int block_pref_nv;   // block: grow the workgroup until a lane holds at most this many vectors
    int block_max_epl;   // block: most elements per lane (1024 threads leave 128 VGPRs each)
    int block_from_bytes;  // rows of at least this many bytes go to the block family even if a wavefront could hold them
    int block_max_nv_narrow;  // block: most vectors per lane when a vector is narrower than 16 bytes (every vector
                              // costs address registers, whatever its width)
    int block_max_epl_2byte;  // block: most elements per lane for 16-byte vectors of 2-byte elements (their loads take
                              // half the registers)
    int block_wide_from_16ths;  // block: 16 wavefronts x 2 vectors replace fewer wavefronts x >= 3 vectors once they
                                // would use at least this many 16ths of their lanes; 0 = never (measured per operation)
    int block_wide_from_16ths_2byte;  // the same for 2-byte elements
    int target_elems_under;  // the same for rows reached with element-aligned accesses (under-aligned mode)
    int block_exact_first;  // block: 1 = prefer a workgroup of 2..8 wavefronts x 3 or 2 vectors that tiles the row exactly
};
#ifndef TURBO_SM_TARGET_ELEMS
#define TURBO_SM_TARGET_ELEMS 32
#endif
// Element-aligned 16-byte accesses stream better with fewer of them in flight: measured +2-5 points of HBM peak for
// every under-aligned softmax shape of the wave family, both element types, with or without an additive mask.
#ifndef TURBO_SM_TARGET_ELEMS_UNDER
#define TURBO_SM_TARGET_ELEMS_UNDER 16
#endif
#ifndef TURBO_LN_TARGET_ELEMS
#define TURBO_LN_TARGET_ELEMS 16
#endif
#ifndef TURBO_SM_BLOCK_PREF_NV
#define TURBO_SM_BLOCK_PREF_NV 2
#endif
#ifndef TURBO_LN_BLOCK_PREF_NV
#define TURBO_LN_BLOCK_PREF_NV 2
#endif
#ifndef TURBO_SM_BLOCK_FROM_BYTES
#define TURBO_SM_BLOCK_FROM_BYTES 4096
#endif
#ifndef TURBO_LN_BLOCK_FROM_BYTES
#define TURBO_LN_BLOCK_FROM_BYTES 4608  // rows of 1152 floats and more (5 vectors per lane in the wave family): +3 points
#endif
constexpr OpLimits kSoftmaxLimits{TURBO_SM_TARGET_ELEMS, 64, TURBO_SM_BLOCK_PREF_NV, 32, TURBO_SM_BLOCK_FROM_BYTES, 16, 32, 12, 14, TURBO_SM_TARGET_ELEMS_UNDER, 0};
constexpr OpLimits kLayerNormLimits{TURBO_LN_TARGET_ELEMS, 24, TURBO_LN_BLOCK_PREF_NV, 16, TURBO_LN_BLOCK_FROM_BYTES, 6, 24, 0, 0, TURBO_LN_TARGET_ELEMS, 1};

struct Plan {
    int path;    // PathKind
    int vec;     // elements per load/store
    int under_aligned;  // 1: accesses are `vec` wide but only element-aligned; the row's last vector is
                        //    shifted back to end at the row end and overlaps its neighbour
    int full;           // 1: lanes * nv * vec (times waves for the block family) equals the row length exactly,
                        //    so no lane needs a bounds check
    int lanes;   // wave: lanes per row (G)
    int nv;      // vectors per lane
    int rows;    // wave: rows a lane group works on concurrently (R)
    int waves;   // block: wavefronts per row (W)
};

struct Overrides {
    int path = -1;
    int max_vec_bytes = -1;
    int grid_waves = -1;
    int grid_blocks = -1;  // > 0: exact grid of the looping kernels
    int no_full = 0;    // 1: the call needs per-row bounds checks (per-request lengths), never the exact-tiling mode
    int no_stream = 0;  // 1: the call cannot use the two-sweep family
    int block_waves = -1;  // 2..16: wavefronts per row in the block family, when the row then fits the register budget
};

inline int round_up_nv(int nv) {
    static const int supported[] = {1, 2, 3, 4, 5, 6, 8, 12, 16};
    for (int s : supported)
        if (nv <= s) return s;
    return -1;
}

// (lanes per row, vectors per lane) pairs the wave family is compiled for.
inline bool wave_shape_supported(int lanes, int nv) {
    if (lanes == 64) return round_up_nv(nv) == nv;
    if (nv == 1) return lanes == 4 || lanes == 8 || lanes == 16 || lanes == 32;
    return (lanes == 32 && (nv == 3 || nv == 5)) || (lanes == 16 && nv == 3);
}

inline int pow2_ceil(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

// Rows in flight per lane group so that a lane holds about `target_elems` values.
inline int rows_in_flight(int nv, int vec, int target_elems) {
    int r = target_elems / (nv * vec);
    if (r >= 8) return 8;
    if (r >= 4) return 4;
    if (r >= 2) return 2;
    return 1;
}

// align_elems: largest power of two (in elements) to which every base pointer and
// every row start is aligned; the vector width never exceeds it.
inline Plan make_plan(int row_len, int elem_size, long long align_elems, long long n_rows, const OpLimits& lim,
                      const Overrides& ovr) {
    Plan p{};
    int vec_bytes = 16;
    if (ovr.max_vec_bytes >= elem_size && ovr.max_vec_bytes < 16) vec_bytes = ovr.max_vec_bytes;
    int vec = vec_bytes / elem_size;
    p.under_aligned = 0;
    if (row_len % vec != 0 || align_elems % vec != 0) {
        if (row_len >= vec && vec > 1 && ovr.max_vec_bytes < 0) {
            p.under_aligned = 1;  // keep the full width; hardware handles element-aligned wide accesses
        } else {
            while (vec > 1 && (row_len % vec != 0 || align_elems % vec != 0)) vec >>= 1;
        }
    }
    p.vec = vec;
    const long long nvec = ((long long)row_len + vec - 1) / vec;

    // wave family: feasible when one wavefront's registers hold the row
    bool wave_ok = false;
    int wave_g = 0, wave_nv = 0;
    if (nvec <= kWaveMaxVecs) {
        int g = pow2_ceil((int)nvec);
        if (g < 4) g = 4;
        if (g > 64) g = 64;
        int nv = round_up_nv((int)((nvec + g - 1) / g));
        if (nv > 0 && nv * vec <= lim.wave_max_epl) {
            wave_ok = true;
            wave_g = g;
            wave_nv = nv;
        }
        // Prefer a lane group that tiles the row exactly (no masked lanes, constant merge weights),
        // e.g. 96 vectors = 32 lanes x 3 rather than 64 lanes x 2 with a quarter of them idle.
        // (those shapes exist only in the mode without bounds checks, which per-row key counts rule out)
        if (!p.under_aligned && !ovr.no_full && (long long)g * nv * vec != row_len) {
            for (int gg = 64; gg >= 4; gg >>= 1) {
                if (nvec % gg != 0) continue;
                int q = (int)(nvec / gg);
                if (q > kMaxNV || !wave_shape_supported(gg, q) || q * vec > lim.wave_max_epl) continue;
                wave_ok = true;
                wave_g = gg;
                wave_nv = q;
                break;
            }
        }
    }
    // block family: the smallest workgroup of at most 8 wavefronts whose lanes hold at most the preferred
    // number of vectors; failing that, up to twice as many vectors with up to 16 wavefronts; failing that,
    // 16 wavefronts with whatever still fits the register budget.
    bool block_ok = false;
    int block_w = 0, block_nv = 0;
    const int block_max_epl = (elem_size == 2 && vec * elem_size >= 16) ? lim.block_max_epl_2byte : lim.block_max_epl;
    auto block_fits = [&](int nv) {
        return (nv * vec <= block_max_epl || nv == 1) && (vec * elem_size >= 16 || nv <= lim.block_max_nv_narrow);
    };
    // Measured for the LayerNorm: a workgroup that tiles the row exactly with 3 or 2 vectors per lane (any number of
    // wavefronts up to 8, e.g. 3 x 3 for 576 vectors, 5 x 2 for 640) beats a larger power-of-two workgroup with idle
    // lanes and bounds checks by up to 12 points.  Workgroups of 5..7 wavefronts that need bounds checks measured
    // worse than 8, so they are taken for exact tilings only.
    if (lim.block_exact_first && !p.under_aligned && !ovr.no_full && vec * elem_size >= 16) {
        for (int nv = 3; nv >= 2 && !block_ok; --nv) {
            if (nvec % (64 * nv) != 0 || !block_fits(nv)) continue;
            const long long w = nvec / (64 * nv);
            // (5..7 wavefronts x 2 vectors: 1-8 points over the next power of two for 2-byte elements, 2-3 for 4-byte ones)
            if (w >= 2 && w <= 8) {
                block_ok = true;
                block_w = (int)w;
                block_nv = nv;
            }
        }
    }
    for (int pass = 0; pass < 3 && !block_ok; ++pass) {
        const int max_w = pass == 0 ? 8 : kBlockMaxWaves;
        const int max_nv = pass == 0 ? lim.block_pref_nv : pass == 1 ? 2 * lim.block_pref_nv : kMaxNV;
        // 2, 3, 4, 8, 16 wavefronts: three serve rows of 257..384 vectors with a quarter fewer idle lanes than four
        for (int w = 2; w <= max_w; w = w == 2 ? 3 : w == 3 ? 4 : 2 * w) {
            long long per_lane = (nvec + 64 * w - 1) / (64 * w);
            if (per_lane > kMaxNV) continue;
            int nv = round_up_nv((int)per_lane);
            const bool fits = block_fits(nv);
            if (fits && nv <= max_nv) {
                block_ok = true;
                block_w = w;
                block_nv = nv;
                break;
            }
        }
    }
    // Rows of 513..704 vectors leave 8 wavefronts x 2 vectors at most 11/16 busy; 4 wavefronts x 3 vectors measured
    // 4-8 points faster there (softmax), and no slower for the LayerNorm.
    if (block_ok && block_w == 8 && block_nv == 2 && nvec <= 704 && vec * elem_size >= 16 && block_fits(3)) {
        block_w = 4;
        block_nv = 3;
    }
    // Rows of 257..384 vectors: 2 wavefronts x 3 vectors cover the same 384 slots as 3 x 2 with one wavefront less at the
    // barrier; measured equal for 4-byte elements and 1.5-3 points faster for 2-byte ones (LayerNorm only: its budget
    // holds 3 vectors per lane, and the softmax reaches such rows in its wave family).
    if (lim.block_exact_first && block_ok && block_w == 3 && block_nv == 2 && vec * elem_size >= 16 && block_fits(3) &&
        nvec % (64 * 3 * 2) != 0) {
        block_w = 2;
        block_nv = 3;
    }
    // (16-byte vectors only: with narrower ones not every count of vectors per lane is compiled)
    if (ovr.block_waves >= 2 && ovr.block_waves <= kBlockMaxWaves && vec * elem_size >= 16) {
        const int w = ovr.block_waves;
        const long long per_lane = (nvec + 64 * w - 1) / (64 * w);
        const int nv = per_lane <= kMaxNV ? round_up_nv((int)per_lane) : -1;
        if (nv > 0 && block_fits(nv)) {
            block_ok = true;
            block_w = w;
            block_nv = nv;
        }
    }
    // Measured for the softmax: a workgroup of 16 wavefronts with 2 vectors per lane streams better than 8 with
    // 3 or 4, provided enough of its lanes have work (rows of 1536..2048 vectors of binary32, 1792..2048 of binary16;
    // below that the idle lanes cost more than the shape gains).
    const int wide_from = elem_size == 2 ? lim.block_wide_from_16ths_2byte : lim.block_wide_from_16ths;
    if (block_ok && ovr.block_waves < 2 && wide_from > 0 && block_w < kBlockMaxWaves && block_nv >= 3 &&
        nvec <= 2LL * 64 * kBlockMaxWaves && 16 * nvec >= (long long)wide_from * 2 * 64 * kBlockMaxWaves &&
        2 * vec <= block_max_epl && vec * elem_size >= 16) {
        block_w = kBlockMaxWaves;
        block_nv = 2;
    }

    int path;
    if (wave_ok) {
        // Long rows with few of them: a workgroup per row exposes more parallelism.
        path = (block_ok && ((long long)row_len * elem_size >= lim.block_from_bytes || (nvec >= 512 && n_rows < 4096))) ? kPathBlock : kPathWave;
    } else {
        path = block_ok ? kPathBlock : kPathStream;
    }
    if (ovr.path == kPathWave && wave_ok) path = kPathWave;
    if (ovr.path == kPathBlock && block_ok) path = kPathBlock;
    if (ovr.path == kPathStream) path = kPathStream;
    if (path == kPathStream && p.under_aligned) {
        // the two-sweep kernels only take aligned vectors: narrow the access instead
        p.under_aligned = 0;
        while (vec > 1 && (row_len % vec != 0 || align_elems % vec != 0)) vec >>= 1;
        p.vec = vec;
    }
    p.path = path;

    if (path == kPathWave) {
        p.lanes = wave_g;
        p.nv = wave_nv;
        p.rows = rows_in_flight(p.nv, vec, (p.under_aligned && !ovr.no_full) ? lim.target_elems_under : lim.target_elems);
        p.waves = 4;
    } else if (path == kPathBlock) {
        p.waves = block_w;
        p.lanes = 64;
        p.nv = block_nv;
        p.rows = 1;
    } else {
        p.waves = kStreamThreads / 64;
        p.lanes = 64;
        p.nv = 1;
        p.rows = 1;
    }
    p.full = 0;
    if (ovr.no_full) return p;
    if (!p.under_aligned && path == kPathWave) p.full = (long long)p.lanes * p.nv * vec == row_len;
    if (!p.under_aligned && path == kPathBlock) p.full = 64ll * p.waves * p.nv * vec == row_len;
    return p;
}

inline int row_mode(const Plan& p) { return p.under_aligned ? kModeUnder : p.full ? kModeFull : kModeRagged; }

inline void describe_plan(const Plan& p, char* buf, int n) {
    static const char* names[] = {"wave", "block", "stream"};
    const char* ua = p.under_aligned ? "u" : p.full ? "f" : "";
    if (p.path == kPathWave)
        std::snprintf(buf, n, "%s vec=%d%s lanes=%d nv=%d rows=%d", names[p.path], p.vec, ua, p.lanes, p.nv, p.rows);
    else
        std::snprintf(buf, n, "%s vec=%d%s waves=%d nv=%d", names[p.path], p.vec, ua, p.waves, p.nv);
}

}  // namespace turbo
