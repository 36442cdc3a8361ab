// Fused bias + residual + LayerNorm kernels for gfx950 (wave64).
//
// Operation (Section 4.1.2, Equation 1, and the "AddBiasLayerNorm" kernel of
// Section 6.2.1): t = x + bias + residual; per row the mean and the population
// variance of t; out = (t - mean) / sqrt(var + eps) * gamma + beta.
//
// The paper reduces sum(x) and sum(x^2) together so that one synchronisation
// yields both statistics.  The same "one exchange chain for both statistics"
// holds here, but the pair that travels is the Welford state (mean, M2) merged
// with Chan's rule: it is one pass as well and does not cancel when |mean| >> std.
// The element counts behind each merge depend only on the lane and the row
// length, so the merge weights are computed once per kernel, not per row.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

#include "device_utils.h"
#include "plan.h"
#include "softmax_kernels.h"  // LaunchCfg, capped_grid, rows_in_flight_c

namespace turbo {

#ifndef TURBO_LN_PRELOAD_ELEMS
#define TURBO_LN_PRELOAD_ELEMS 16
#endif
constexpr int kParamPreloadElems = TURBO_LN_PRELOAD_ELEMS;     // keep bias/gamma/beta in registers up to this many columns per lane
// The block family runs with 128 registers per lane (1024-thread workgroups) and also holds the next row's loads:
// at 16 columns per lane the three parameter vectors no longer fit beside them unless the row mode is the one
// without bounds checks.
#ifndef TURBO_LN_BLOCK_PRELOAD_ELEMS
#define TURBO_LN_BLOCK_PRELOAD_ELEMS 12
#endif
#ifndef TURBO_LN_BLOCK_PRELOAD_FULL_ELEMS
#define TURBO_LN_BLOCK_PRELOAD_FULL_ELEMS 16
#endif
constexpr int kBlockParamPreloadElems = TURBO_LN_BLOCK_PRELOAD_ELEMS;
constexpr int kBlockParamPreloadFullElems = TURBO_LN_BLOCK_PRELOAD_FULL_ELEMS;
#ifndef TURBO_LN_BLOCK_PRELOAD_HALF_ELEMS
#define TURBO_LN_BLOCK_PRELOAD_HALF_ELEMS 24
#endif
constexpr int kBlockParamPreloadHalfElems = TURBO_LN_BLOCK_PRELOAD_HALF_ELEMS;  // 16-byte vectors of 2-byte elements

struct LayerNormArgs {
    const void* x;
    const void* residual;  // may be null
    const void* bias;      // may be null
    const void* gamma;
    const void* beta;
    void* out;
    int n_rows;
    int hidden;
    float eps;
    float inv_hidden;
    // Length-aware mode for zero-padded batches: rows are (b, s) with s < S; rows with s >= lengths[b] are
    // padding and are neither read nor written.  lengths == nullptr: every row is processed.
    const int* lengths;
    int S;
    FastDiv div_s;
};

// Whether `row` is a padding row in length-aware mode.
__device__ __forceinline__ bool is_padding_row(const LayerNormArgs& a, int row) {
    if (a.lengths == nullptr) return false;
    const unsigned b = fastdiv((unsigned)row, a.div_s);
    const int s = (int)((unsigned)row - b * (unsigned)a.S);
    return s >= a.lengths[b];
}

constexpr int log2_c(int g) { return g <= 1 ? 0 : 1 + log2_c(g / 2); }

// Weights of the Chan merges along the exchange chain S = 1, 2, ..., G/2 for a
// lane that holds `cnt` valid elements: after the call w1[i] = n_b/(n_a+n_b) and
// w2[i] = n_a*n_b/(n_a+n_b) for step i, and the return value is the group total.
template <int S, int G, int I, int N>
__device__ __forceinline__ void merge_weights_step(float& n, float (&w1)[N], float (&w2)[N]) {
    if constexpr (S < G) {
        float na, nb;
        exchange<S>(n, na, nb);
        float nt = na + nb;
        float inv = nt > 0.f ? fast_rcp(nt) : 0.f;  // counts are small integers; 1 ulp on a weight is harmless
        w1[I] = nb * inv;
        w2[I] = na * nb * inv;
        n = nt;
        merge_weights_step<S * 2, G, I + 1, N>(n, w1, w2);
    }
}

// The same weights when every lane holds exactly `cnt` elements: n_a = n_b = cnt * 2^i at step i.
template <int N>
__device__ __forceinline__ void merge_weights_full(float cnt, float (&w1)[N], float (&w2)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
        w1[i] = 0.5f;
        w2[i] = cnt * (float)(1 << i) * 0.5f;
    }
}

template <int S, int G, int I, int R, int N>
__device__ __forceinline__ void merge_stats_step(float (&mean)[R], float (&m2)[R], const float (&w1)[N],
                                                 const float (&w2)[N]) {
    if constexpr (S < G) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float ma, mb, qa, qb;
            exchange<S>(mean[r], ma, mb);
            exchange<S>(m2[r], qa, qb);
            float d = mb - ma;
            mean[r] = fmaf(d, w1[I], ma);
            m2[r] = fmaf(d * d, w2[I], qa + qb);
        }
        merge_stats_step<S * 2, G, I + 1, R, N>(mean, m2, w1, w2);
    }
}

// One parameter vector widened to float.  `col` must be a readable column (callers
// clamp columns past the row end to 0; what those lanes hold is never used).
template <typename T, int VEC, bool UA = false>
__device__ __forceinline__ void load_param(const T* p, int col, float (&dst)[VEC]) {
    Pack<T, VEC> raw = load_pack<T, VEC, UA>(p + col);
#pragma unroll
    for (int j = 0; j < VEC; ++j) dst[j] = (float)raw.v[j];
}
// Tells the compiler that a packed register set may have changed (it has not): placed at the top of a loop
// iteration it keeps the widening conversions of 2-byte parameters inside the loop, i.e. the parameters stay packed
// in half the registers across iterations instead of being widened once and held in full width.
template <typename T, int VEC>
__device__ __forceinline__ void keep_packed(Pack<T, VEC>& p) {
    if constexpr (sizeof(T) == 2 && VEC % 2 == 0) {
        struct Words { unsigned w[VEC / 2]; };
        Words x = __builtin_bit_cast(Words, p);
#pragma unroll
        for (int i = 0; i < VEC / 2; ++i) asm volatile("" : "+v"(x.w[i]));
        p = __builtin_bit_cast(Pack<T, VEC>, x);
    }
}

// The bias may be absent: a null pointer reads as zeros (wave-uniform branch).
template <typename T, int VEC, bool UA = false>
__device__ __forceinline__ void load_bias(const T* p, int col, float (&dst)[VEC]) {
    if (p != nullptr) {
        load_param<T, VEC, UA>(p, col, dst);
    } else {
#pragma unroll
        for (int j = 0; j < VEC; ++j) dst[j] = 0.f;
    }
}

// ---------------------------------------------------------------------------
// wave family: G lanes per row, NV vectors per lane, R rows per lane group, one
// tile of rows per workgroup.  The loads of the tile are issued first; the
// set-up (merge weights, parameter vectors) runs while they are in flight.
// Measured on MI355X, short-lived workgroups stream better here than
// persistent ones that keep the parameters across tiles.
// ---------------------------------------------------------------------------
template <typename T, int VEC, int G, int NV, bool RES, int MODE, bool VARLEN>
__global__ __launch_bounds__(64 * kWaveFamilyWaves) void layernorm_wave_kernel(LayerNormArgs a, int n_tiles) {
    constexpr bool UA = MODE == kModeUnder;
    constexpr bool FULL = MODE == kModeFull;
    constexpr int R = rows_in_flight_c(NV, VEC, kLayerNormLimits.target_elems);
    constexpr int GPW = kWave / G;
    constexpr int kWaves = kWaveFamilyWaves;
    constexpr int TILE_ROWS = R * GPW * kWaves;
    constexpr int STEPS = log2_c(G) > 0 ? log2_c(G) : 1;
    constexpr bool PRELOAD = NV * VEC <= kParamPreloadElems;

    const T* __restrict__ x = reinterpret_cast<const T*>(a.x);
    const T* __restrict__ res = reinterpret_cast<const T*>(a.residual);
    const T* __restrict__ bias = reinterpret_cast<const T*>(a.bias);
    const T* __restrict__ gamma = reinterpret_cast<const T*>(a.gamma);
    const T* __restrict__ beta = reinterpret_cast<const T*>(a.beta);
    T* out = reinterpret_cast<T*>(a.out);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int gl = lane % G;
    const int grp = lane / G;
    const int hidden = a.hidden;

    const int tile = blockIdx.x;
    if (tile >= n_tiles) return;

    Pack<T, VEC> xr[R][NV];
    Pack<T, VEC> rr[R][NV];
    bool live[R];  // the row exists and is not padding: only live rows are stored
    auto issue_loads = [&](int tl) {
        const int row_base = tl * TILE_ROWS + wave * (R * GPW) + grp;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            int row = row_base + r * GPW;
            live[r] = row < a.n_rows;
            if constexpr (VARLEN) live[r] = live[r] && !is_padding_row(a, row);
            int rowc = live[r] ? row : (VARLEN ? 0 : a.n_rows - 1);  // other rows recompute a valid row, unstored
            const long long off = (long long)rowc * hidden;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                int colc = FULL ? (v * G + gl) * VEC : vec_start<VEC, UA>((v * G + gl) * VEC, hidden);
                xr[r][v] = load_stream<T, VEC, UA>(x + off + colc);
                if constexpr (RES) rr[r][v] = load_stream<T, VEC, UA>(res + off + colc);
            }
        }
    };
    if constexpr (VARLEN) {  // a wavefront whose rows are all padding issues no memory traffic
        bool any_row = false;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int row = tile * TILE_ROWS + wave * (R * GPW) + grp + r * GPW;
            any_row = any_row || (row < a.n_rows && !is_padding_row(a, row));
        }
        if (__ballot(any_row) == 0) return;
    }
    issue_loads(tile);

    float pb[PRELOAD ? NV : 1][VEC], pg[PRELOAD ? NV : 1][VEC], pe[PRELOAD ? NV : 1][VEC];
    if constexpr (PRELOAD) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int col = (v * G + gl) * VEC;
            int colc = FULL ? col : vec_start<VEC, UA>(col, hidden);
            load_bias<T, VEC, UA>(bias, colc, pb[v]);
            load_param<T, VEC, UA>(gamma, colc, pg[v]);
            load_param<T, VEC, UA>(beta, colc, pe[v]);
        }
    }

    float cnt = (float)(NV * VEC);
    float w1[STEPS], w2[STEPS];
    if constexpr (FULL) {
        merge_weights_full<STEPS>(cnt, w1, w2);
    } else {
        cnt = 0.f;
#pragma unroll
        for (int v = 0; v < NV; ++v)
            if ((v * G + gl) * VEC < hidden) cnt += (float)(VEC - vec_overlap<VEC, UA>((v * G + gl) * VEC, hidden));
        float n = cnt;
        merge_weights_step<1, G, 0, STEPS>(n, w1, w2);
    }
    const float inv_cnt = cnt > 0.f ? fast_rcp(cnt) : 0.f;

    {
        const int row_base = tile * TILE_ROWS + wave * (R * GPW) + grp;
        float t[R][NV][VEC];
        float mean[R], m2[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float sum = 0.f;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                int col = (v * G + gl) * VEC;
                const bool ok = FULL || col < hidden;
                const int dup = vec_overlap<VEC, UA>(col, hidden);
                float b[VEC];
                if constexpr (PRELOAD) {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) b[j] = pb[v][j];
                } else {
                    load_bias<T, VEC, UA>(bias, FULL ? col : vec_start<VEC, UA>(col, hidden), b);
                }
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    float tv = (float)xr[r][v].v[j] + b[j];
                    if constexpr (RES) tv += (float)rr[r][v].v[j];
                    tv = ok ? tv : 0.f;
                    t[r][v][j] = tv;
                    sum += (UA && j < dup) ? 0.f : tv;  // overlapped elements are counted by the neighbouring vector
                }
            }
            const float mu = sum * inv_cnt;
            float q = 0.f;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const bool ok = FULL || (v * G + gl) * VEC < hidden;
                const int dup = vec_overlap<VEC, UA>((v * G + gl) * VEC, hidden);
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    float d = t[r][v][j] - mu;
                    q += (ok && !(UA && j < dup)) ? d * d : 0.f;
                }
            }
            mean[r] = mu;
            m2[r] = q;
        }
        merge_stats_step<1, G, 0, R, STEPS>(mean, m2, w1, w2);

#pragma unroll
        for (int r = 0; r < R; ++r) {
            int row = row_base + r * GPW;
            const float rstd = fast_rsqrt(fmaf(m2[r], a.inv_hidden, a.eps));
            T* op = out + (long long)row * hidden;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                int col = (v * G + gl) * VEC;
                if (live[r] && (FULL || col < hidden)) {
                    const int colc = FULL ? col : vec_start<VEC, UA>(col, hidden);
                    float g[VEC], be[VEC];
                    if constexpr (PRELOAD) {
#pragma unroll
                        for (int j = 0; j < VEC; ++j) {
                            g[j] = pg[v][j];
                            be[j] = pe[v][j];
                        }
                    } else {
                        load_param<T, VEC, UA>(gamma, colc, g);
                        load_param<T, VEC, UA>(beta, colc, be);
                    }
                    Pack<T, VEC> o;
#pragma unroll
                    for (int j = 0; j < VEC; ++j) o.v[j] = (T)fmaf((t[r][v][j] - mean[r]) * rstd, g[j], be[j]);
                    store_stream<T, VEC, UA>(op + colc, o);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Cross-wavefront combine of (count, mean, M2) through LDS, one barrier per row.
// ---------------------------------------------------------------------------
struct LayerNormLds {
    float n[2][kBlockMaxWaves];
    float mean[2][kBlockMaxWaves];
    float m2[2][kBlockMaxWaves];
};

__device__ __forceinline__ void layernorm_block_combine(LayerNormLds& lds, int slot, int wave, int lane, int n_waves,
                                                        float n_w, float& mean, float& m2) {
    if (lane == 0) {
        lds.n[slot][wave] = n_w;
        lds.mean[slot][wave] = mean;
        lds.m2[slot][wave] = m2;
    }
    __syncthreads();
    float n = 0.f, mu = 0.f, q = 0.f;
    for (int w = 0; w < n_waves; ++w) {
        float nb = lds.n[slot][w];
        float nt = n + nb;
        float inv = fast_rcp(fmaxf(nt, 1.f));
        float d = lds.mean[slot][w] - mu;
        mu = fmaf(d, nb * inv, mu);
        q = fmaf(d * d, n * nb * inv, q + lds.m2[slot][w]);
        n = nt;
    }
    mean = mu;
    m2 = q;
}

// block family: a workgroup of blockDim.x/64 wavefronts per row, NV vectors per lane.
// Rotated like the wave family: the next row's loads are issued before this
// row's barrier and stores.
// Whether a workgroup of up to 16 wavefronts (128 registers per lane) can keep bias/gamma/beta in registers beside the
// current and the prefetched row.  16-byte vectors of 2-byte elements hold their prefetched row in half the registers:
// they fit like the mode without bounds checks does.
template <typename T, int VEC, int NV, int MODE>
constexpr bool block_params_fit_128() {
    return NV * VEC <= ((sizeof(T) == 2 && VEC == 8)
                            ? (MODE == kModeFull ? kBlockParamPreloadHalfElems : kBlockParamPreloadFullElems)
                            : MODE == kModeFull ? kBlockParamPreloadFullElems : kBlockParamPreloadElems);
}

// ROOMY: the kernel is built for workgroups of at most 8 wavefronts, which leaves every lane up to 256 registers, and
// keeps the parameters in registers whatever the shape; used for the shapes whose parameters do not fit 128 registers
// (they would be re-read from the vector cache for every row: three more vector loads per slot and row on the path the
// streams need) whenever the row is served by 8 wavefronts or fewer.
template <typename T, int VEC, int NV, bool RES, int MODE, bool ROOMY = false>
__global__ __launch_bounds__(ROOMY ? 512 : 1024) void layernorm_block_kernel(LayerNormArgs a) {
    constexpr bool UA = MODE == kModeUnder;
    constexpr bool FULL = MODE == kModeFull;
    __shared__ LayerNormLds lds;
    constexpr bool PRELOAD = ROOMY || block_params_fit_128<T, VEC, NV, MODE>();
    const T* __restrict__ x = reinterpret_cast<const T*>(a.x);
    const T* __restrict__ res = reinterpret_cast<const T*>(a.residual);
    const T* __restrict__ bias = reinterpret_cast<const T*>(a.bias);
    const T* __restrict__ gamma = reinterpret_cast<const T*>(a.gamma);
    const T* __restrict__ beta = reinterpret_cast<const T*>(a.beta);
    T* out = reinterpret_cast<T*>(a.out);
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int n_waves = blockDim.x >> 6;
    const int hidden = a.hidden;
    const int bd = (int)blockDim.x;

    // rows of this workgroup: blockIdx.x, + gridDim.x, ... without the padding rows of length-aware mode
    auto next_live_row = [&](int rw) {
        while (rw < a.n_rows && is_padding_row(a, rw)) rw += (int)gridDim.x;
        return rw;
    };
    int row = next_live_row(blockIdx.x);
    if (row >= a.n_rows) return;

    Pack<T, VEC> xr[NV];
    Pack<T, VEC> rr[NV];
    auto issue_loads = [&](int rw) {
        const long long off = (long long)rw * hidden;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int colc = FULL ? (v * bd + tid) * VEC : vec_start<VEC, UA>((v * bd + tid) * VEC, hidden);
            xr[v] = load_stream<T, VEC, UA>(x + off + colc);
            if constexpr (RES) rr[v] = load_stream<T, VEC, UA>(res + off + colc);
        }
    };
    issue_loads(row);

    // kept in the storage type (2-byte elements take half the registers) and widened where they are used
    Pack<T, VEC> pb[PRELOAD ? NV : 1], pg[PRELOAD ? NV : 1], pe[PRELOAD ? NV : 1];
    if constexpr (PRELOAD) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int col = (v * bd + tid) * VEC;
            int colc = FULL ? col : vec_start<VEC, UA>(col, hidden);
            if (bias != nullptr) {
                pb[v] = load_pack<T, VEC, UA>(bias + colc);
            } else {
#pragma unroll
                for (int j = 0; j < VEC; ++j) pb[v].v[j] = (T)0.f;
            }
            pg[v] = load_pack<T, VEC, UA>(gamma + colc);
            pe[v] = load_pack<T, VEC, UA>(beta + colc);
        }
    }

    float cnt = (float)(NV * VEC);
    float w1[6], w2[6];
    float n_w = cnt * (float)kWave;
    if constexpr (FULL) {
        merge_weights_full<6>(cnt, w1, w2);
    } else {
        cnt = 0.f;
#pragma unroll
        for (int v = 0; v < NV; ++v)
            if ((v * bd + tid) * VEC < hidden) cnt += (float)(VEC - vec_overlap<VEC, UA>((v * bd + tid) * VEC, hidden));
        n_w = cnt;
        merge_weights_step<1, kWave, 0, 6>(n_w, w1, w2);
    }
    const float inv_cnt = cnt > 0.f ? fast_rcp(cnt) : 0.f;

    int slot = 0;
    while (true) {
        const long long off = (long long)row * hidden;
        if constexpr (PRELOAD) {
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                keep_packed(pb[v]);
                keep_packed(pg[v]);
                keep_packed(pe[v]);
            }
        }
        float t[NV][VEC];
        float sum = 0.f;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int col = (v * bd + tid) * VEC;
            const bool ok = FULL || col < hidden;
            const int dup = vec_overlap<VEC, UA>(col, hidden);
            float b[VEC];
            if constexpr (PRELOAD) {
#pragma unroll
                for (int j = 0; j < VEC; ++j) b[j] = (float)pb[v].v[j];
            } else {
                load_bias<T, VEC, UA>(bias, FULL ? col : vec_start<VEC, UA>(col, hidden), b);
            }
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                float tv = (float)xr[v].v[j] + b[j];
                if constexpr (RES) tv += (float)rr[v].v[j];
                tv = ok ? tv : 0.f;
                t[v][j] = tv;
                sum += (UA && j < dup) ? 0.f : tv;
            }
        }
        float mean[1] = {sum * inv_cnt};
        float m2[1] = {0.f};
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const bool ok = FULL || (v * bd + tid) * VEC < hidden;
            const int dup = vec_overlap<VEC, UA>((v * bd + tid) * VEC, hidden);
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                float d = t[v][j] - mean[0];
                m2[0] += (ok && !(UA && j < dup)) ? d * d : 0.f;
            }
        }
        merge_stats_step<1, kWave, 0, 1, 6>(mean, m2, w1, w2);

        const int next = next_live_row(row + (int)gridDim.x);
        const bool more = next < a.n_rows;
        if (more) issue_loads(next);  // the raw registers are dead: refill them before the barrier

        layernorm_block_combine(lds, slot, wave, lane, n_waves, n_w, mean[0], m2[0]);
        const float rstd = fast_rsqrt(fmaf(m2[0], a.inv_hidden, a.eps));

#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int col = (v * bd + tid) * VEC;
            if (FULL || col < hidden) {
                const int colc = FULL ? col : vec_start<VEC, UA>(col, hidden);
                float g[VEC], be[VEC];
                if constexpr (PRELOAD) {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) {
                        g[j] = (float)pg[v].v[j];
                        be[j] = (float)pe[v].v[j];
                    }
                } else {
                    load_param<T, VEC, UA>(gamma, colc, g);
                    load_param<T, VEC, UA>(beta, colc, be);
                }
                Pack<T, VEC> o;
#pragma unroll
                for (int j = 0; j < VEC; ++j) o.v[j] = (T)fmaf((t[v][j] - mean[0]) * rstd, g[j], be[j]);
                store_stream<T, VEC, UA>(out + off + colc, o);
            }
        }
        if (!more) break;
        row = next;
        slot ^= 1;
    }
}

// stream family: rows too long for the block family's registers.  A workgroup of 16 wavefronts owns a row and makes two
// sweeps over it: statistics first (running Welford state per lane, merged chunk by chunk), output second.  The
// t = x + bias + residual values of the row's first kStreamLdsElems columns wait in LDS between the sweeps (as binary32,
// every lane reads back what it wrote itself), so only the columns beyond them are read from memory twice.
constexpr int kStreamLdsElems = 32768;  // 128 KB of the compute unit's 160 KB: one such workgroup per compute unit
template <typename T, int VEC, bool RES>
__global__ __launch_bounds__(kStreamThreads) void layernorm_stream_kernel(LayerNormArgs a) {
    __shared__ LayerNormLds lds;
    __shared__ __attribute__((aligned(16))) float t_lds[kStreamLdsElems];
    const T* __restrict__ x = reinterpret_cast<const T*>(a.x);
    const T* __restrict__ res = reinterpret_cast<const T*>(a.residual);
    const T* __restrict__ bias = reinterpret_cast<const T*>(a.bias);
    const T* __restrict__ gamma = reinterpret_cast<const T*>(a.gamma);
    const T* __restrict__ beta = reinterpret_cast<const T*>(a.beta);
    T* out = reinterpret_cast<T*>(a.out);
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int n_waves = blockDim.x >> 6;
    const int hidden = a.hidden;
    const int step = (int)blockDim.x * VEC;
    constexpr int kStreamUnroll = stream_unroll<VEC>();
    // columns [0, kept) wait in LDS: the whole row, or a whole number of the workgroup's chunks of `step` columns
    const int kept = hidden < kStreamLdsElems ? hidden : kStreamLdsElems;

    float cnt = 0.f;
    for (long long col = (long long)tid * VEC; col < hidden; col += step) cnt += (float)VEC;
    float w1[6], w2[6];
    float n_w = cnt;
    merge_weights_step<1, kWave, 0, 6>(n_w, w1, w2);

    int slot = 0;
    for (int row = blockIdx.x; row < a.n_rows; row += gridDim.x) {
        if (is_padding_row(a, row)) continue;  // uniform over the workgroup
        const long long off = (long long)row * hidden;
        float n_run = 0.f, mu_run = 0.f, q_run = 0.f;
        // one vector of t joins the lane's running statistics
        auto absorb = [&](const float (&t)[VEC]) {
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < VEC; ++j) s += t[j];
            const float cm = s * (1.0f / VEC);
            float cq = 0.f;
#pragma unroll
            for (int j = 0; j < VEC; ++j) cq += (t[j] - cm) * (t[j] - cm);
            const float nt = n_run + (float)VEC;
            const float inv = fast_rcp(nt);
            const float d = cm - mu_run;
            mu_run = fmaf(d, (float)VEC * inv, mu_run);
            q_run = fmaf(d * d, n_run * (float)VEC * inv, q_run + cq);
            n_run = nt;
        };
        // U vectors of the lane, `step` columns apart from `col` on: all loads first, then the arithmetic
        auto first_sweep = [&](long long col, auto u_tag, auto kept_tag) {
            constexpr int U = decltype(u_tag)::value;
            constexpr bool KEPT = decltype(kept_tag)::value;  // all U vectors lie in the kept columns / none does
            Pack<T, VEC> xr[U], rr[U];
            float b[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const long long c = col + (long long)u * step;
                // kept columns are not read again: streaming loads; the others come back in the second sweep
                xr[u] = KEPT ? load_stream<T, VEC>(x + off + c) : load_pack<T, VEC>(x + off + c);
                if constexpr (RES) rr[u] = KEPT ? load_stream<T, VEC>(res + off + c) : load_pack<T, VEC>(res + off + c);
                load_bias<T, VEC>(bias, (int)c, b[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const long long c = col + (long long)u * step;
                float t[VEC];
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    t[j] = (float)xr[u].v[j] + b[u][j];
                    if constexpr (RES) t[j] += (float)rr[u].v[j];
                }
                if constexpr (KEPT) {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) t_lds[c + j] = t[j];
                }
                absorb(t);
            }
        };
        // a lane's columns are tid * VEC + k * step: first those below `kept`, then the rest
        long long col = (long long)tid * VEC;
        stream_columns<kStreamUnroll>(col, kept, step, [&](long long c, auto u) { first_sweep(c, u, std::true_type{}); });
        stream_columns<kStreamUnroll>(col, hidden, step, [&](long long c, auto u) { first_sweep(c, u, std::false_type{}); });

        float mean[1] = {mu_run};
        float m2[1] = {q_run};
        merge_stats_step<1, kWave, 0, 1, 6>(mean, m2, w1, w2);
        layernorm_block_combine(lds, slot, wave, lane, n_waves, n_w, mean[0], m2[0]);
        const float rstd = fast_rsqrt(fmaf(m2[0], a.inv_hidden, a.eps));

        auto second_sweep = [&](long long col, auto u_tag, auto kept_tag) {
            constexpr int U = decltype(u_tag)::value;
            constexpr bool KEPT = decltype(kept_tag)::value;
            Pack<T, VEC> xr[U], rr[U];
            float b[U][VEC], g[U][VEC], be[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const long long c = col + (long long)u * step;
                if constexpr (!KEPT) {
                    xr[u] = load_stream<T, VEC>(x + off + c);
                    if constexpr (RES) rr[u] = load_stream<T, VEC>(res + off + c);
                    load_bias<T, VEC>(bias, (int)c, b[u]);
                }
                load_param<T, VEC>(gamma, (int)c, g[u]);
                load_param<T, VEC>(beta, (int)c, be[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const long long c = col + (long long)u * step;
                float t[VEC];
                if constexpr (KEPT) {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) t[j] = t_lds[c + j];
                } else {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) {
                        t[j] = (float)xr[u].v[j] + b[u][j];
                        if constexpr (RES) t[j] += (float)rr[u].v[j];
                    }
                }
                Pack<T, VEC> o;
#pragma unroll
                for (int j = 0; j < VEC; ++j) o.v[j] = (T)fmaf((t[j] - mean[0]) * rstd, g[u][j], be[u][j]);
                store_stream<T, VEC>(out + off + c, o);
            }
        };
        col = (long long)tid * VEC;
        stream_columns<kStreamUnroll>(col, kept, step, [&](long long c, auto u) { second_sweep(c, u, std::true_type{}); });
        stream_columns<kStreamUnroll>(col, hidden, step, [&](long long c, auto u) { second_sweep(c, u, std::false_type{}); });
        slot ^= 1;  // only rows that used the LDS slot advance it
    }
}

// ---------------------------------------------------------------------------
// host-side launch
// ---------------------------------------------------------------------------
template <typename T, int VEC, int G, int NV, bool RES, int MODE>
hipError_t launch_layernorm_wave(const LayerNormArgs& a, const LaunchCfg& lc, hipStream_t s) {
    (void)lc;
    constexpr int R = rows_in_flight_c(NV, VEC, kLayerNormLimits.target_elems);
    constexpr int TILE_ROWS = R * (kWave / G) * kWaveFamilyWaves;
    int n_tiles = (int)(((long long)a.n_rows + TILE_ROWS - 1) / TILE_ROWS);
    if (a.lengths != nullptr)
        hipLaunchKernelGGL((layernorm_wave_kernel<T, VEC, G, NV, RES, MODE, true>), dim3(n_tiles),
                           dim3(64 * kWaveFamilyWaves), 0, s, a, n_tiles);
    else
        hipLaunchKernelGGL((layernorm_wave_kernel<T, VEC, G, NV, RES, MODE, false>), dim3(n_tiles),
                           dim3(64 * kWaveFamilyWaves), 0, s, a, n_tiles);
    return hipGetLastError();
}

// The shapes the planner can ask for (same rule as make_plan's register budget for the block family).
template <typename T, int VEC, int NV>
constexpr bool block_shape_compiled() {
    return (NV * VEC <= ((sizeof(T) == 2 && VEC == 8) ? kLayerNormLimits.block_max_epl_2byte : kLayerNormLimits.block_max_epl) ||
            NV == 1) &&
           (VEC * (int)sizeof(T) >= 16 || NV <= kLayerNormLimits.block_max_nv_narrow);
}

template <typename T, int VEC, int NV, bool RES, int MODE, bool ROOMY>
hipError_t launch_layernorm_block_r(const Plan& p, const LayerNormArgs& a, const LaunchCfg& lc, hipStream_t s) {
    // The kernel loops over rows with a fixed assignment of rows to workgroups; the grid is a whole multiple of the
    // compute-unit count and never more than the chip holds at once.
    // Workgroups of w wavefronts of THIS kernel that one compute unit of device d holds; 0 = not asked yet.  One table per
    // kernel instantiation, keyed by device and workgroup size.  Concurrent first calls store the same number, so
    // relaxed atomics suffice.
    static std::atomic<int> resident[kMaxDevices][kBlockMaxWaves + 1];
    const bool cached = lc.device >= 0 && lc.device < kMaxDevices;
    int per_cu = cached ? resident[lc.device][p.waves].load(std::memory_order_relaxed) : 0;
    if (per_cu == 0) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, layernorm_block_kernel<T, VEC, NV, RES, MODE, ROOMY>, 64 * p.waves, 0) !=
                hipSuccess || n < 1) {
            (void)hipGetLastError();
            n = 16 / p.waves;
        }
        per_cu = n;
        if (cached) resident[lc.device][p.waves].store(n, std::memory_order_relaxed);
    }
    int grid;
    if (lc.grid_blocks > 0) {
        grid = a.n_rows < lc.grid_blocks ? a.n_rows : lc.grid_blocks;
    } else if (lc.waves_per_cu > 0) {
        grid = capped_grid(a.n_rows, p.waves, kLayerNormBlockCap, lc);
    } else {
        // Measured over workgroups of 2..16 wavefronts, 1..8 workgroups per compute unit, both element types, row counts
        // that divide the grid and row counts that do not: the kernel streams best with the same number of workgroups on
        // every compute unit (a grid of 683 or 820 instead of 768 loses 3-8 points of HBM peak) and about 8 wavefronts
        // per compute unit, each looping over many rows -- 12 for workgroups of 2 or 3 wavefronts are no worse, and
        // workgroups of 8 wavefronts whose lanes need bounds checks want two per compute unit.  [4096, 4096] fp32:
        // 77.0 % of HBM peak with 256 workgroups of 16 rows each, 75.0 % with the 768 that fit the chip at once.
        int per_cu_wanted = p.waves <= 3 ? 4 : p.waves <= 7 ? 2 : (p.waves == 8 && MODE != kModeFull) ? 2 : 1;
        if (per_cu_wanted > per_cu) per_cu_wanted = per_cu;
        const long long cap = (long long)lc.num_cus * per_cu_wanted;
        grid = (int)(a.n_rows < cap ? a.n_rows : cap);
    }
    hipLaunchKernelGGL((layernorm_block_kernel<T, VEC, NV, RES, MODE, ROOMY>), dim3(grid), dim3(64 * p.waves), 0, s, a);
    return hipGetLastError();
}

template <typename T, int VEC, int NV, bool RES, int MODE>
hipError_t launch_layernorm_block(const Plan& p, const LayerNormArgs& a, const LaunchCfg& lc, hipStream_t s) {
    if constexpr (!block_params_fit_128<T, VEC, NV, MODE>()) {
        if (p.waves <= 8) return launch_layernorm_block_r<T, VEC, NV, RES, MODE, true>(p, a, lc, s);
    }
    return launch_layernorm_block_r<T, VEC, NV, RES, MODE, false>(p, a, lc, s);
}

template <typename T, int VEC, bool RES, int MODE>
hipError_t launch_layernorm_vr(const Plan& p, const LayerNormArgs& a, const LaunchCfg& lc, hipStream_t s) {
    if (p.path == kPathWave) {
        if (p.lanes < 64) {
            if (p.nv == 1) {
                switch (p.lanes) {
                    case 4: return launch_layernorm_wave<T, VEC, 4, 1, RES, MODE>(a, lc, s);
                    case 8: return launch_layernorm_wave<T, VEC, 8, 1, RES, MODE>(a, lc, s);
                    case 16: return launch_layernorm_wave<T, VEC, 16, 1, RES, MODE>(a, lc, s);
                    case 32: return launch_layernorm_wave<T, VEC, 32, 1, RES, MODE>(a, lc, s);
                }
            } else if constexpr (MODE == kModeFull) {  // narrower groups with several vectors only when they tile the row
                if (p.lanes == 32 && p.nv == 3) return launch_layernorm_wave<T, VEC, 32, 3, RES, MODE>(a, lc, s);
                if constexpr (5 * VEC <= kLayerNormLimits.wave_max_epl)
                    if (p.lanes == 32 && p.nv == 5) return launch_layernorm_wave<T, VEC, 32, 5, RES, MODE>(a, lc, s);
                if (p.lanes == 16 && p.nv == 3) return launch_layernorm_wave<T, VEC, 16, 3, RES, MODE>(a, lc, s);
            }
            return hipErrorInvalidValue;
        }
        switch (p.nv) {
            case 1: if constexpr (1 * VEC <= kLayerNormLimits.wave_max_epl) return launch_layernorm_wave<T, VEC, 64, 1, RES, MODE>(a, lc, s); else break;
            case 2: if constexpr (2 * VEC <= kLayerNormLimits.wave_max_epl) return launch_layernorm_wave<T, VEC, 64, 2, RES, MODE>(a, lc, s); else break;
            case 3: if constexpr (3 * VEC <= kLayerNormLimits.wave_max_epl) return launch_layernorm_wave<T, VEC, 64, 3, RES, MODE>(a, lc, s); else break;
            case 4: if constexpr (4 * VEC <= kLayerNormLimits.wave_max_epl) return launch_layernorm_wave<T, VEC, 64, 4, RES, MODE>(a, lc, s); else break;
            case 5: if constexpr (5 * VEC <= kLayerNormLimits.wave_max_epl) return launch_layernorm_wave<T, VEC, 64, 5, RES, MODE>(a, lc, s); else break;
            case 6: if constexpr (6 * VEC <= kLayerNormLimits.wave_max_epl) return launch_layernorm_wave<T, VEC, 64, 6, RES, MODE>(a, lc, s); else break;
            case 8: if constexpr (8 * VEC <= kLayerNormLimits.wave_max_epl) return launch_layernorm_wave<T, VEC, 64, 8, RES, MODE>(a, lc, s); else break;
            case 12: if constexpr (12 * VEC <= kLayerNormLimits.wave_max_epl) return launch_layernorm_wave<T, VEC, 64, 12, RES, MODE>(a, lc, s); else break;
            case 16: if constexpr (16 * VEC <= kLayerNormLimits.wave_max_epl) return launch_layernorm_wave<T, VEC, 64, 16, RES, MODE>(a, lc, s); else break;
        }
        return hipErrorInvalidValue;
    }
    if (p.path == kPathBlock) {
        switch (p.nv) {
            case 1: if constexpr (block_shape_compiled<T, VEC, 1>()) return launch_layernorm_block<T, VEC, 1, RES, MODE>(p, a, lc, s); else break;
            case 2: if constexpr (block_shape_compiled<T, VEC, 2>()) return launch_layernorm_block<T, VEC, 2, RES, MODE>(p, a, lc, s); else break;
            case 3: if constexpr (block_shape_compiled<T, VEC, 3>()) return launch_layernorm_block<T, VEC, 3, RES, MODE>(p, a, lc, s); else break;
            case 4: if constexpr (block_shape_compiled<T, VEC, 4>()) return launch_layernorm_block<T, VEC, 4, RES, MODE>(p, a, lc, s); else break;
            case 5: if constexpr (block_shape_compiled<T, VEC, 5>()) return launch_layernorm_block<T, VEC, 5, RES, MODE>(p, a, lc, s); else break;
            case 6: if constexpr (block_shape_compiled<T, VEC, 6>()) return launch_layernorm_block<T, VEC, 6, RES, MODE>(p, a, lc, s); else break;
            case 8: if constexpr (block_shape_compiled<T, VEC, 8>()) return launch_layernorm_block<T, VEC, 8, RES, MODE>(p, a, lc, s); else break;
            case 12: if constexpr (block_shape_compiled<T, VEC, 12>()) return launch_layernorm_block<T, VEC, 12, RES, MODE>(p, a, lc, s); else break;
            case 16: if constexpr (block_shape_compiled<T, VEC, 16>()) return launch_layernorm_block<T, VEC, 16, RES, MODE>(p, a, lc, s); else break;
        }
        return hipErrorInvalidValue;
    }
    // (its LDS row cache leaves room for one workgroup per compute unit)
    hipLaunchKernelGGL((layernorm_stream_kernel<T, VEC, RES>),
                       dim3(capped_grid(a.n_rows, kStreamThreads / 64, kStreamThreads / 64, lc)), dim3(kStreamThreads), 0, s, a);
    return hipGetLastError();
}

template <typename T, int VEC, bool RES, bool UA_OK>
hipError_t launch_layernorm_m(const Plan& p, const LayerNormArgs& a, const LaunchCfg& lc, hipStream_t s) {
    switch (row_mode(p)) {
        case kModeFull: return launch_layernorm_vr<T, VEC, RES, kModeFull>(p, a, lc, s);
        case kModeRagged: return launch_layernorm_vr<T, VEC, RES, kModeRagged>(p, a, lc, s);
        case kModeUnder:
            if constexpr (UA_OK) return launch_layernorm_vr<T, VEC, RES, kModeUnder>(p, a, lc, s);
            break;
    }
    return hipErrorInvalidValue;
}

template <typename T, int VEC, bool UA_OK = false>
hipError_t launch_layernorm_v(const Plan& p, const LayerNormArgs& a, const LaunchCfg& lc, hipStream_t s) {
    return a.residual ? launch_layernorm_m<T, VEC, true, UA_OK>(p, a, lc, s)
                      : launch_layernorm_m<T, VEC, false, UA_OK>(p, a, lc, s);
}

hipError_t launch_layernorm_f32(const Plan& p, const LayerNormArgs& a, const LaunchCfg& lc, hipStream_t s);
hipError_t launch_layernorm_f16(const Plan& p, const LayerNormArgs& a, const LaunchCfg& lc, hipStream_t s);

}  // namespace turbo
