// Softmax over a row-packed variable-length batch: no padding in memory.
//
// The paper zero-pads the requests of a batch to the longest one (Sections 2.1 and 5) and its kernels work on the
// padding.  Here request b stores its attention scores as [H][len_b][len_b] and the requests follow one another, so
// neither bytes nor arithmetic are spent on padding.  Rows of one launch now differ in length, so the compile-time
// row shapes of the padded kernels do not apply: one wavefront owns one row, holds it in registers (NV vectors per
// lane, sized for the longest request) and masks what lies beyond the row's own length.  Row starts have element
// alignment only, so the 16-byte accesses are the element-aligned ones; the last, partial vector of a row is moved
// element by element by the one lane that owns it.
#pragma once
#include <hip/hip_runtime.h>

#include "device_utils.h"

namespace turbo {

struct PackedSoftmaxArgs {
    void* scores;
    const int* cu_seqlens;           // [B+1] cumulative request lengths, cu_seqlens[0] = 0
    const long long* score_offsets;  // [B+1] element offset of each request's [H][len][len] block
    int B, H;
    int n_rows;  // H * cu_seqlens[B]
    float scale;
};

constexpr int kPackedWaves = 4;  // wavefronts per workgroup

// Rows a wavefront works on at once (all their loads are issued before the first use): short rows alone would
// leave too few bytes in flight per compute unit.
#ifndef TURBO_PACKED_TARGET_ELEMS
#define TURBO_PACKED_TARGET_ELEMS 16
#endif
constexpr int packed_rows_in_flight(int nv, int vec) {
    const int r = TURBO_PACKED_TARGET_ELEMS / (nv * vec);
    return r >= 4 ? 4 : r >= 2 ? 2 : 1;
}

template <typename T, int VEC, int NV>
__global__ __launch_bounds__(64 * kPackedWaves) void softmax_packed_kernel(PackedSoftmaxArgs a) {
    constexpr int R = packed_rows_in_flight(NV, VEC);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int row0 = ((int)blockIdx.x * kPackedWaves + wave) * R;
    if (row0 >= a.n_rows) return;

    // Up to 63 requests: every lane holds one entry of the two tables (one coalesced load each), a row finds its
    // request with one ballot and fetches the three values it needs by lane index.  Larger batches search the
    // table in memory instead.
    const bool in_lanes = a.B < kWave;
    int cu_l = 0x7FFFFFFF;
    long long off_l = 0;
    if (in_lanes && lane <= a.B) {
        cu_l = a.cu_seqlens[lane];
        off_l = a.score_offsets[lane];
    }

    int len[R];  // 0: nothing to do for this row
    T* rp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int row = row0 + r;
        len[r] = 0;
        rp[r] = reinterpret_cast<T*>(a.scores);
        if (row >= a.n_rows) continue;
        // request of this row: the largest b with H * cu_seqlens[b] <= row (requests without tokens own no row)
        int first, next;
        long long base;
        if (in_lanes) {
            const int lo = __popcll(__ballot((long long)a.H * cu_l <= row)) - 1;  // entry 0 is 0: at least one lane votes
            first = __shfl(cu_l, lo);
            next = __shfl(cu_l, lo + 1);
            base = __shfl(off_l, lo);
        } else {
            int lo = 0, hi = a.B;
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if ((long long)a.H * a.cu_seqlens[mid] <= row)
                    lo = mid;
                else
                    hi = mid;
            }
            first = a.cu_seqlens[lo];
            next = a.cu_seqlens[lo + 1];
            base = a.score_offsets[lo];
        }
        const int n = next - first;
        if (n <= 0 || n > kWave * NV * VEC) continue;  // longer than the caller's max_len: the row is left untouched
        len[r] = n;
        // (h, q) of the row inside its request: row - H * first = h * n + q
        rp[r] = reinterpret_cast<T*>(a.scores) + base + (long long)(row - a.H * first) * n;
    }

    // len[r] is the same in every lane, so "this vector slot lies wholly beyond the row" is a scalar branch: short
    // rows skip the slots they do not use instead of issuing their (empty) loads.
    float z[R][NV][VEC];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int c = (v * kWave + lane) * VEC;
#pragma unroll
            for (int j = 0; j < VEC; ++j) z[r][v][j] = -INFINITY;
            if (v * kWave * VEC >= len[r]) continue;
            if (c + VEC <= len[r]) {
                const Pack<T, VEC> raw = load_stream<T, VEC, true>(rp[r] + c);
#pragma unroll
                for (int j = 0; j < VEC; ++j) z[r][v][j] = (float)raw.v[j] * a.scale;
            } else if (c < len[r]) {  // the row's last, partial vector: one lane per row
#pragma unroll
                for (int j = 0; j < VEC; ++j)
                    if (c + j < len[r]) z[r][v][j] = (float)__builtin_nontemporal_load(rp[r] + c + j) * a.scale;
            }
        }

    float m[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        m[r] = -INFINITY;
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int j = 0; j < VEC; ++j) m[r] = fmaxf(m[r], z[r][v][j]);
    }
    group_allreduce<kWave, R>(m, MaxOp{});

    float l[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const float shift = len[r] > 0 ? -m[r] * kLog2e : 0.f;  // a row without work has no maximum
        l[r] = 0.f;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int c = (v * kWave + lane) * VEC;
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                const float e = c + j < len[r] ? fast_exp2(fmaf(z[r][v][j], kLog2e, shift)) : 0.f;
                z[r][v][j] = e;
                l[r] += e;
            }
        }
    }
    group_allreduce<kWave, R>(l, SumOp{});

#pragma unroll
    for (int r = 0; r < R; ++r) {
        const float inv = fast_rcp(l[r]);
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int c = (v * kWave + lane) * VEC;
            if (v * kWave * VEC >= len[r]) continue;
            if (c + VEC <= len[r]) {
                Pack<T, VEC> o;
#pragma unroll
                for (int j = 0; j < VEC; ++j) o.v[j] = (T)(z[r][v][j] * inv);
                store_stream<T, VEC, true>(rp[r] + c, o);
            } else if (c < len[r]) {
#pragma unroll
                for (int j = 0; j < VEC; ++j)
                    if (c + j < len[r]) __builtin_nontemporal_store((T)(z[r][v][j] * inv), rp[r] + c + j);
            }
        }
    }
}

// max_len decides the register shape; returns hipErrorInvalidValue when a row of max_len does not fit a wavefront.
hipError_t launch_softmax_packed(const PackedSoftmaxArgs& a, int elem_size, int max_len, hipStream_t s);

}  // namespace turbo
