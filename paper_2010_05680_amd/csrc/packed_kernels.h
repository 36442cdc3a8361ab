// Softmax over a row-packed variable-length batch: no padding in memory.
//
// The paper zero-pads the requests of a batch to the longest one (Sections 2.1 and 5) and its kernels work on the
// padding.  Here request b stores its attention scores as [H][len_b][len_b] and the requests follow one another, so
// neither bytes nor arithmetic are spent on padding.  Rows of one launch now differ in length, so the compile-time
// row shapes of the padded kernels do not apply: one wavefront owns one row, holds it in registers (NV vectors per
// lane, sized for the longest request) and masks what lies beyond the row's own length.  Row starts have element
// alignment only, so the 16-byte accesses are the element-aligned ones; the lane that owns a row's last, partial
// vector accesses the vector that ends at the row end instead (overlapping its neighbour's), so a row costs no extra
// memory instructions; only rows shorter than one vector are moved element by element.
#pragma once
#include <hip/hip_runtime.h>

#include "device_utils.h"
#include "softmax_kernels.h"  // SoftmaxLds, softmax_block_combine

namespace turbo {

struct PackedSoftmaxArgs {
    void* scores;
    const int* cu_seqlens;           // [B+1] cumulative request lengths, cu_seqlens[0] = 0
    const long long* score_offsets;  // [B+1] element offset of each request's [H][len][len] block
    int B, H;
    int n_rows;  // H * cu_seqlens[B]
    float scale;
    int long_from;  // workgroup-per-row kernel: rows of at most this many elements are another kernel's and are skipped
};

// Longest row one wavefront holds in registers (16 vectors of 16 bytes per lane); longer rows take a workgroup.
template <typename T>
constexpr int packed_wave_max_len() {
    return kWave * 16 * (16 / (int)sizeof(T));
}
constexpr int kPackedBlockMaxLen = 32768;  // 16 wavefronts x 64 lanes x 32 elements per lane, either element type

constexpr int kPackedWaves = 4;  // wavefronts per workgroup

// Rows a wavefront works on at once (all their loads are issued before the first use): short rows alone would
// leave too few bytes in flight per compute unit.
#ifndef TURBO_PACKED_TARGET_ELEMS
#define TURBO_PACKED_TARGET_ELEMS 16
#endif
constexpr int packed_rows_in_flight(int nv, int vec) {
    const int r = TURBO_PACKED_TARGET_ELEMS / (nv * vec);
    return r >= 2 ? 2 : 1;  // measured: four rows of one fp32 vector per lane are 4-20 % slower than two
}

// First element of the vector that a lane assigned to column c of a row of n >= VEC elements accesses: c itself, or
// n - VEC for the row's last, partial vector.
template <int VEC>
__device__ __forceinline__ int packed_vec_start(int c, int n) {
    return c + VEC <= n ? c : (n - VEC > 0 ? n - VEC : 0);
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

    // All loads of a row are issued together and before the first use (a load under a per-slot branch would be followed by
    // its own wait); slots beyond the row re-read its first vector and are masked afterwards.  len[r] is the same in
    // every lane, so the branches below are scalar.
    float z[R][NV][VEC];
    Pack<T, VEC> raw[R][NV];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (len[r] >= VEC) {
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int c = (v * kWave + lane) * VEC;
                // the lane that owns the row's last, partial vector reads the vector that ends at the row end instead
                // (it overlaps the neighbour's by VEC - len % VEC elements, which this lane leaves out of the sum)
                raw[r][v] = load_stream<T, VEC, true>(rp[r] + (c < len[r] ? packed_vec_start<VEC>(c, len[r]) : 0));
            }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int c = (v * kWave + lane) * VEC;
            if (len[r] >= VEC) {
#pragma unroll
                for (int j = 0; j < VEC; ++j) z[r][v][j] = c < len[r] ? (float)raw[r][v].v[j] * a.scale : -INFINITY;
            } else {  // a row shorter than one vector: element by element, one lane
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    z[r][v][j] = -INFINITY;
                    if (c == 0 && j < len[r]) z[r][v][j] = (float)__builtin_nontemporal_load(rp[r] + j) * a.scale;
                }
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
            const int dup = c - packed_vec_start<VEC>(c, len[r]);  // leading elements that the neighbour already counts
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                const float e = fast_exp2(fmaf(z[r][v][j], kLog2e, shift));  // 0 where nothing was loaded (-inf)
                z[r][v][j] = e;
                l[r] += j >= dup ? e : 0.f;
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
            if (len[r] >= VEC) {
                if (c < len[r]) {  // the overlapped elements are written twice, with the same values
                    Pack<T, VEC> o;
#pragma unroll
                    for (int j = 0; j < VEC; ++j) o.v[j] = (T)(z[r][v][j] * inv);
                    store_stream<T, VEC, true>(rp[r] + packed_vec_start<VEC>(c, len[r]), o);
                }
            } else if (c == 0) {
#pragma unroll
                for (int j = 0; j < VEC; ++j)
                    if (j < len[r]) __builtin_nontemporal_store((T)(z[r][v][j] * inv), rp[r] + j);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Batches of up to 63 requests: the row shape follows each request's own length.
//
// All rows of a request have its length, so a wavefront that works on one request at a time can use the lane-group
// shape of the padded kernels for exactly that length: a request of 100 floats gets 32 lanes per row and four rows
// per wavefront in flight instead of one row on 25 of 64 lanes.  The unit of work is a "task": `rows per wavefront`
// consecutive rows of one request.  Every wavefront derives the task list itself from the length table (one entry per
// lane, one prefix sum over the wavefront), so the host, which never sees the lengths, only needs an upper bound on
// the number of tasks for the grid.
// ---------------------------------------------------------------------------
struct PackedShape {
    int g;   // lanes per row: 8, 16, 32 or 64
    int nv;  // vectors per lane: 1 unless g == 64, then a power of two
    int r;   // rows in flight per lane group
};

template <int VEC>
__host__ __device__ constexpr PackedShape packed_shape(int n) {
    const int nvec = (n + VEC - 1) / VEC;
    PackedShape s{nvec <= 8 ? 8 : nvec <= 16 ? 16 : nvec <= 32 ? 32 : 64, 1, 1};
    while (kWave * s.nv < nvec) s.nv *= 2;
    s.r = packed_rows_in_flight(s.nv, VEC);
    return s;
}
// rows of one task; a power of two that does not grow with n, so the longest request bounds the task count
template <int VEC>
__host__ __device__ constexpr int packed_task_rows(int n) {
    const PackedShape s = packed_shape<VEC>(n);
    return (kWave / s.g) * s.r;
}

// One task: rows row0 .. row0 + (64/G)*R - 1 of a request whose rows (n elements each) start at `base`.
template <typename T, int VEC, int G, int NV>
__device__ __forceinline__ void packed_task(T* base, int n, int row0, int rows_b, float scale, int lane) {
    constexpr int R = packed_rows_in_flight(NV, VEC);
    constexpr int GPW = kWave / G;
    const int grp = lane / G;
    const int gl = lane & (G - 1);

    int len[R];  // n, or 0 for a row past the request's last one
    T* rp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int row = row0 + r * GPW + grp;
        len[r] = row < rows_b ? n : 0;
        rp[r] = base + (long long)(row < rows_b ? row : 0) * n;
    }

    // All loads of the task are issued before the first use, unconditionally: a load under a per-slot branch would be
    // followed by its own wait, which leaves a wavefront one load in flight at a time.  Slots beyond the row (and
    // rows beyond the request) re-read the start of a valid row and are masked afterwards.
    float z[R][NV][VEC];
    if (n >= VEC) {
        Pack<T, VEC> raw[R][NV];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int c = (v * G + gl) * VEC;
                raw[r][v] = load_stream<T, VEC, true>(rp[r] + (c < n ? packed_vec_start<VEC>(c, n) : 0));
            }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const bool live = (v * G + gl) * VEC < len[r];
#pragma unroll
                for (int j = 0; j < VEC; ++j) z[r][v][j] = live ? (float)raw[r][v].v[j] * scale : -INFINITY;
            }
    } else {  // rows shorter than one vector: element by element, one lane per row
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    z[r][v][j] = -INFINITY;
                    if (v == 0 && gl == 0 && j < len[r]) z[r][v][j] = (float)__builtin_nontemporal_load(rp[r] + j) * scale;
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
    group_allreduce<G, R>(m, MaxOp{});

    float l[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const float shift = len[r] > 0 ? -m[r] * kLog2e : 0.f;
        l[r] = 0.f;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int c = (v * G + gl) * VEC;
            const int dup = c - packed_vec_start<VEC>(c, n);
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                const float e = fast_exp2(fmaf(z[r][v][j], kLog2e, shift));
                z[r][v][j] = e;
                l[r] += j >= dup ? e : 0.f;
            }
        }
    }
    group_allreduce<G, R>(l, SumOp{});

#pragma unroll
    for (int r = 0; r < R; ++r) {
        const float inv = fast_rcp(l[r]);
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int c = (v * G + gl) * VEC;
            if (v * G * VEC >= n) continue;
            if (n >= VEC) {
                if (c < len[r]) {
                    Pack<T, VEC> o;
#pragma unroll
                    for (int j = 0; j < VEC; ++j) o.v[j] = (T)(z[r][v][j] * inv);
                    store_stream<T, VEC, true>(rp[r] + packed_vec_start<VEC>(c, n), o);
                }
            } else if (gl == 0) {
#pragma unroll
                for (int j = 0; j < VEC; ++j)
                    if (j < len[r]) __builtin_nontemporal_store((T)(z[r][v][j] * inv), rp[r] + j);
            }
        }
    }
}

// Rows of 32 elements per lane stream best with at most five wavefronts per SIMD (element-aligned accesses like fewer of
// them in flight); the fp32 kernel's registers would allow six, so that build is held at five: 12 requests of
// 1000-2000 floats 474 -> 460 us.
template <typename T, int NVMAX>
constexpr int packed_groups_waves_per_simd() {
    return (sizeof(T) == 4 && NVMAX == 8) ? 5 : 8;
}

// NVMAX: vectors per lane that the longest request needs (a power of two); longer requests are left untouched.
template <typename T, int VEC, int NVMAX>
__global__ __launch_bounds__(64 * kPackedWaves) __attribute__((amdgpu_waves_per_eu(1, packed_groups_waves_per_simd<T, NVMAX>())))
void softmax_packed_groups_kernel(PackedSoftmaxArgs a) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave_id = (int)blockIdx.x * kPackedWaves + (int)(threadIdx.x >> 6);
    const int n_waves = (int)gridDim.x * kPackedWaves;

    // lane b holds request b's length, block offset and task count (B <= 63, so lane B holds the end of the table)
    int cu_l = 0;
    long long off_l = 0;
    if (lane <= a.B) {
        cu_l = a.cu_seqlens[lane];
        off_l = a.score_offsets[lane];
    }
    int n_l = __shfl_down(cu_l, 1) - cu_l;
    if (lane >= a.B || n_l < 0 || n_l > kWave * NVMAX * VEC) n_l = 0;
    const int rows_l = a.H * n_l;
    const int task_rows_l = packed_task_rows<VEC>(n_l > 0 ? n_l : 1);
    const int tasks_l = (rows_l + task_rows_l - 1) / task_rows_l;
    int incl = tasks_l;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(incl, d);
        if (lane >= d) incl += up;
    }
    const int total = __shfl(incl, kWave - 1);
    const int excl = lane < a.B ? incl - tasks_l : 0x7FFFFFFF;

    for (int t = wave_id; t < total; t += n_waves) {
        // the request of task t: the last lane whose first task is <= t (requests without tasks share their
        // successor's first task and are passed over)
        const int b = __builtin_amdgcn_readfirstlane(__popcll(__ballot(excl <= t)) - 1);
        const int n = __builtin_amdgcn_readfirstlane(__shfl(n_l, b));
        const int first = __builtin_amdgcn_readfirstlane(__shfl(excl, b));
        const long long off = __shfl(off_l, b);
        T* base = reinterpret_cast<T*>(a.scores) + off;
        const int rows_b = a.H * n;
        const int row0 = (t - first) * packed_task_rows<VEC>(n);
        const int nvec = (n + VEC - 1) / VEC;
        if (nvec <= 8) {
            packed_task<T, VEC, 8, 1>(base, n, row0, rows_b, a.scale, lane);
        } else if (nvec <= 16) {
            packed_task<T, VEC, 16, 1>(base, n, row0, rows_b, a.scale, lane);
        } else if (nvec <= 32) {
            packed_task<T, VEC, 32, 1>(base, n, row0, rows_b, a.scale, lane);
        } else if (nvec <= 64) {
            packed_task<T, VEC, 64, 1>(base, n, row0, rows_b, a.scale, lane);
        } else {
            if constexpr (NVMAX >= 2) {
                if (nvec <= 128) {
                    packed_task<T, VEC, 64, 2>(base, n, row0, rows_b, a.scale, lane);
                } else {
                    if constexpr (NVMAX >= 4) {
                        if (nvec <= 256) {
                            packed_task<T, VEC, 64, 4>(base, n, row0, rows_b, a.scale, lane);
                        } else {
                            if constexpr (NVMAX >= 8) {
                                if (nvec <= 512) {
                                    packed_task<T, VEC, 64, 8>(base, n, row0, rows_b, a.scale, lane);
                                } else {
                                    if constexpr (NVMAX >= 16) packed_task<T, VEC, 64, 16>(base, n, row0, rows_b, a.scale, lane);
                                }
                            }
                        }
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Requests longer than one wavefront's registers: a workgroup of blockDim.x / 64 wavefronts per row, NV vectors per
// lane, the per-wavefront (reference, sum) pairs combined through LDS with one barrier -- the padded block family's
// scheme on a row whose length and start come from the request tables.  One row per workgroup (short-lived
// workgroups stream best for the softmax).  Rows of at most `long_from` elements belong to the wavefront-per-row
// kernels, which run over the same batch and in turn leave the long rows alone; those workgroups exit at once.
// ---------------------------------------------------------------------------
template <typename T, int VEC, int NV>
__global__ __launch_bounds__(1024) void softmax_packed_block_kernel(PackedSoftmaxArgs a) {
    __shared__ SoftmaxLds lds;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int n_waves = blockDim.x >> 6;
    const int bd = (int)blockDim.x;
    const int row = blockIdx.x;
    if (row >= a.n_rows) return;

    // request of this row: the largest b with H * cu_seqlens[b] <= row (the same for the whole workgroup)
    int lo = 0, hi = a.B;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((long long)a.H * a.cu_seqlens[mid] <= row)
            lo = mid;
        else
            hi = mid;
    }
    const int first = a.cu_seqlens[lo];
    const int n = a.cu_seqlens[lo + 1] - first;
    if (n <= a.long_from || n > bd * NV * VEC) return;  // another kernel's row, or longer than the caller's max_len
    T* rp = reinterpret_cast<T*>(a.scores) + a.score_offsets[lo] + (long long)(row - a.H * first) * n;

    // every load before the first use; slots beyond the row re-read its first vector and are masked (n >= VEC here, and
    // the last, partial vector is the one that ends at the row end)
    Pack<T, VEC> raw[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int c = (v * bd + tid) * VEC;
        raw[v] = load_stream<T, VEC, true>(rp + (c < n ? packed_vec_start<VEC>(c, n) : 0));
    }
    float z[NV][VEC];
    float m[1] = {-INFINITY};
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const bool live = (v * bd + tid) * VEC < n;
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            z[v][j] = live ? (float)raw[v].v[j] * a.scale : -INFINITY;
            m[0] = fmaxf(m[0], z[v][j]);
        }
    }
    group_allreduce<kWave, 1>(m, MaxOp{});
    const float mu_w = m[0] * kLog2e;  // the wavefront's reference in the exponent domain, rounded once
    const float shift = (mu_w == -INFINITY) ? 0.f : -mu_w;

    float l[1] = {0.f};
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int c = (v * bd + tid) * VEC;
        const int dup = c < n ? c - packed_vec_start<VEC>(c, n) : 0;  // leading elements that the neighbour already counts
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            const float e = fast_exp2(fmaf(z[v][j], kLog2e, shift));  // 0 where nothing was loaded (-inf)
            z[v][j] = e;
            l[0] += j >= dup ? e : 0.f;
        }
    }
    group_allreduce<kWave, 1>(l, SumOp{});
    const float f = softmax_block_combine(lds, 0, wave, lane, n_waves, mu_w, l[0]);

#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int c = (v * bd + tid) * VEC;
        if (c < n) {  // the overlapped elements are written twice, with the same values
            Pack<T, VEC> o;
#pragma unroll
            for (int j = 0; j < VEC; ++j) o.v[j] = (T)(z[v][j] * f);
            store_stream<T, VEC, true>(rp + packed_vec_start<VEC>(c, n), o);
        }
    }
}

// max_len decides the register shape: up to one wavefront's capacity the request-shaped kernel (or, for 64 requests and
// more, the wavefront-per-row kernel) does everything; beyond it that kernel serves the requests that fit a wavefront
// and the workgroup-per-row kernel the longer ones.  Returns hipErrorInvalidValue beyond kPackedBlockMaxLen.
// num_cus / grid_cap_per_cu (workgroups per compute unit, 0 = none) size the grid of the request-shaped kernel.
hipError_t launch_softmax_packed(const PackedSoftmaxArgs& a, int elem_size, int max_len, int num_cus, int grid_cap_per_cu,
                                 bool rows_kernel, hipStream_t s);

}  // namespace turbo
