// Instantiations and launchers of the element-wise fused kernels (both element types).
#include "elementwise_kernels.h"

namespace turbo {

namespace {

int grid_for(long long n_vec) {
    long long tiles = (n_vec + kElemThreads * kElemUnroll - 1) / (kElemThreads * kElemUnroll);
    return (int)(tiles < 1 ? 1 : tiles);
}

// Threads per workgroup of the row-slab kernel: the multiple of 64 (at most 256) that wastes the fewest lanes on
// `hv` vector columns; the larger one on a tie.
int slab_threads(int hv) {
    int best = 64;
    long long best_cost = -1;
    for (int t = 64; t <= kElemThreads; t += 64) {
        const long long cost = (long long)((hv + t - 1) / t) * t;
        if (best_cost < 0 || cost <= best_cost) {
            best_cost = cost;
            best = t;
        }
    }
    return best;
}

template <typename T, int VEC>
hipError_t gelu_tv(const GeluArgs& a0, bool ua, hipStream_t s) {
    GeluArgs a = a0;
    if constexpr (VEC > 1) {
        // rows of at least a wavefront of whole vectors: one bias load per lane serves kElemUnroll rows
        if (a.hidden % VEC == 0 && a.hidden / VEC >= kWave && a.rows >= kElemUnroll && !a.force_flat) {
            a.hv = a.hidden / VEC;
            const int threads = slab_threads(a.hv);
            const unsigned n_ct = (unsigned)((a.hv + threads - 1) / threads);
            a.div_ct = make_fastdiv(n_ct);
            const long long row_tiles = ((long long)a.rows + kElemUnroll - 1) / kElemUnroll;
            const dim3 grid((unsigned)(row_tiles * n_ct)), block(threads);
#define TURBO_GELU_ROWS(APPROX, UA) \
    hipLaunchKernelGGL((add_bias_gelu_rows_kernel<T, VEC, APPROX, UA>), grid, block, 0, s, a)
            if (a.approximate) { if (ua) TURBO_GELU_ROWS(true, true); else TURBO_GELU_ROWS(true, false); }
            else               { if (ua) TURBO_GELU_ROWS(false, true); else TURBO_GELU_ROWS(false, false); }
#undef TURBO_GELU_ROWS
            return hipGetLastError();
        }
    }
    const bool wrap = a.hidden % VEC != 0;
    const dim3 grid(grid_for(a.total / VEC)), block(kElemThreads);
#define TURBO_GELU(APPROX, WRAP, UA) \
    hipLaunchKernelGGL((add_bias_gelu_kernel<T, VEC, APPROX, WRAP, UA>), grid, block, 0, s, a)
    if constexpr (VEC == 1) {  // one element per access: no vector can straddle a row end or be misaligned
        if (a.approximate) TURBO_GELU(true, false, false); else TURBO_GELU(false, false, false);
    } else if (a.approximate) {
        if (wrap) { if (ua) TURBO_GELU(true, true, true); else TURBO_GELU(true, true, false); }
        else      { if (ua) TURBO_GELU(true, false, true); else TURBO_GELU(true, false, false); }
    } else {
        if (wrap) { if (ua) TURBO_GELU(false, true, true); else TURBO_GELU(false, true, false); }
        else      { if (ua) TURBO_GELU(false, false, true); else TURBO_GELU(false, false, false); }
    }
#undef TURBO_GELU
    return hipGetLastError();
}

// Items (D elements) of at most this many bytes go through the LDS-tiled kernel: 256 where the input is the side with
// the short runs (the head split; binary16 Q/K/V split of [64,512,3,H,D]: D = 16 23 -> 69 % of HBM peak, D = 32
// 63 -> 74-77 %, D = 64 76 -> 79 %, and [8,4096,3,32,64] 63 -> 75 %; binary32 D = 64 on that shape 67 -> 76 %), 32 where
// the output is (the head merge, whose strided 1 KiB reads do not stream as well as the split's strided writes:
// D = 16 binary16 48 -> 58 %, but D = 32 70 -> 64 %, whatever the tile shape or the number of resident wavefronts).
#ifndef TURBO_PERMUTE_TILED_MAX_ITEM_BYTES
#define TURBO_PERMUTE_TILED_MAX_ITEM_BYTES 256
#endif
#ifndef TURBO_PERMUTE_TILED_MAX_ITEM_BYTES_MERGE
#define TURBO_PERMUTE_TILED_MAX_ITEM_BYTES_MERGE 32
#endif

int log2_floor(int v) {
    int l = 0;
    while ((2 << l) <= v) ++l;
    return l;
}

// The tiled kernel needs whole 16-byte vectors, a power-of-two number of them per item, and a tile count that fits
// the grid; returns false when the shape is not for it.
template <typename T, int VEC>
bool launch_permute_tiled(const PermuteArgs& a, hipStream_t s, hipError_t* err) {
  if constexpr (VEC * (int)sizeof(T) != 16) {
    return false;
  } else {
    if (!a.tiled) return false;
    const int dv = a.D / VEC;
    const int item_bytes = a.D * (int)sizeof(T);
    const int max_item = a.out_order ? TURBO_PERMUTE_TILED_MAX_ITEM_BYTES_MERGE : TURBO_PERMUTE_TILED_MAX_ITEM_BYTES;
    if (dv < 1 || (dv & (dv - 1)) != 0 || item_bytes > max_item) return false;
    // runs of up to 1 KiB on both sides, 16 KiB of items per tile; a short dimension hands its share to the other
    int t_log2 = log2_floor(1024 / item_bytes);
    int t2_log2 = t_log2, t1_log2 = t_log2;
    auto ceil_log2 = [](int n) { int l = 0; while ((1 << l) < n) ++l; return l; };
    if (ceil_log2(a.N2) < t2_log2) { t1_log2 += t2_log2 - ceil_log2(a.N2); t2_log2 = ceil_log2(a.N2); }
    if (ceil_log2(a.N1) < t1_log2) { const int spare = t1_log2 - ceil_log2(a.N1); t1_log2 -= spare; t2_log2 += spare; }
    if (ceil_log2(a.N2) < t2_log2) t2_log2 = ceil_log2(a.N2);
    PermuteTileArgs t;
    t.x = a.x; t.bias = a.bias; t.out = a.out;
    t.B = a.B; t.N1 = a.N1; t.K = a.K; t.N2 = a.N2; t.D = a.D;
    t.t1_log2 = t1_log2; t.t2_log2 = t2_log2; t.dv_log2 = log2_floor(dv);
    const int row_vecs = dv << t2_log2;
    t.row_stride = row_vecs + ((dv - row_vecs) % 16 + 16) % 16;  // congruent to dv modulo 16 vectors
    t.tiles1 = (a.N1 + (1 << t1_log2) - 1) >> t1_log2;
    t.tiles2 = (a.N2 + (1 << t2_log2) - 1) >> t2_log2;
    const long long n_tiles = (long long)a.K * a.B * t.tiles1 * t.tiles2;
    if (n_tiles > 0x7FFFFFFFll) return false;
    t.div_tiles2 = make_fastdiv((unsigned)t.tiles2);
    t.div_tiles1 = make_fastdiv((unsigned)t.tiles1);
    t.div_b = make_fastdiv((unsigned)a.B);
    const size_t lds = (size_t)t.row_stride * 16 * ((size_t)1 << t1_log2);
    const dim3 grid((unsigned)n_tiles), block(kElemThreads);
    if (a.bias)
        hipLaunchKernelGGL((permute_heads_tiled_kernel<T, VEC, true>), grid, block, lds, s, t);
    else
        hipLaunchKernelGGL((permute_heads_tiled_kernel<T, VEC, false>), grid, block, lds, s, t);
    *err = hipGetLastError();
    return true;
  }
}

template <typename T, int VEC>
hipError_t permute_tv(const PermuteArgs& a, hipStream_t s) {
    {
        hipError_t err = hipSuccess;
        if (launch_permute_tiled<T, VEC>(a, s, &err)) return err;
    }
    if (a.grouped) {
        const long long items = a.total / (VEC * kElemUnroll);
        const dim3 g((unsigned)((items + kElemThreads - 1) / kElemThreads)), blk(kElemThreads);
        if (a.bias) {
            // with a bias the unrolled dimension must not enter the bias index: true for the split (input order)
            hipLaunchKernelGGL((permute_heads_grouped_kernel<T, VEC, true, false>), g, blk, 0, s, a);
        } else if (a.out_order) {
            hipLaunchKernelGGL((permute_heads_grouped_kernel<T, VEC, false, true>), g, blk, 0, s, a);
        } else {
            hipLaunchKernelGGL((permute_heads_grouped_kernel<T, VEC, false, false>), g, blk, 0, s, a);
        }
        return hipGetLastError();
    }
    const dim3 grid(grid_for(a.total / VEC)), block(kElemThreads);
    if (a.bias) {
        if (a.out_order) return hipErrorInvalidValue;  // only the split (input order) takes a bias
        hipLaunchKernelGGL((permute_heads_kernel<T, VEC, true, false>), grid, block, 0, s, a);
    } else {
        if (a.out_order)
            hipLaunchKernelGGL((permute_heads_kernel<T, VEC, false, true>), grid, block, 0, s, a);
        else
            hipLaunchKernelGGL((permute_heads_kernel<T, VEC, false, false>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_add_bias_gelu(const GeluArgs& a, int elem_size, int vec, bool under_aligned, hipStream_t s) {
    if (elem_size == 4) {
        if (vec == 4) return gelu_tv<float, 4>(a, under_aligned, s);
        if (vec == 1) return gelu_tv<float, 1>(a, false, s);
    } else {
        if (vec == 8) return gelu_tv<_Float16, 8>(a, under_aligned, s);
        if (vec == 1) return gelu_tv<_Float16, 1>(a, false, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_stream_probe(const float* in0, const float* in1, float* out, long long n_vec, hipStream_t s) {
    const dim3 grid(grid_for(n_vec)), block(kElemThreads);
    if (in1)
        hipLaunchKernelGGL((stream_probe_kernel<true>), grid, block, 0, s, in0, in1, out, n_vec);
    else
        hipLaunchKernelGGL((stream_probe_kernel<false>), grid, block, 0, s, in0, in1, out, n_vec);
    return hipGetLastError();
}

hipError_t launch_permute_heads(const PermuteArgs& a, int elem_size, int vec, hipStream_t s) {
    if (elem_size == 4) {
        switch (vec) {
            case 4: return permute_tv<float, 4>(a, s);
            case 2: return permute_tv<float, 2>(a, s);
            case 1: return permute_tv<float, 1>(a, s);
        }
    } else {
        switch (vec) {
            case 8: return permute_tv<_Float16, 8>(a, s);
            case 4: return permute_tv<_Float16, 4>(a, s);
            case 2: return permute_tv<_Float16, 2>(a, s);
            case 1: return permute_tv<_Float16, 1>(a, s);
        }
    }
    return hipErrorInvalidValue;
}

}  // namespace turbo
