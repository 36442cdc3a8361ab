// Scaled, masked softmax kernels for gfx950 (wave64).
//
// Operation (Sections 2.1 and 4.1.2 of the paper): for every row of the 2-D view
// [B*H*Sq, Sk] of the attention scores, z = scale*s + mask, then a maximum and a
// sum over the row, then exp(z - max)/sum written back in place.
//
// Every element crosses HBM once in and once out: a row lives in registers
// between the load and the store (wave and block families).  The maximum and the
// sum are reduced with DPP / permlane exchanges; R rows are reduced together so
// their exchange chains interleave (the paper's "reduce X rows at once" idea,
// re-derived for 64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "device_utils.h"
#include "plan.h"

namespace turbo {


// How the keys of a row are restricted.
//   kMaskNone     : not at all
//   kMaskAdditive : an additive mask tensor is added to the scaled scores
//   kMaskLengths  : per-request lengths: keys k >= k_len[b] get weight exactly 0 without being read, and rows
//                   q >= q_len[b] are skipped altogether (the variable-length batches of Section 2.1, without
//                   the cost of their zero padding)
//   kMaskCausal   : the same, and query q also sees only the keys k <= q + (Sk - Sq); a build of its own because
//                   every row then ends elsewhere, which changes what the lanes past a row's end should read
enum MaskKind { kMaskNone = 0, kMaskAdditive = 1, kMaskLengths = 2, kMaskCausal = 3 };
constexpr bool mask_by_lengths(int mask_kind) { return mask_kind >= kMaskLengths; }

struct SoftmaxArgs {
    void* scores;
    const void* mask;
    long long mask_stride_b;
    long long mask_stride_q;
    const int* k_lengths;  // kMaskLengths: [B] valid keys per request, or null = all Sk keys
    const int* q_lengths;  // kMaskLengths: [B] valid query rows per request, or null = all rows
    int causal;            // 1 = the launcher takes the kMaskCausal build (the kernels do not read this)
    int n_rows;      // B*H*Sq
    int Sq;
    int Sk;
    int B, H;
    int compact;     // kMaskLengths, wave family, B <= 63: 1 = workgroups loop over the tiles that hold live rows only
    float scale;
    FastDiv div_rows_per_batch;  // H*Sq
    FastDiv div_sq;              // Sq
};

constexpr int kMaxDevices = 64;  // devices with a slot in the per-device launch caches (others are asked every time)

struct LaunchCfg {
    int device;    // the current HIP device
    int num_cus;
    int waves_per_cu;  // caller's cap on resident wavefronts per compute unit used to size the grid; <= 0: family default
    int grid_blocks;   // > 0: exact grid of the looping kernels (testing hook), still capped by the work items
};

// Default grid caps, in wavefronts per compute unit (0 = one tile or row per workgroup, no cap).
// Softmax has no per-workgroup set-up, and a grid of short-lived workgroups streams best.
// LayerNorm's workgroup-per-row family keeps bias/gamma/beta in registers, so it is persistent and loops;
// its lane-group family launches one tile of rows per workgroup.
constexpr int kSoftmaxWaveCap = 0;
constexpr int kSoftmaxBlockCap = 0;
constexpr int kSoftmaxCompactCap = 96;  // length-aware wave family over live tiles only (24 workgroups per compute unit: 16..64 measured alike, 8 was 8 % slower)
constexpr int kLayerNormBlockCap = 32;  // only with the caller's cap; by default its grid is whole rounds of resident workgroups

// Elements of the rows in flight per lane in the wave family: fewer for element-aligned accesses, except with
// per-request lengths, where half of a lane's vectors are typically not loaded at all.
constexpr int softmax_wave_target_elems(int mask_kind, int mode, int row_elems_per_lane) {
    if (mode != kModeUnder || mask_by_lengths(mask_kind)) return kSoftmaxLimits.target_elems;
    // with an additive mask two rows in flight let a per-request key mask be read once for both
    if (mask_kind == kMaskAdditive && row_elems_per_lane == kSoftmaxLimits.target_elems_under) return 2 * row_elems_per_lane;
    return kSoftmaxLimits.target_elems_under;
}

constexpr int rows_in_flight_c(int nv, int vec, int target) {
    int r = target / (nv * vec);
    return r >= 8 ? 8 : r >= 4 ? 4 : r >= 2 ? 2 : 1;
}

// kMaskLengths / kMaskCausal: number of valid keys of `row` (clamped to 0..Sk); 0 also for rows that are skipped.
template <bool CAUSAL>
__device__ __forceinline__ int row_key_count(const SoftmaxArgs& a, int row) {
    const unsigned b = fastdiv((unsigned)row, a.div_rows_per_batch);
    int klen = a.k_lengths != nullptr ? a.k_lengths[b] : a.Sk;
    klen = klen < 0 ? 0 : (klen > a.Sk ? a.Sk : klen);
    if (CAUSAL || a.q_lengths != nullptr) {
        const int q = (int)((unsigned)row - fastdiv((unsigned)row, a.div_sq) * (unsigned)a.Sq);
        if constexpr (CAUSAL) {
            const int visible = q + (a.Sk - a.Sq) + 1;  // may be <= 0 when there are more queries than keys
            klen = visible < klen ? (visible < 0 ? 0 : visible) : klen;
        }
        if (a.q_lengths != nullptr && q >= a.q_lengths[b]) klen = 0;
    }
    return klen;
}

template <typename T, bool MASK>
__device__ __forceinline__ const T* mask_row_ptr(const SoftmaxArgs& a, int row) {
    if constexpr (MASK) {
        unsigned b = fastdiv((unsigned)row, a.div_rows_per_batch);
        unsigned q = (unsigned)row - fastdiv((unsigned)row, a.div_sq) * (unsigned)a.Sq;
        return reinterpret_cast<const T*>(a.mask) + (long long)b * a.mask_stride_b + (long long)q * a.mask_stride_q;
    } else {
        return nullptr;
    }
}

// Where the vector that nominally starts at column `col` is read and written.
// Aligned mode: at `col` (row lengths are multiples of VEC).  Under-aligned mode:
// the row's last vector is shifted back so that it ends exactly at the row end;
// it then overlaps its left neighbour by vec_overlap() elements, which are
// excluded from the row sums and written twice with the same value.  A vector
// past the row end reads column 0 and is never stored.
template <int VEC, bool UA>
__device__ __forceinline__ int vec_start(int col, int row_len) {
    if (col >= row_len) return 0;
    if constexpr (UA) return col + VEC <= row_len ? col : row_len - VEC;
    return col;
}
// Address that the lanes of a length-aware kernel read when their vector holds no valid key (they are not masked off:
// loads under a branch are waited for one by one).  Any address inside the tensor will do, the data is discarded; one
// per workgroup, 512 bytes apart, spreads these reads over the L2 channels where a single fixed address would send
// every wavefront of the grid to the same one.
template <typename T, int VEC>
__device__ __forceinline__ const T* skipped_vector_address(const T* tensor, long long n_elems) {
    const long long off = (long long)(blockIdx.x & 255) * (512 / (int)sizeof(T));
    return off + VEC <= n_elems ? tensor + off : tensor;
}
template <int VEC, bool UA>
__device__ __forceinline__ int vec_overlap(int col, int row_len) {
    if constexpr (UA) return (col < row_len && col + VEC > row_len) ? col + VEC - row_len : 0;
    return 0;
}

// ---------------------------------------------------------------------------
// wave family: G lanes per row, NV vectors per lane, R rows per lane group.
// Lane `gl` of a group holds vectors gl, gl+G, gl+2G, ... of its row, so one load
// instruction of a wavefront covers 64/G consecutive rows in 16*G-byte pieces.
// ---------------------------------------------------------------------------
// WPE: most wavefronts per SIMD the kernel wants resident (8 = whatever its registers allow).  The compiler sizes
// the kernel's register allocation so that no more fit; nothing else changes.
template <typename T, int VEC, int G, int NV, int MK, int MODE, int WPE = 8>
__global__ __launch_bounds__(64 * kWaveFamilyWaves) __attribute__((amdgpu_waves_per_eu(1, WPE)))
void softmax_wave_kernel(SoftmaxArgs a, int n_tiles) {
    constexpr bool MASK = MK == kMaskAdditive;
    constexpr bool VARLEN = mask_by_lengths(MK);
    constexpr bool CAUSAL = MK == kMaskCausal;
    constexpr bool UA = MODE == kModeUnder;
    constexpr bool FULL = MODE == kModeFull;
    static_assert(!(VARLEN && FULL), "per-row key counts need the bounds checks");
    constexpr int R = rows_in_flight_c(NV, VEC, softmax_wave_target_elems(MK, MODE, NV * VEC));
    constexpr int GPW = kWave / G;  // lane groups per wavefront
    constexpr int kWaves = kWaveFamilyWaves;
    constexpr int TILE_ROWS = R * GPW * kWaves;
    // Element-aligned rows of 2-byte elements with an additive mask: when the mask does not depend on the query (a
    // per-request key mask) and the workgroup's rows belong to one request, one lane group fetches the mask row and hands
    // it to the others through LDS in register layout, so the element-aligned mask loads -- the expensive operand, it
    // comes through the vector cache, and at an odd element offset it is not even 4-byte aligned -- are issued once per
    // workgroup instead of once per wavefront.  Measured against the same build without it (binary16, [B,Sk] mask):
    // 197 / 333 / 777 / 1001 keys +2.7 / +1.8 / +3.3 / +1.5 points of HBM peak, 778 keys +3.6; rows whose two rows in
    // flight already share their mask and whose mask rows are 4-byte aligned lose 0.5-4 points to the barrier (198, 334,
    // 494 keys), as do 4-byte elements (-0.4..-2.9), so those keep the per-wavefront loads.
    constexpr bool LDS_MASK = MASK && UA && sizeof(T) == 2;
    __shared__ Pack<T, VEC> mask_lds[LDS_MASK ? NV * G : 1];

    T* __restrict__ scores = reinterpret_cast<T*>(a.scores);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int gl = lane % G;
    const int grp = lane / G;
    const int Sk = a.Sk;
    const float scale = a.scale;
    const T* skip_addr = scores;  // what lanes without a valid key read
    if constexpr (VARLEN) skip_addr = skipped_vector_address<T, VEC>(scores, (long long)a.n_rows * Sk);

    // Compact mode (per-request lengths, up to 63 requests): the padding rows q >= q_len[b] of a zero-padded batch
    // can be most of the tensor, and tiles made of them alone would still cost a workgroup launch each, or, with a
    // looping grid, leave the live tiles unevenly spread over the workgroups.  So the tiles are redefined per
    // (request, head) as chunks of TILE_ROWS live rows, lane b of every wavefront holds request b's tile count, one
    // prefix sum over the wavefront gives each request's first tile, and the workgroups loop over live tiles only.
    bool compact = false;
    int chunks_l = 0, qlen_l = 0, first_l = 0x7FFFFFFF;
    if constexpr (VARLEN) {
        compact = a.compact != 0;
        if (compact) {
            if (lane < a.B) {
                qlen_l = a.q_lengths != nullptr ? a.q_lengths[lane] : a.Sq;
                qlen_l = qlen_l < 0 ? 0 : (qlen_l > a.Sq ? a.Sq : qlen_l);
                if (a.k_lengths != nullptr && a.k_lengths[lane] <= 0) qlen_l = 0;  // no keys: nothing to do
            }
            chunks_l = (qlen_l + TILE_ROWS - 1) / TILE_ROWS;
            const int tiles_l = a.H * chunks_l;
            int incl = tiles_l;
#pragma unroll
            for (int d = 1; d < kWave; d <<= 1) {
                const int up = __shfl_up(incl, d);
                if (lane >= d) incl += up;
            }
            n_tiles = __shfl(incl, kWave - 1);
            if (lane < a.B) first_l = incl - tiles_l;
        }
    }

    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        int row_base = tile * TILE_ROWS + wave * (R * GPW) + grp;
        int row_limit = a.n_rows;  // rows from here on are not this tile's
        if constexpr (VARLEN) {
            if (compact) {
                // the request of this tile: the last lane whose first tile is <= tile (requests without live rows
                // share their successor's first tile and are passed over)
                const int b = __builtin_amdgcn_readfirstlane(__popcll(__ballot(first_l <= tile)) - 1);
                const int c = tile - __builtin_amdgcn_readfirstlane(__shfl(first_l, b));
                const int chunks = __builtin_amdgcn_readfirstlane(__shfl(chunks_l, b));
                const int h = c / chunks;
                const int row0 = (b * a.H + h) * a.Sq;
                row_base = row0 + (c - h * chunks) * TILE_ROWS + wave * (R * GPW) + grp;
                row_limit = row0 + __builtin_amdgcn_readfirstlane(__shfl(qlen_l, b));
            }
        }

        Pack<T, VEC> raw[R][NV];
        Pack<T, VEC> mraw[R][NV];
        int klen[R];  // kMaskLengths: valid keys of the row, 0 = skip the row
        if constexpr (VARLEN) {
            bool any_row = false;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                int row = row_base + r * GPW;
                klen[r] = row < row_limit ? row_key_count<CAUSAL>(a, row) : 0;
                any_row = any_row || klen[r] > 0;
            }
            if (__ballot(any_row) == 0) continue;  // a wavefront whose rows are all padding issues no memory traffic
        }
        // Element-aligned 16-byte loads are the expensive kind, so an under-aligned kernel whose mask does not depend on
        // the query (stride 0: a per-request key mask) reads the mask once for all rows of the wavefront's share of the
        // tile, provided they belong to one request (they almost always do: a request has H * Sq rows).
        bool share_mask = false;
        if constexpr (MASK && UA && R > 1) {
            const int first = tile * TILE_ROWS + wave * (R * GPW);
            int last = first + R * GPW - 1;
            last = last < a.n_rows ? last : a.n_rows - 1;
            share_mask = a.mask_stride_q == 0 && first < a.n_rows &&
                         fastdiv((unsigned)first, a.div_rows_per_batch) == fastdiv((unsigned)last, a.div_rows_per_batch);
        }
        bool wg_share = false;  // the same for every lane of the workgroup
        if constexpr (LDS_MASK) {
            const int first = tile * TILE_ROWS;
            int last = first + TILE_ROWS - 1;
            last = last < a.n_rows ? last : a.n_rows - 1;
            wg_share = a.mask_stride_q == 0 && (R == 1 || (a.mask_stride_b & 1) != 0) &&
                       fastdiv((unsigned)first, a.div_rows_per_batch) == fastdiv((unsigned)last, a.div_rows_per_batch);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            int row = row_base + r * GPW;
            int rowc = row < a.n_rows ? row : a.n_rows - 1;  // out-of-range rows recompute the last row, unstored
            const T* rp = scores + (long long)rowc * Sk;
            const T* mp = mask_row_ptr<T, MASK>(a, rowc);
            if constexpr (!VARLEN) klen[r] = Sk;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                int colc = FULL ? (v * G + gl) * VEC : vec_start<VEC, UA>((v * G + gl) * VEC, Sk);
                if constexpr (VARLEN) {
                    const bool needed = (v * G + gl) * VEC < Sk && colc < klen[r];
                    if constexpr (CAUSAL) {
                        // every row ends elsewhere: repeat the address of the row's last valid vector, which joins
                        // the neighbouring lane's request and touches no further cache line (2-byte elements: +3..5 %
                        // over skip_addr; with per-request key counts alone it measured 1..11 % slower than skip_addr)
                        const int last = klen[r] > 0 ? vec_start<VEC, UA>((klen[r] - 1) / VEC * VEC, Sk) : 0;
                        raw[r][v] = load_stream<T, VEC, UA>(rp + (needed ? colc : last));
                    } else {
                        raw[r][v] = load_stream<T, VEC, UA>(needed ? rp + colc : skip_addr);
                    }
                } else {
                    raw[r][v] = load_stream<T, VEC, UA>(rp + colc);
                }
                if constexpr (MASK) {
                    if (LDS_MASK && wg_share) {
                        // lane group 0 of wavefront 0 fetches the row's mask for everyone (below, after all score loads)
                    } else if (UA && R > 1 && r > 0 && share_mask) {
                        mraw[r][v] = mraw[0][v];
                    } else {
                        mraw[r][v] = load_pack<T, VEC, UA>(mp + colc);
                    }
                }
            }
        }
        if constexpr (LDS_MASK) {
            if (wg_share) {
                if (wave == 0 && grp == 0) {
                    const int rowc = tile * TILE_ROWS < a.n_rows ? tile * TILE_ROWS : a.n_rows - 1;
                    const T* mp = mask_row_ptr<T, MASK>(a, rowc);
#pragma unroll
                    for (int v = 0; v < NV; ++v)
                        mask_lds[v * G + gl] = load_pack<T, VEC, UA>(mp + vec_start<VEC, UA>((v * G + gl) * VEC, Sk));
                }
                __syncthreads();
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const Pack<T, VEC> mv = mask_lds[v * G + gl];
#pragma unroll
                    for (int r = 0; r < R; ++r) mraw[r][v] = mv;
                }
                __syncthreads();  // the next tile of a looping grid overwrites the LDS copy
            }
        }

        float z[R][NV][VEC];
        float m[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            m[r] = -INFINITY;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const bool ok = FULL || (v * G + gl) * VEC < Sk;
                const int c0 = VARLEN ? vec_start<VEC, UA>((v * G + gl) * VEC, Sk) : 0;  // column of element 0
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    float s = (float)raw[r][v].v[j];
                    float t;
                    if constexpr (MASK)
                        t = fmaf(s, scale, (float)mraw[r][v].v[j]);
                    else
                        t = s * scale;
                    t = (ok && (!VARLEN || c0 + j < klen[r])) ? t : -INFINITY;
                    z[r][v][j] = t;
                    m[r] = fmaxf(m[r], t);
                }
            }
        }
        group_allreduce<G, R>(m, MaxOp{});

        float l[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float shift = (VARLEN && klen[r] == 0) ? 0.f : -m[r] * kLog2e;  // a skipped row has no maximum
            l[r] = 0.f;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int dup = vec_overlap<VEC, UA>((v * G + gl) * VEC, Sk);
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    float e = fast_exp2(fmaf(z[r][v][j], kLog2e, shift));
                    z[r][v][j] = e;
                    l[r] += (UA && j < dup) ? 0.f : e;  // overlapped elements belong to the neighbouring vector
                }
            }
        }
        group_allreduce<G, R>(l, SumOp{});

#pragma unroll
        for (int r = 0; r < R; ++r) {
            int row = row_base + r * GPW;
            const float inv = fast_rcp(l[r]);
            T* rp = scores + (long long)row * Sk;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                int col = (v * G + gl) * VEC;
                if (row < a.n_rows && (FULL || col < Sk) && (!VARLEN || klen[r] > 0)) {
                    Pack<T, VEC> o;  // keys past the row's count hold exp2(-inf) = 0
#pragma unroll
                    for (int j = 0; j < VEC; ++j) o.v[j] = (T)(z[r][v][j] * inv);
                    store_stream<T, VEC, UA>(rp + (FULL ? col : vec_start<VEC, UA>(col, Sk)), o);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Cross-wavefront combine of (reference, sum-of-exp) pairs through LDS.
// Each wavefront publishes the reference it subtracted in the exponent and its sum
// taken relative to that reference; one barrier later every lane rebuilds the
// row's reference M and sum L and the factor that rescales its own exponentials.
//
// The reference travels in the base-2 exponent domain: mu_w = fl(m_w * log2 e),
// rounded ONCE, and that very number is what the wavefront's exponentials
// exp2(z * log2 e - mu_w) subtracted.  The rescaling exp2(mu_w - M) between two
// wavefronts then uses the same numbers, so the rounding of m_w * log2 e (an
// absolute error of |m_w| * 2^-24 in the exponent, 1e-5 relative on the result
// once |z| reaches a few hundred) cancels between wavefronts exactly as it
// cancels inside one.  Forming exp2((m_w - M) * log2 e) from the maxima instead
// would leave every wavefront with its own uncancelled rounding.
// Two LDS slots alternate between consecutive rows so one barrier per row is enough.
// ---------------------------------------------------------------------------
struct SoftmaxLds {
    float mu[2][kBlockMaxWaves];
    float l[2][kBlockMaxWaves];
};

// mu_w: the wavefront's reference (-inf when it saw no element); l_w: its sum of exp2(z log2 e - mu_w).
// Returns exp2(mu_w - M) / L with M = max_w mu_w and L = sum_w l_w exp2(mu_w - M).
__device__ __forceinline__ float softmax_block_combine(SoftmaxLds& lds, int slot, int wave, int lane, int n_waves,
                                                       float mu_w, float l_w) {
    if (lane == 0) {
        lds.mu[slot][wave] = mu_w;
        lds.l[slot][wave] = l_w;
    }
    __syncthreads();
    float M = -INFINITY;
    for (int w = 0; w < n_waves; ++w) M = fmaxf(M, lds.mu[slot][w]);
    float L = 0.f;
    for (int w = 0; w < n_waves; ++w) L += lds.l[slot][w] * fast_exp2(lds.mu[slot][w] - M);
    return fast_exp2(mu_w - M) * fast_rcp(L);  // a wavefront that saw no element has mu_w = -inf: factor 0
}

// block family: a workgroup of blockDim.x/64 wavefronts per row, NV vectors per lane.
// Wavefronts per SIMD the kernel is built to allow at least: 4 lets one workgroup of 16 wavefronts onto a compute unit (what
// 1024 threads need anyway); 8 makes the compiler stay within 64 registers so that two fit, for the one shape that would
// otherwise miss it by two registers (32768 halfs per row: 4 vectors of 8 per lane).
template <typename T, int VEC, int NV, int MK, int MODE>
constexpr int softmax_block_min_waves() {
    // (with an additive mask on element-aligned rows the shape does not fit 64 registers)
    return (sizeof(T) == 2 && VEC == 8 && NV == 4 && !mask_by_lengths(MK) && !(MK == kMaskAdditive && MODE == kModeUnder)) ? 8 : 4;
}

template <typename T, int VEC, int NV, int MK, int MODE>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(softmax_block_min_waves<T, VEC, NV, MK, MODE>(), 8)))
void softmax_block_kernel(SoftmaxArgs a) {
    constexpr bool MASK = MK == kMaskAdditive;
    constexpr bool VARLEN = mask_by_lengths(MK);
    constexpr bool CAUSAL = MK == kMaskCausal;
    constexpr bool UA = MODE == kModeUnder;
    constexpr bool FULL = MODE == kModeFull;
    static_assert(!(VARLEN && FULL), "per-row key counts need the bounds checks");
    __shared__ SoftmaxLds lds;
    T* __restrict__ scores = reinterpret_cast<T*>(a.scores);
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int n_waves = blockDim.x >> 6;
    const int Sk = a.Sk;
    const float scale = a.scale;
    const T* skip_addr = scores;  // what lanes without a valid key read
    if constexpr (VARLEN) skip_addr = skipped_vector_address<T, VEC>(scores, (long long)a.n_rows * Sk);

    int slot = 0;
    for (int row = blockIdx.x; row < a.n_rows; row += gridDim.x) {
        T* rp = scores + (long long)row * Sk;
        const T* mp = mask_row_ptr<T, MASK>(a, row);
        int klen = Sk;
        if constexpr (VARLEN) {
            klen = row_key_count<CAUSAL>(a, row);
            if (klen == 0) continue;  // the whole workgroup skips the row together
        }

        Pack<T, VEC> raw[NV];
        Pack<T, VEC> mraw[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int colc = FULL ? (v * (int)blockDim.x + tid) * VEC : vec_start<VEC, UA>((v * (int)blockDim.x + tid) * VEC, Sk);
            if constexpr (VARLEN) {
                const bool needed = (v * (int)blockDim.x + tid) * VEC < Sk && colc < klen;
                if constexpr (CAUSAL)  // as in the wave kernel
                    raw[v] = load_stream<T, VEC, UA>(rp + (needed ? colc : vec_start<VEC, UA>((klen - 1) / VEC * VEC, Sk)));
                else
                    raw[v] = load_stream<T, VEC, UA>(needed ? rp + colc : skip_addr);
            } else {
                raw[v] = load_stream<T, VEC, UA>(rp + colc);
            }
            if constexpr (MASK) mraw[v] = load_pack<T, VEC, UA>(mp + colc);
        }

        float z[NV][VEC];
        float m[1] = {-INFINITY};
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const bool ok = FULL || (v * (int)blockDim.x + tid) * VEC < Sk;
            const int c0 = VARLEN ? vec_start<VEC, UA>((v * (int)blockDim.x + tid) * VEC, Sk) : 0;
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                float s = (float)raw[v].v[j];
                float t;
                if constexpr (MASK)
                    t = fmaf(s, scale, (float)mraw[v].v[j]);
                else
                    t = s * scale;
                t = (ok && (!VARLEN || c0 + j < klen)) ? t : -INFINITY;
                z[v][j] = t;
                m[0] = fmaxf(m[0], t);
            }
        }
        group_allreduce<kWave, 1>(m, MaxOp{});
        const float mu_w = m[0] * kLog2e;  // the wavefront's reference in the exponent domain, rounded once
        const float shift = (mu_w == -INFINITY) ? 0.f : -mu_w;

        float l[1] = {0.f};
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int dup = vec_overlap<VEC, UA>((v * (int)blockDim.x + tid) * VEC, Sk);
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                float e = fast_exp2(fmaf(z[v][j], kLog2e, shift));
                z[v][j] = e;
                l[0] += (UA && j < dup) ? 0.f : e;
            }
        }
        group_allreduce<kWave, 1>(l, SumOp{});

        const float f = softmax_block_combine(lds, slot, wave, lane, n_waves, mu_w, l[0]);

#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int col = (v * (int)blockDim.x + tid) * VEC;
            if (FULL || col < Sk) {
                Pack<T, VEC> o;
#pragma unroll
                for (int j = 0; j < VEC; ++j) o.v[j] = (T)(z[v][j] * f);
                store_stream<T, VEC, UA>(rp + (FULL ? col : vec_start<VEC, UA>(col, Sk)), o);
            }
        }
        slot ^= 1;  // only rows that used the LDS slot advance it (skipped rows execute no barrier)
    }
}

// stream family: rows too long for registers.  First sweep keeps a running
// (max, sum) per lane, rescaling the sum whenever the maximum grows; after the
// combine a second sweep writes the result.  The scores of the row's first
// kStreamLdsBytes wait in LDS between the sweeps (every lane reads back what it
// wrote itself), so only the columns beyond them are read from memory twice.  With
// per-request lengths the first sweep stops at the row's last valid key and the
// second writes zeros beyond it without reading; rows without valid keys are skipped.
constexpr int kStreamLdsBytes = 128 * 1024;  // of the compute unit's 160 KB: one such workgroup per compute unit
// LayerNorm: vectors per lane whose loads are issued together (their widened parameters must fit the registers too)
template <int VEC>
constexpr int stream_unroll() {
    return VEC >= 8 ? 2 : VEC == 4 ? 3 : 4;
}

// Walks a lane's columns col, col + step, ... below `end`: groups of U vectors while they last, then the rest as ONE
// group of its own size (single vectors would each wait for their own load).  body(first column, group size tag).
template <int U, typename Body>
__device__ __forceinline__ void stream_columns(long long& col, long long end, int step, Body body) {
    for (; col + (long long)(U - 1) * step < end; col += (long long)U * step) body(col, std::integral_constant<int, U>{});
    if constexpr (U > 3) {
        if (col + 2ll * step < end) {
            body(col, std::integral_constant<int, 3>{});
            col += 3ll * step;
        }
    }
    if constexpr (U > 2) {
        if (col + (long long)step < end) {
            body(col, std::integral_constant<int, 2>{});
            col += 2ll * step;
        }
    }
    if (col < end) {
        body(col, std::integral_constant<int, 1>{});
        col += step;
    }
}

template <typename T, int VEC, int MK>
__global__ __launch_bounds__(kStreamThreads) void softmax_stream_kernel(SoftmaxArgs a) {
    constexpr bool MASK = MK == kMaskAdditive;
    constexpr bool VARLEN = mask_by_lengths(MK);
    constexpr bool CAUSAL = MK == kMaskCausal;
    constexpr int UNROLL = 4;  // vectors per lane whose loads are issued together
    constexpr int LDS_ELEMS = kStreamLdsBytes / (int)sizeof(T);
    __shared__ SoftmaxLds lds;
    __shared__ Pack<T, VEC> row_lds[LDS_ELEMS / VEC];
    T* __restrict__ scores = reinterpret_cast<T*>(a.scores);
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int n_waves = blockDim.x >> 6;
    const int Sk = a.Sk;
    const float scale = a.scale;
    const int step = (int)blockDim.x * VEC;
    using One = std::integral_constant<int, 1>;

    int slot = 0;
    for (int row = blockIdx.x; row < a.n_rows; row += gridDim.x) {
        int klen = Sk;
        if constexpr (VARLEN) {
            klen = row_key_count<CAUSAL>(a, row);
            if (klen == 0) continue;  // the whole workgroup skips the row together
        }
        T* rp = scores + (long long)row * Sk;
        const T* mp = mask_row_ptr<T, MASK>(a, row);
        // columns [0, kept) wait in LDS: every column that is read, or a whole number of the workgroup's chunks
        const int kept = klen < LDS_ELEMS ? klen : LDS_ELEMS;

        // running reference in the exponent domain (see softmax_block_combine): mu_run = fl(max * log2 e)
        float mu_run = -INFINITY, l_run = 0.f;
        // U vectors of the lane, `step` columns apart from `col` on, all below `kept` or none: loads first, then arithmetic
        auto first_sweep = [&](long long col, auto u_tag, auto kept_tag) {
            constexpr int U = decltype(u_tag)::value;
            constexpr bool KEPT = decltype(kept_tag)::value;
            Pack<T, VEC> raw[U], mraw[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const long long c = col + (long long)u * step;
                // kept columns are not read again: streaming loads; the others come back in the second sweep
                raw[u] = KEPT ? load_stream<T, VEC>(rp + c) : load_pack<T, VEC>(rp + c);
                if constexpr (MASK) mraw[u] = load_pack<T, VEC>(mp + c);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const long long c = col + (long long)u * step;
                if constexpr (KEPT) row_lds[c / VEC] = raw[u];
                float z[VEC];
                float cm = -INFINITY;
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    float s = (float)raw[u].v[j];
                    if constexpr (MASK)
                        z[j] = fmaf(s, scale, (float)mraw[u].v[j]);
                    else
                        z[j] = s * scale;
                    if constexpr (VARLEN) z[j] = c + j < klen ? z[j] : -INFINITY;  // element 0 of the vector is valid
                    cm = fmaxf(cm, z[j]);
                }
                const float cmu = cm * kLog2e;
                if (cmu > mu_run) {
                    l_run *= fast_exp2(mu_run - cmu);  // first chunk: 0 * exp2(-inf) = 0
                    mu_run = cmu;
                }
#pragma unroll
                for (int j = 0; j < VEC; ++j) l_run += fast_exp2(fmaf(z[j], kLog2e, -mu_run));
            }
        };
        // a lane's columns are tid * VEC + k * step: first those below `kept`, then the rest up to the last valid key
        long long col = (long long)tid * VEC;
        stream_columns<UNROLL>(col, kept, step, [&](long long c, auto u) { first_sweep(c, u, std::true_type{}); });
        stream_columns<UNROLL>(col, klen, step, [&](long long c, auto u) { first_sweep(c, u, std::false_type{}); });

        float m[1] = {mu_run};
        group_allreduce<kWave, 1>(m, MaxOp{});
        const float mu_w = m[0];
        float l[1];
        l[0] = (mu_run == -INFINITY) ? 0.f : l_run * fast_exp2(mu_run - mu_w);
        group_allreduce<kWave, 1>(l, SumOp{});

        // factor = exp2(mu_w - M) / L; the second sweep needs exp2(z log2 e - M) / L, so fold mu_w back in
        const float f = softmax_block_combine(lds, slot, wave, lane, n_waves, mu_w, l[0]);
        // exp2(z log2 e - mu_w) * f == exp(z - max)/L; a wavefront with no element stores nothing but zeros
        const float shift = (mu_w == -INFINITY) ? 0.f : -mu_w;

        // SRC: 0 = the vectors wait in LDS, 1 = read them again, 2 = beyond the last valid key (zeros, nothing is read)
        auto second_sweep = [&](long long col, auto u_tag, auto src_tag) {
            constexpr int U = decltype(u_tag)::value;
            constexpr int SRC = decltype(src_tag)::value;
            Pack<T, VEC> raw[U], mraw[U];
            if constexpr (SRC != 2) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const long long c = col + (long long)u * step;
                    if constexpr (SRC == 1) raw[u] = load_stream<T, VEC>(rp + c);
                    if constexpr (MASK) mraw[u] = load_pack<T, VEC>(mp + c);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const long long c = col + (long long)u * step;
                Pack<T, VEC> o;
                if constexpr (SRC == 2) {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) o.v[j] = (T)0.f;
                } else {
                    if constexpr (SRC == 0) raw[u] = row_lds[c / VEC];
#pragma unroll
                    for (int j = 0; j < VEC; ++j) {
                        float s = (float)raw[u].v[j];
                        float zz;
                        if constexpr (MASK)
                            zz = fmaf(s, scale, (float)mraw[u].v[j]);
                        else
                            zz = s * scale;
                        const float y = fast_exp2(fmaf(zz, kLog2e, shift)) * f;
                        o.v[j] = (T)((!VARLEN || c + j < klen) ? y : 0.f);
                    }
                }
                store_stream<T, VEC>(rp + c, o);
            }
        };
        using Lds = std::integral_constant<int, 0>;
        using Again = std::integral_constant<int, 1>;
        using Zeros = std::integral_constant<int, 2>;
        col = (long long)tid * VEC;
        stream_columns<UNROLL>(col, kept, step, [&](long long c, auto u) { second_sweep(c, u, Lds{}); });
        stream_columns<UNROLL>(col, klen, step, [&](long long c, auto u) { second_sweep(c, u, Again{}); });
        if constexpr (VARLEN)
            for (; col < Sk; col += step) second_sweep(col, One{}, Zeros{});
        slot ^= 1;  // only rows that used the LDS slot advance it (skipped rows execute no barrier)
    }
}

// ---------------------------------------------------------------------------
// host-side launch
// ---------------------------------------------------------------------------
inline int capped_grid(long long work_items, int waves_per_block, int default_cap, const LaunchCfg& lc) {
    const int cap_waves = lc.waves_per_cu > 0 ? lc.waves_per_cu : default_cap;
    long long g = work_items;
    if (lc.grid_blocks > 0) {  // every kernel sized here loops over its tiles or rows
        if (g > lc.grid_blocks) g = lc.grid_blocks;
    } else if (cap_waves > 0) {
        long long cap = (long long)lc.num_cus * cap_waves / waves_per_block;
        if (cap < lc.num_cus) cap = lc.num_cus;
        if (g > cap) g = cap;
    }
    if (g > 0x7FFFFFFF) g = 0x7FFFFFFF;
    return (int)(g < 1 ? 1 : g);
}

template <typename T, int VEC, int G, int NV, int MK, int MODE>
hipError_t launch_softmax_wave(const SoftmaxArgs& a, const LaunchCfg& lc, hipStream_t s) {
    constexpr int R = rows_in_flight_c(NV, VEC, softmax_wave_target_elems(MK, MODE, NV * VEC));
    constexpr int TILE_ROWS = R * (kWave / G) * kWaveFamilyWaves;
    int n_tiles = (int)(((long long)a.n_rows + TILE_ROWS - 1) / TILE_ROWS);
    if constexpr (mask_by_lengths(MK)) {
        // (element-aligned 4-byte rows: see below; with per-request lengths 6 wavefronts per SIMD measured 1-2 % faster
        // than 7, and 5 faster again by as much for rows of 3 and more vectors per lane)
        constexpr int WPE = (MODE == kModeUnder && sizeof(T) == 4 && G == 64 && NV >= 2) ? (NV >= 3 ? 5 : 6) : 8;
        if (a.B < kWave && a.q_lengths != nullptr) {
            // live tiles only: at most this many (every request with all its rows), shared by a grid of looping workgroups
            SoftmaxArgs c = a;
            c.compact = 1;
            const long long bound = (long long)a.B * a.H * ((a.Sq + TILE_ROWS - 1) / TILE_ROWS);
            n_tiles = (int)(bound < 0x7FFFFFFF ? bound : 0x7FFFFFFF);
            hipLaunchKernelGGL((softmax_wave_kernel<T, VEC, G, NV, MK, MODE, WPE>),
                               dim3(capped_grid(n_tiles, kWaveFamilyWaves, kSoftmaxCompactCap, lc)), dim3(64 * kWaveFamilyWaves), 0, s,
                               c, n_tiles);
            return hipGetLastError();
        }
        hipLaunchKernelGGL((softmax_wave_kernel<T, VEC, G, NV, MK, MODE, WPE>),
                           dim3(capped_grid(n_tiles, kWaveFamilyWaves, kSoftmaxWaveCap, lc)), dim3(64 * kWaveFamilyWaves), 0, s, a, n_tiles);
        return hipGetLastError();
    } else {
        // Element-aligned 4-byte rows stream best with few wavefronts resident (their accesses straddle cache lines, and the
        // more of them are in flight the more they thrash): the kernel is built to hold a SIMD at 5 wavefronts (20 per compute
        // unit), at 4 for rows of 384 floats and more.  Measured on 77..1001 floats, with and without an additive mask:
        // +1..4 points of HBM peak (config 2: 128.8 -> 123.2 us); 2-byte elements, which have half the bytes in flight per
        // wavefront, lose with any such limit.  Rows of 384 floats and more have at least 2 vectors per lane on 64 lanes,
        // shorter rows at most 2, so only that shape needs both builds.
        const dim3 grid(capped_grid(n_tiles, kWaveFamilyWaves, kSoftmaxWaveCap, lc)), block(64 * kWaveFamilyWaves);
        if constexpr (MODE == kModeUnder && sizeof(T) == 4) {
            if constexpr (G < 64 || NV == 1) {
                hipLaunchKernelGGL((softmax_wave_kernel<T, VEC, G, NV, MK, MODE, 5>), grid, block, 0, s, a, n_tiles);
            } else if constexpr (NV >= 3) {
                hipLaunchKernelGGL((softmax_wave_kernel<T, VEC, G, NV, MK, MODE, 4>), grid, block, 0, s, a, n_tiles);
            } else if (a.Sk < 384) {
                hipLaunchKernelGGL((softmax_wave_kernel<T, VEC, G, NV, MK, MODE, 5>), grid, block, 0, s, a, n_tiles);
            } else {
                hipLaunchKernelGGL((softmax_wave_kernel<T, VEC, G, NV, MK, MODE, 4>), grid, block, 0, s, a, n_tiles);
            }
        } else {
            hipLaunchKernelGGL((softmax_wave_kernel<T, VEC, G, NV, MK, MODE>), grid, block, 0, s, a, n_tiles);
        }
        return hipGetLastError();
    }
}

// The shapes the planner can ask for: within the register budget; and with vectors of one or two elements its
// last pass (smallest workgroup that fits) never lands on 5, 6 or 8 vectors per lane.
template <int VEC, int NV>
constexpr bool softmax_block_shape_compiled() {
    return (NV * VEC <= kSoftmaxLimits.block_max_epl || NV == 1) && (VEC > 2 || (NV != 5 && NV != 6 && NV != 8));
}

template <typename T, int VEC, int NV, int MK, int MODE>
hipError_t launch_softmax_block(const Plan& p, const SoftmaxArgs& a, const LaunchCfg& lc, hipStream_t s) {
    hipLaunchKernelGGL((softmax_block_kernel<T, VEC, NV, MK, MODE>),
                       dim3(capped_grid(a.n_rows, p.waves, kSoftmaxBlockCap, lc)), dim3(64 * p.waves), 0, s, a);
    return hipGetLastError();
}

template <typename T, int VEC, int MK, int MODE>
hipError_t launch_softmax_vm(const Plan& p, const SoftmaxArgs& a, const LaunchCfg& lc, hipStream_t s) {
    if (p.path == kPathWave) {
        if (p.lanes < 64) {
            if (p.nv == 1) {
                switch (p.lanes) {
                    case 4: return launch_softmax_wave<T, VEC, 4, 1, MK, MODE>(a, lc, s);
                    case 8: return launch_softmax_wave<T, VEC, 8, 1, MK, MODE>(a, lc, s);
                    case 16: return launch_softmax_wave<T, VEC, 16, 1, MK, MODE>(a, lc, s);
                    case 32: return launch_softmax_wave<T, VEC, 32, 1, MK, MODE>(a, lc, s);
                }
            } else if constexpr (MODE == kModeFull) {  // narrower groups with several vectors only when they tile the row
                if (p.lanes == 32 && p.nv == 3) return launch_softmax_wave<T, VEC, 32, 3, MK, MODE>(a, lc, s);
                if constexpr (5 * VEC <= kSoftmaxLimits.wave_max_epl)
                    if (p.lanes == 32 && p.nv == 5) return launch_softmax_wave<T, VEC, 32, 5, MK, MODE>(a, lc, s);
                if (p.lanes == 16 && p.nv == 3) return launch_softmax_wave<T, VEC, 16, 3, MK, MODE>(a, lc, s);
            }
            return hipErrorInvalidValue;
        }
        switch (p.nv) {
            case 1: if constexpr (1 * VEC <= kSoftmaxLimits.wave_max_epl) return launch_softmax_wave<T, VEC, 64, 1, MK, MODE>(a, lc, s); else break;
            case 2: if constexpr (2 * VEC <= kSoftmaxLimits.wave_max_epl) return launch_softmax_wave<T, VEC, 64, 2, MK, MODE>(a, lc, s); else break;
            case 3: if constexpr (3 * VEC <= kSoftmaxLimits.wave_max_epl) return launch_softmax_wave<T, VEC, 64, 3, MK, MODE>(a, lc, s); else break;
            case 4: if constexpr (4 * VEC <= kSoftmaxLimits.wave_max_epl) return launch_softmax_wave<T, VEC, 64, 4, MK, MODE>(a, lc, s); else break;
            case 5: if constexpr (5 * VEC <= kSoftmaxLimits.wave_max_epl) return launch_softmax_wave<T, VEC, 64, 5, MK, MODE>(a, lc, s); else break;
            case 6: if constexpr (6 * VEC <= kSoftmaxLimits.wave_max_epl) return launch_softmax_wave<T, VEC, 64, 6, MK, MODE>(a, lc, s); else break;
            case 8: if constexpr (8 * VEC <= kSoftmaxLimits.wave_max_epl) return launch_softmax_wave<T, VEC, 64, 8, MK, MODE>(a, lc, s); else break;
            case 12: if constexpr (12 * VEC <= kSoftmaxLimits.wave_max_epl) return launch_softmax_wave<T, VEC, 64, 12, MK, MODE>(a, lc, s); else break;
            case 16: if constexpr (16 * VEC <= kSoftmaxLimits.wave_max_epl) return launch_softmax_wave<T, VEC, 64, 16, MK, MODE>(a, lc, s); else break;
        }
        return hipErrorInvalidValue;
    }
    if (p.path == kPathBlock) {
        switch (p.nv) {
            case 1: if constexpr (softmax_block_shape_compiled<VEC, 1>()) return launch_softmax_block<T, VEC, 1, MK, MODE>(p, a, lc, s); else break;
            case 2: if constexpr (softmax_block_shape_compiled<VEC, 2>()) return launch_softmax_block<T, VEC, 2, MK, MODE>(p, a, lc, s); else break;
            case 3: if constexpr (softmax_block_shape_compiled<VEC, 3>()) return launch_softmax_block<T, VEC, 3, MK, MODE>(p, a, lc, s); else break;
            case 4: if constexpr (softmax_block_shape_compiled<VEC, 4>()) return launch_softmax_block<T, VEC, 4, MK, MODE>(p, a, lc, s); else break;
            case 5: if constexpr (softmax_block_shape_compiled<VEC, 5>()) return launch_softmax_block<T, VEC, 5, MK, MODE>(p, a, lc, s); else break;
            case 6: if constexpr (softmax_block_shape_compiled<VEC, 6>()) return launch_softmax_block<T, VEC, 6, MK, MODE>(p, a, lc, s); else break;
            case 8: if constexpr (softmax_block_shape_compiled<VEC, 8>()) return launch_softmax_block<T, VEC, 8, MK, MODE>(p, a, lc, s); else break;
            case 12: if constexpr (softmax_block_shape_compiled<VEC, 12>()) return launch_softmax_block<T, VEC, 12, MK, MODE>(p, a, lc, s); else break;
            case 16: if constexpr (softmax_block_shape_compiled<VEC, 16>()) return launch_softmax_block<T, VEC, 16, MK, MODE>(p, a, lc, s); else break;
        }
        return hipErrorInvalidValue;
    }
    // (its LDS row cache leaves room for one workgroup per compute unit)
    hipLaunchKernelGGL((softmax_stream_kernel<T, VEC, MK>),
                       dim3(capped_grid(a.n_rows, kStreamThreads / 64, kStreamThreads / 64, lc)), dim3(kStreamThreads), 0, s, a);
    return hipGetLastError();
}

// UA_OK: the under-aligned flavour exists only for the widest vector of each element type.
template <typename T, int VEC, int MK, bool UA_OK>
hipError_t launch_softmax_m(const Plan& p, const SoftmaxArgs& a, const LaunchCfg& lc, hipStream_t s) {
    switch (row_mode(p)) {
        case kModeFull:
            if constexpr (!mask_by_lengths(MK)) return launch_softmax_vm<T, VEC, MK, kModeFull>(p, a, lc, s);
            break;
        case kModeRagged: return launch_softmax_vm<T, VEC, MK, kModeRagged>(p, a, lc, s);
        case kModeUnder:
            if constexpr (UA_OK) return launch_softmax_vm<T, VEC, MK, kModeUnder>(p, a, lc, s);
            break;
    }
    return hipErrorInvalidValue;
}

template <typename T, int VEC, bool UA_OK = false>
hipError_t launch_softmax_v(const Plan& p, const SoftmaxArgs& a, const LaunchCfg& lc, hipStream_t s) {
    if (a.causal) return launch_softmax_m<T, VEC, kMaskCausal, UA_OK>(p, a, lc, s);
    if (a.k_lengths || a.q_lengths) return launch_softmax_m<T, VEC, kMaskLengths, UA_OK>(p, a, lc, s);
    return a.mask ? launch_softmax_m<T, VEC, kMaskAdditive, UA_OK>(p, a, lc, s)
                  : launch_softmax_m<T, VEC, kMaskNone, UA_OK>(p, a, lc, s);
}

// Defined once per element type in softmax_f32.hip / softmax_f16.hip.
hipError_t launch_softmax_f32(const Plan& p, const SoftmaxArgs& a, const LaunchCfg& lc, hipStream_t s);
hipError_t launch_softmax_f16(const Plan& p, const SoftmaxArgs& a, const LaunchCfg& lc, hipStream_t s);

}  // namespace turbo
