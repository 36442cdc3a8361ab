// C ABI of the library: argument validation, variant choice, launch.
// Validation runs before the first HIP call, so every error except
// TURBO_ERR_LAUNCH is reported without a GPU.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <cstring>

#include "../../include/turbo_reduce.h"
#include "../../include/turbo_reduce_testing.h"
#include "elementwise_kernels.h"
#include "layernorm_kernels.h"
#include "packed_kernels.h"
#include "plan.h"
#include "softmax_kernels.h"

namespace {

// Process-wide switches of the testing hooks (turbo_reduce_testing.h).  Relaxed atomics: a test flips them between
// calls, never during one; the atomics only keep a concurrent reader free of a data race.
std::atomic<int> g_ovr_value[TURBO_OVR_COUNT_] = {{-1}, {-1}, {-1}, {-1}, {-1}};

turbo::Overrides current_overrides() {
    turbo::Overrides o;
    o.path = g_ovr_value[TURBO_OVR_PATH].load(std::memory_order_relaxed);
    o.max_vec_bytes = g_ovr_value[TURBO_OVR_MAX_VEC_BYTES].load(std::memory_order_relaxed);
    o.grid_waves = g_ovr_value[TURBO_OVR_GRID_WAVES].load(std::memory_order_relaxed);
    o.block_waves = g_ovr_value[TURBO_OVR_BLOCK_WAVES].load(std::memory_order_relaxed);
    o.grid_blocks = g_ovr_value[TURBO_OVR_GRID_BLOCKS].load(std::memory_order_relaxed);
    return o;
}

constexpr int kMaxRows = 0x7FFF0000;  // leaves headroom for tile rounding in 32-bit row indices
// Compute units per device, asked once per device.  Two threads that race on the first call both store the same
// number, so relaxed atomics are enough.
std::atomic<int> g_num_cus[turbo::kMaxDevices];

int elem_size_of(int dtype) { return dtype == TURBO_F32 ? 4 : dtype == TURBO_F16 ? 2 : 0; }

// Largest power of two (bytes, at most 16) dividing the address.
long long byte_alignment(const void* p) {
    uintptr_t v = reinterpret_cast<uintptr_t>(p) | 16u;
    return (long long)(v & (~v + 1));
}

long long min_ll(long long a, long long b) { return a < b ? a : b; }

// Largest power of two (elements, at most 16) dividing a stride; a zero stride constrains nothing.
long long stride_alignment(long long stride) {
    if (stride == 0) return 16;
    long long v = stride | 16;
    return v & (~v + 1);
}

// The current device and its compute-unit count.
int current_device(turbo::LaunchCfg* lc) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return TURBO_ERR_LAUNCH;
    const bool cached = dev >= 0 && dev < turbo::kMaxDevices;
    int n = cached ? g_num_cus[dev].load(std::memory_order_relaxed) : 0;
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            return TURBO_ERR_LAUNCH;
        if (cached) g_num_cus[dev].store(n, std::memory_order_relaxed);
    }
    lc->device = dev;
    lc->num_cus = n;
    return TURBO_OK;
}

int launch_cfg(const turbo::Overrides& ovr, turbo::LaunchCfg* lc) {
    if (int st = current_device(lc)) return st;
    lc->grid_blocks = ovr.grid_blocks > 0 ? ovr.grid_blocks : 0;
    lc->waves_per_cu = ovr.grid_waves > 0 ? (ovr.grid_waves > (1 << 20) ? (1 << 22) : ovr.grid_waves * 4) : 0;
    return TURBO_OK;
}

int softmax_impl(void* scores, const void* mask, long long msb, long long msq, const int* q_lengths,
                 const int* k_lengths, int B, int H, int Sq, int Sk, float scale, int dtype, void* stream,
                 int causal = 0) {
    if (scores == nullptr) return TURBO_ERR_NULL;
    const int es = elem_size_of(dtype);
    if (es == 0) return TURBO_ERR_DTYPE;
    if (B <= 0 || H <= 0 || Sq <= 0 || Sk <= 0) return TURBO_ERR_SHAPE;
    const long long rows_per_batch = (long long)H * Sq;  // two 31-bit factors: fits
    if (rows_per_batch > kMaxRows || rows_per_batch * B > kMaxRows) return TURBO_ERR_SHAPE;  // <= 2^31 * 2^31
    const long long n_rows = rows_per_batch * B;
    if (mask != nullptr && (msb < 0 || msq < 0)) return TURBO_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(scores) % es != 0) return TURBO_ERR_ALIGN;
    if (mask != nullptr && reinterpret_cast<uintptr_t>(mask) % es != 0) return TURBO_ERR_ALIGN;

    long long align_elems = byte_alignment(scores) / es;
    if (mask != nullptr) {
        align_elems = min_ll(align_elems, byte_alignment(mask) / es);
        align_elems = min_ll(align_elems, stride_alignment(msb));
        align_elems = min_ll(align_elems, stride_alignment(msq));
    }
    turbo::Overrides ovr = current_overrides();
    if (k_lengths != nullptr || q_lengths != nullptr || causal) {  // per-row key counts: the kernels need their bounds checks
        if (reinterpret_cast<uintptr_t>(k_lengths) % 4 != 0 || reinterpret_cast<uintptr_t>(q_lengths) % 4 != 0)
            return TURBO_ERR_ALIGN;
        ovr.no_full = 1;
    }
    const turbo::Plan plan = turbo::make_plan(Sk, es, align_elems, n_rows, turbo::kSoftmaxLimits, ovr);

    turbo::SoftmaxArgs a;
    a.scores = scores;
    a.mask = mask;
    a.k_lengths = k_lengths;
    a.q_lengths = q_lengths;
    a.causal = causal;
    a.mask_stride_b = msb;
    a.mask_stride_q = msq;
    a.n_rows = (int)n_rows;
    a.Sq = Sq;
    a.Sk = Sk;
    a.B = B;
    a.H = H;
    a.compact = 0;
    a.scale = scale;
    a.div_rows_per_batch = turbo::make_fastdiv((unsigned)((long long)H * Sq));
    a.div_sq = turbo::make_fastdiv((unsigned)Sq);

    turbo::LaunchCfg lc;
    if (int st = launch_cfg(ovr, &lc)) return st;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    hipError_t err = dtype == TURBO_F32 ? turbo::launch_softmax_f32(plan, a, lc, s)
                                        : turbo::launch_softmax_f16(plan, a, lc, s);
    return err == hipSuccess ? TURBO_OK : TURBO_ERR_LAUNCH;
}

int layernorm_impl(const void* x, const void* residual, const void* bias, const void* gamma, const void* beta,
                   int rows, int hidden, float eps, void* out, int dtype, void* stream, const int* lengths = nullptr,
                   int S = 1) {
    if (x == nullptr || gamma == nullptr || beta == nullptr || out == nullptr) return TURBO_ERR_NULL;
    const int es = elem_size_of(dtype);
    if (es == 0) return TURBO_ERR_DTYPE;
    if (rows <= 0 || hidden <= 0 || rows > kMaxRows) return TURBO_ERR_SHAPE;
    const void* ptrs[6] = {x, residual, bias, gamma, beta, out};
    long long align_elems = 16;
    for (const void* p : ptrs) {
        if (p == nullptr) continue;
        if (reinterpret_cast<uintptr_t>(p) % es != 0) return TURBO_ERR_ALIGN;
        align_elems = min_ll(align_elems, byte_alignment(p) / es);
    }
    const turbo::Overrides ovr = current_overrides();
    const turbo::Plan plan = turbo::make_plan(hidden, es, align_elems, rows, turbo::kLayerNormLimits, ovr);

    turbo::LayerNormArgs a;
    a.x = x;
    a.residual = residual;
    a.bias = bias;
    a.gamma = gamma;
    a.beta = beta;
    a.out = out;
    a.n_rows = rows;
    a.hidden = hidden;
    a.eps = eps;
    a.inv_hidden = 1.0f / (float)hidden;
    a.lengths = lengths;
    a.S = S;
    a.div_s = turbo::make_fastdiv((unsigned)S);

    turbo::LaunchCfg lc;
    if (int st = launch_cfg(ovr, &lc)) return st;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    hipError_t err = dtype == TURBO_F32 ? turbo::launch_layernorm_f32(plan, a, lc, s)
                                        : turbo::launch_layernorm_f16(plan, a, lc, s);
    return err == hipSuccess ? TURBO_OK : TURBO_ERR_LAUNCH;
}

int gelu_impl(const void* x, const void* bias, int rows, int hidden, int approximate, void* out, int dtype,
              void* stream) {
    if (x == nullptr || out == nullptr) return TURBO_ERR_NULL;
    const int es = elem_size_of(dtype);
    if (es == 0) return TURBO_ERR_DTYPE;
    if (rows <= 0 || hidden <= 0 || hidden > (1 << 27)) return TURBO_ERR_SHAPE;
    const long long total = (long long)rows * hidden;
    const int full_vec = 16 / es;
    if (total / full_vec > 0x7FFFFFFFll) return TURBO_ERR_SHAPE;
    long long align_elems = 16;
    for (const void* p : {x, bias, (const void*)out}) {
        if (p == nullptr) continue;
        if (reinterpret_cast<uintptr_t>(p) % es != 0) return TURBO_ERR_ALIGN;
        align_elems = min_ll(align_elems, byte_alignment(p) / es);
    }
    const turbo::Overrides ovr = current_overrides();
    int vec = full_vec;
    if (ovr.max_vec_bytes >= es && ovr.max_vec_bytes < 16) vec = 1;  // testing hook: the narrow kernel
    if (total < vec) vec = 1;
    const bool under_aligned = vec > 1 && align_elems % vec != 0;

    turbo::GeluArgs a;
    a.x = x;
    a.bias = bias;
    a.out = out;
    a.total = total;
    a.hidden = hidden;
    a.approximate = approximate != 0;
    a.div_hidden = turbo::make_fastdiv((unsigned)hidden);
    a.div_hv = turbo::make_fastdiv((unsigned)(hidden % vec == 0 ? hidden / vec : 1));
    a.rows = rows;
    a.hv = 0;
    a.div_ct = turbo::make_fastdiv(1);
    a.force_flat = ovr.path == 2;  // testing hook, as for the head permutations
    hipError_t err = turbo::launch_add_bias_gelu(a, es, vec, under_aligned, reinterpret_cast<hipStream_t>(stream));
    return err == hipSuccess ? TURBO_OK : TURBO_ERR_LAUNCH;
}

// in [B][N1][K][N2][D] -> out [K][B][N2][N1][D] (+ bias [K][N2][D])
int permute_impl(const void* x, const void* bias, int B, int N1, int K, int N2, int D, void* out, int dtype,
                 int out_order, void* stream) {
    if (x == nullptr || out == nullptr) return TURBO_ERR_NULL;
    const int es = elem_size_of(dtype);
    if (es == 0) return TURBO_ERR_DTYPE;
    if (B <= 0 || N1 <= 0 || K <= 0 || N2 <= 0 || D <= 0) return TURBO_ERR_SHAPE;
    long long total = 1;  // B*N1*K*N2*D, at most 2^40 elements; checked factor by factor so nothing overflows
    for (const int dim : {B, N1, K, N2, D}) {
        if (total > (1ll << 40) / dim) return TURBO_ERR_SHAPE;
        total *= dim;
    }
    long long align_elems = 16;
    for (const void* p : {x, bias, (const void*)out}) {
        if (p == nullptr) continue;
        if (reinterpret_cast<uintptr_t>(p) % es != 0) return TURBO_ERR_ALIGN;
        align_elems = min_ll(align_elems, byte_alignment(p) / es);
    }
    const turbo::Overrides ovr = current_overrides();
    int vec = 16 / es;
    if (ovr.max_vec_bytes >= es && ovr.max_vec_bytes < 16) vec = ovr.max_vec_bytes / es;
    while (vec > 1 && (D % vec != 0 || align_elems % vec != 0)) vec >>= 1;
    if (total / vec > 0x7FFFFFFFll) return TURBO_ERR_SHAPE;

    turbo::PermuteArgs a;
    a.x = x;
    a.bias = bias;
    a.out = out;
    a.total = total;
    a.B = B;
    a.N1 = N1;
    a.K = K;
    a.N2 = N2;
    a.D = D;
    a.div_dv = turbo::make_fastdiv((unsigned)(D / vec));
    a.div_n2 = turbo::make_fastdiv((unsigned)N2);
    a.div_k = turbo::make_fastdiv((unsigned)K);
    a.div_n1 = turbo::make_fastdiv((unsigned)N1);
    a.div_b = turbo::make_fastdiv((unsigned)B);
    a.out_order = out_order;
    // grouped kernel: the unrolled dimension (n2 when walking the output, n1 when walking the input) must divide
    // evenly, and a bias is only supported when it does not depend on that dimension (input order)
    const int unrolled = out_order ? N2 : N1;
    a.grouped = unrolled % turbo::kElemUnroll == 0 && !(bias != nullptr && out_order) && ovr.path != 2;
    a.tiled = ovr.path < 0;  // testing hook: any forced family selects the kernels without LDS
    a.div_n1u = turbo::make_fastdiv((unsigned)(N1 % turbo::kElemUnroll == 0 ? N1 / turbo::kElemUnroll : 1));
    a.div_n2u = turbo::make_fastdiv((unsigned)(N2 % turbo::kElemUnroll == 0 ? N2 / turbo::kElemUnroll : 1));
    hipError_t err = turbo::launch_permute_heads(a, es, vec, reinterpret_cast<hipStream_t>(stream));
    return err == hipSuccess ? TURBO_OK : TURBO_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int turbo_add_bias_gelu(const void* x, const void* bias, int rows, int hidden, int approximate, void* out, int dtype,
                        void* stream) {
    return gelu_impl(x, bias, rows, hidden, approximate, out, dtype, stream);
}

int turbo_add_bias_split_heads(const void* x, const void* bias, int B, int S, int n_split, int H, int D, void* out,
                               int dtype, void* stream) {
    // measured on MI355X: the split streams best walking its input, the merge walking its output
    return permute_impl(x, bias, B, S, n_split, H, D, out, dtype, 0, stream);
}

int turbo_merge_heads(const void* x, int B, int H, int S, int D, void* out, int dtype, void* stream) {
    return permute_impl(x, nullptr, B, H, 1, S, D, out, dtype, 1, stream);
}

int turbo_masked_softmax(void* scores, const void* mask, int B, int H, int Sq, int Sk, float scale, int dtype,
                         void* stream) {
    return softmax_impl(scores, mask, (long long)Sq * Sk, Sk, nullptr, nullptr, B, H, Sq, Sk, scale, dtype, stream);
}

int turbo_masked_softmax_ex(void* scores, const void* mask, long long mask_stride_b, long long mask_stride_q, int B,
                            int H, int Sq, int Sk, float scale, int dtype, void* stream) {
    return softmax_impl(scores, mask, mask_stride_b, mask_stride_q, nullptr, nullptr, B, H, Sq, Sk, scale, dtype, stream);
}

int turbo_masked_softmax_varlen(void* scores, const int* q_lengths, const int* k_lengths, int B, int H, int Sq, int Sk,
                                float scale, int dtype, void* stream) {
    if (k_lengths == nullptr) return TURBO_ERR_NULL;
    return softmax_impl(scores, nullptr, 0, 0, q_lengths, k_lengths, B, H, Sq, Sk, scale, dtype, stream);
}

int turbo_masked_softmax_causal(void* scores, const int* q_lengths, const int* k_lengths, int B, int H, int Sq, int Sk,
                                float scale, int dtype, void* stream) {
    return softmax_impl(scores, nullptr, 0, 0, q_lengths, k_lengths, B, H, Sq, Sk, scale, dtype, stream, 1);
}

int turbo_add_bias_layernorm(const void* x, const void* residual, const void* bias, const void* gamma,
                             const void* beta, int rows, int hidden, float eps, void* out, void* stream) {
    return layernorm_impl(x, residual, bias, gamma, beta, rows, hidden, eps, out, TURBO_F32, stream);
}

int turbo_add_bias_layernorm_dt(const void* x, const void* residual, const void* bias, const void* gamma,
                                const void* beta, int rows, int hidden, float eps, void* out, int dtype,
                                void* stream) {
    return layernorm_impl(x, residual, bias, gamma, beta, rows, hidden, eps, out, dtype, stream);
}

int turbo_add_bias_layernorm_varlen(const void* x, const void* residual, const void* bias, const void* gamma,
                                    const void* beta, const int* lengths, int B, int S, int hidden, float eps,
                                    void* out, int dtype, void* stream) {
    if (lengths == nullptr) return TURBO_ERR_NULL;
    if (B <= 0 || S <= 0 || (long long)B * S > kMaxRows) return TURBO_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(lengths) % 4 != 0) return TURBO_ERR_ALIGN;
    return layernorm_impl(x, residual, bias, gamma, beta, B * S, hidden, eps, out, dtype, stream, lengths, S);
}

int turbo_masked_softmax_packed(void* scores, const int* cu_seqlens, const long long* score_offsets, int B, int H,
                                int total_tokens, int max_len, float scale, int dtype, void* stream) {
    if (scores == nullptr || cu_seqlens == nullptr || score_offsets == nullptr) return TURBO_ERR_NULL;
    const int es = elem_size_of(dtype);
    if (es == 0) return TURBO_ERR_DTYPE;
    if (B <= 0 || H <= 0 || total_tokens <= 0 || max_len <= 0 || max_len > total_tokens) return TURBO_ERR_SHAPE;
    if ((long long)H * total_tokens > kMaxRows) return TURBO_ERR_SHAPE;
    if (max_len > turbo::kPackedBlockMaxLen) return TURBO_ERR_SHAPE;  // a workgroup's registers hold a row
    if (reinterpret_cast<uintptr_t>(scores) % es != 0 || reinterpret_cast<uintptr_t>(cu_seqlens) % 4 != 0 ||
        reinterpret_cast<uintptr_t>(score_offsets) % 8 != 0)
        return TURBO_ERR_ALIGN;
    turbo::PackedSoftmaxArgs a;
    a.scores = scores;
    a.cu_seqlens = cu_seqlens;
    a.score_offsets = score_offsets;
    a.B = B;
    a.H = H;
    a.n_rows = H * total_tokens;
    a.scale = scale;
    a.long_from = 0;
    const turbo::Overrides ovr = current_overrides();
    turbo::LaunchCfg lc;
    if (int st = launch_cfg(ovr, &lc)) return st;
    // testing hooks: TURBO_OVR_PATH = 0 selects the kernel that gives every row a whole wavefront (the one batches of
    // 64 or more requests use), TURBO_OVR_GRID_WAVES caps the grid
    const hipError_t err = turbo::launch_softmax_packed(a, es, max_len, lc.num_cus, ovr.grid_waves > 0 ? ovr.grid_waves : 0,
                                                        ovr.path == 0, reinterpret_cast<hipStream_t>(stream));
    return err == hipSuccess ? TURBO_OK : TURBO_ERR_LAUNCH;
}

const char* turbo_status_string(int status) {
    switch (status) {
        case TURBO_OK: return "ok";
        case TURBO_ERR_NULL: return "a required pointer is NULL";
        case TURBO_ERR_SHAPE: return "a dimension or stride is out of range";
        case TURBO_ERR_DTYPE: return "unknown dtype";
        case TURBO_ERR_ALIGN: return "a pointer is not aligned to its element size";
        case TURBO_ERR_LAUNCH: return "HIP reported an error at kernel launch";
    }
    return "unknown status";
}

int turbo_set_override(int key, int value) {
    if (key < 0 || key >= TURBO_OVR_COUNT_) return TURBO_ERR_SHAPE;
    g_ovr_value[key].store(value, std::memory_order_relaxed);
    return TURBO_OK;
}

int turbo_describe_plan(int op, int rows, int row_len, int dtype, int aligned16, char* buf, int buf_len) {
    if (buf == nullptr) return TURBO_ERR_NULL;
    const int es = elem_size_of(dtype);
    if (es == 0) return TURBO_ERR_DTYPE;
    if ((op != 0 && op != 1) || rows <= 0 || row_len <= 0 || buf_len <= 0) return TURBO_ERR_SHAPE;
    const turbo::OpLimits& lim = op == 0 ? turbo::kSoftmaxLimits : turbo::kLayerNormLimits;
    const turbo::Plan p = turbo::make_plan(row_len, es, aligned16 ? 16 / es : 1, rows, lim, current_overrides());
    turbo::describe_plan(p, buf, buf_len);
    return TURBO_OK;
}

int turbo_stream_probe(const void* in0, const void* in1, void* out, long long n_bytes, void* stream) {
    if (in0 == nullptr || out == nullptr) return TURBO_ERR_NULL;
    // whole 16-byte vectors only; the workgroup count (1024 vectors each) must fit a 31-bit grid
    if (n_bytes <= 0 || n_bytes % 16 != 0 || n_bytes / 16 / 1024 > 0x7FFFFFF0ll) return TURBO_ERR_SHAPE;
    const uintptr_t bits = (uintptr_t)in0 | (uintptr_t)out | (uintptr_t)in1;
    if (bits % 16 != 0) return TURBO_ERR_ALIGN;
    const hipError_t e = turbo::launch_stream_probe((const float*)in0, (const float*)in1, (float*)out, n_bytes / 16,
                                                    (hipStream_t)stream);
    return e == hipSuccess ? TURBO_OK : TURBO_ERR_LAUNCH;
}

unsigned turbo_debug_fastdiv(unsigned n, unsigned d) {
    if (d == 0) return 0;
    return turbo::fastdiv(n, turbo::make_fastdiv(d));
}

}  // extern "C"
