// C ABI of the library: argument validation, variant choice, launch.
// Validation runs before the first HIP call, so every error except
// TURBO_ERR_LAUNCH is reported without a GPU.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>

#include "../../include/turbo_reduce.h"
#include "layernorm_kernels.h"
#include "plan.h"
#include "softmax_kernels.h"

namespace {

turbo::Overrides g_ovr;

constexpr int kMaxRows = 0x7FFF0000;  // leaves headroom for tile rounding in 32-bit row indices
constexpr int kMaxDevices = 64;
int g_num_cus[kMaxDevices];

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

int current_num_cus(int* out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return TURBO_ERR_LAUNCH;
    if (dev < 0 || dev >= kMaxDevices) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            return TURBO_ERR_LAUNCH;
        *out = n;
        return TURBO_OK;
    }
    if (g_num_cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            return TURBO_ERR_LAUNCH;
        g_num_cus[dev] = n;
    }
    *out = g_num_cus[dev];
    return TURBO_OK;
}

turbo::LaunchCfg launch_cfg(int num_cus) {
    turbo::LaunchCfg lc;
    lc.num_cus = num_cus;
    lc.waves_per_cu = g_ovr.grid_waves > 0 ? (g_ovr.grid_waves > (1 << 20) ? (1 << 22) : g_ovr.grid_waves * 4) : 0;
    return lc;
}

int softmax_impl(void* scores, const void* mask, long long msb, long long msq, int B, int H, int Sq, int Sk,
                 float scale, int dtype, void* stream) {
    if (scores == nullptr) return TURBO_ERR_NULL;
    const int es = elem_size_of(dtype);
    if (es == 0) return TURBO_ERR_DTYPE;
    if (B <= 0 || H <= 0 || Sq <= 0 || Sk <= 0) return TURBO_ERR_SHAPE;
    const long long n_rows = (long long)B * H * Sq;
    if ((long long)H * Sq > kMaxRows || n_rows > kMaxRows) return TURBO_ERR_SHAPE;
    if (mask != nullptr && (msb < 0 || msq < 0)) return TURBO_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(scores) % es != 0) return TURBO_ERR_ALIGN;
    if (mask != nullptr && reinterpret_cast<uintptr_t>(mask) % es != 0) return TURBO_ERR_ALIGN;

    long long align_elems = byte_alignment(scores) / es;
    if (mask != nullptr) {
        align_elems = min_ll(align_elems, byte_alignment(mask) / es);
        align_elems = min_ll(align_elems, stride_alignment(msb));
        align_elems = min_ll(align_elems, stride_alignment(msq));
    }
    const turbo::Plan plan = turbo::make_plan(Sk, es, align_elems, n_rows, turbo::kSoftmaxLimits, g_ovr);

    turbo::SoftmaxArgs a;
    a.scores = scores;
    a.mask = mask;
    a.mask_stride_b = msb;
    a.mask_stride_q = msq;
    a.n_rows = (int)n_rows;
    a.Sq = Sq;
    a.Sk = Sk;
    a.scale = scale;
    a.div_rows_per_batch = turbo::make_fastdiv((unsigned)((long long)H * Sq));
    a.div_sq = turbo::make_fastdiv((unsigned)Sq);

    int num_cus = 0;
    if (int st = current_num_cus(&num_cus)) return st;
    const turbo::LaunchCfg lc = launch_cfg(num_cus);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    hipError_t err = dtype == TURBO_F32 ? turbo::launch_softmax_f32(plan, a, lc, s)
                                        : turbo::launch_softmax_f16(plan, a, lc, s);
    return err == hipSuccess ? TURBO_OK : TURBO_ERR_LAUNCH;
}

int layernorm_impl(const void* x, const void* residual, const void* bias, const void* gamma, const void* beta,
                   int rows, int hidden, float eps, void* out, int dtype, void* stream) {
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
    const turbo::Plan plan = turbo::make_plan(hidden, es, align_elems, rows, turbo::kLayerNormLimits, g_ovr);

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

    int num_cus = 0;
    if (int st = current_num_cus(&num_cus)) return st;
    const turbo::LaunchCfg lc = launch_cfg(num_cus);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    hipError_t err = dtype == TURBO_F32 ? turbo::launch_layernorm_f32(plan, a, lc, s)
                                        : turbo::launch_layernorm_f16(plan, a, lc, s);
    return err == hipSuccess ? TURBO_OK : TURBO_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int turbo_masked_softmax(void* scores, const void* mask, int B, int H, int Sq, int Sk, float scale, int dtype,
                         void* stream) {
    return softmax_impl(scores, mask, (long long)Sq * Sk, Sk, B, H, Sq, Sk, scale, dtype, stream);
}

int turbo_masked_softmax_ex(void* scores, const void* mask, long long mask_stride_b, long long mask_stride_q, int B,
                            int H, int Sq, int Sk, float scale, int dtype, void* stream) {
    return softmax_impl(scores, mask, mask_stride_b, mask_stride_q, B, H, Sq, Sk, scale, dtype, stream);
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
    switch (key) {
        case TURBO_OVR_PATH: g_ovr.path = value; return TURBO_OK;
        case TURBO_OVR_MAX_VEC_BYTES: g_ovr.max_vec_bytes = value; return TURBO_OK;
        case TURBO_OVR_GRID_WAVES: g_ovr.grid_waves = value; return TURBO_OK;
    }
    return TURBO_ERR_SHAPE;
}

int turbo_describe_plan(int op, int rows, int row_len, int dtype, int aligned16, char* buf, int buf_len) {
    if (buf == nullptr) return TURBO_ERR_NULL;
    const int es = elem_size_of(dtype);
    if (es == 0) return TURBO_ERR_DTYPE;
    if ((op != 0 && op != 1) || rows <= 0 || row_len <= 0 || buf_len <= 0) return TURBO_ERR_SHAPE;
    const turbo::OpLimits& lim = op == 0 ? turbo::kSoftmaxLimits : turbo::kLayerNormLimits;
    const turbo::Plan p = turbo::make_plan(row_len, es, aligned16 ? 16 / es : 1, rows, lim, g_ovr);
    turbo::describe_plan(p, buf, buf_len);
    return TURBO_OK;
}

unsigned turbo_debug_fastdiv(unsigned n, unsigned d) {
    if (d == 0) return 0;
    return turbo::fastdiv(n, turbo::make_fastdiv(d));
}

}  // extern "C"
