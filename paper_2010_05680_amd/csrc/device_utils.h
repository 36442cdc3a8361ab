// Device-side building blocks shared by the softmax and LayerNorm kernels:
// packed loads/stores, wave64 lane exchanges, group all-reduces.
//
// The paper's kernel-level idea (Section 4.1.2) is to reduce X independent
// rows together so that the lane-exchange latency of one row hides behind the
// arithmetic of the others and one synchronisation serves X results.  Here the
// same idea is expressed for 64-wide wavefronts: every exchange helper below is
// called for R rows back to back, which gives the scheduler R independent
// DPP / permlane chains to interleave.
#pragma once
#include <hip/hip_runtime.h>

namespace turbo {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;

// VEC elements of T moved by one load/store instruction (2..16 bytes).
template <typename T, int VEC>
struct alignas(sizeof(T) * VEC) Pack {
    T v[VEC];
};

// Streamed tensors (scores, x, residual, out) are touched exactly once per
// launch, so their loads and stores carry the non-temporal hint; small operands
// that every row re-reads (mask rows, bias, gamma, beta) use plain loads.
#ifndef TURBO_NT_LOADS
#define TURBO_NT_LOADS 1
#endif
#ifndef TURBO_NT_STORES
#define TURBO_NT_STORES 1
#endif

// Vector register type for VEC elements of T.  UA ("under-aligned") declares the
// memory operand aligned to one element only: gfx950 executes 16-byte global
// loads and stores at any element-aligned address, which keeps rows whose
// length is not a multiple of the vector width on the wide-access path.
template <typename T, int VEC, bool UA>
struct VecType {
    typedef T reg __attribute__((ext_vector_type(VEC)));
    typedef reg mem __attribute__((aligned(UA ? sizeof(T) : sizeof(T) * VEC)));
};
template <typename T, bool UA>
struct VecType<T, 1, UA> {
    typedef T reg;
    typedef T mem;
};

// plain load: data with reuse
template <typename T, int VEC, bool UA = false>
__device__ __forceinline__ Pack<T, VEC> load_pack(const T* p) {
    using V = VecType<T, VEC, UA>;
    typename V::reg v = *reinterpret_cast<const typename V::mem*>(p);
    return __builtin_bit_cast(Pack<T, VEC>, v);
}
// streaming load / store: data used once
template <typename T, int VEC, bool UA = false>
__device__ __forceinline__ Pack<T, VEC> load_stream(const T* p) {
    using V = VecType<T, VEC, UA>;
#if TURBO_NT_LOADS
    typename V::reg v = __builtin_nontemporal_load(reinterpret_cast<const typename V::mem*>(p));
#else
    typename V::reg v = *reinterpret_cast<const typename V::mem*>(p);
#endif
    return __builtin_bit_cast(Pack<T, VEC>, v);
}
template <typename T, int VEC, bool UA = false>
__device__ __forceinline__ void store_stream(T* p, const Pack<T, VEC>& v) {
    using V = VecType<T, VEC, UA>;
#if TURBO_NT_STORES
    __builtin_nontemporal_store(__builtin_bit_cast(typename V::reg, v), reinterpret_cast<typename V::mem*>(p));
#else
    *reinterpret_cast<typename V::mem*>(p) = __builtin_bit_cast(typename V::reg, v);
#endif
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ float fast_rsqrt(float x) { return __builtin_amdgcn_rsqf(x); }

// ---- lane exchanges --------------------------------------------------------
// exchange<S>(v, a, b) hands every lane the pair of values held by itself and by
// its partner at distance S inside an aligned group of 2*S lanes.  Which of
// (a, b) is the lane's own value is unspecified; callers combine a and b with a
// symmetric rule.  After log2(G) exchanges, S = 1, 2, ..., G/2, a symmetric
// combine has visited all G lanes of the group (an all-reduce).
//
//   S = 1, 2 : DPP quad permutes (xor 1, xor 2).
//   S = 4    : DPP row_half_mirror (lane i <-> 7-i of each 8).  The partner is
//              in the other quad, which is all that matters once quads agree.
//   S = 8    : DPP row_mirror (lane i <-> 15-i of each 16), same argument.
//   S = 16   : v_permlane16_swap: rows (16 lanes) 1,3 of the first operand are
//              swapped with rows 0,2 of the second; with both operands = v the
//              two results hold row pairs {r0,r0,r2,r2} and {r1,r1,r3,r3}.
//   S = 32   : v_permlane32_swap: {r0,r1,r0,r1} and {r2,r3,r2,r3}.
// No exchange goes through LDS.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}

template <int S>
__device__ __forceinline__ void exchange(float v, float& a, float& b) {
    static_assert(S == 1 || S == 2 || S == 4 || S == 8 || S == 16 || S == 32, "lane distance");
    if constexpr (S == 1) {
        a = v;
        b = dpp_move<0xB1>(v);  // quad_perm [1,0,3,2]
    } else if constexpr (S == 2) {
        a = v;
        b = dpp_move<0x4E>(v);  // quad_perm [2,3,0,1]
    } else if constexpr (S == 4) {
        a = v;
        b = dpp_move<0x141>(v);  // row_half_mirror
    } else if constexpr (S == 8) {
        a = v;
        b = dpp_move<0x140>(v);  // row_mirror
    } else if constexpr (S == 16) {
        const unsigned u = __builtin_bit_cast(unsigned, v);
        auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
        const unsigned r0 = r[0], r1 = r[1];  // scalars first: a bit_cast applied to r[1] directly reads r[0]
        a = __builtin_bit_cast(float, r0);
        b = __builtin_bit_cast(float, r1);
    } else {
        const unsigned u = __builtin_bit_cast(unsigned, v);
        auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
        const unsigned r0 = r[0], r1 = r[1];
        a = __builtin_bit_cast(float, r0);
        b = __builtin_bit_cast(float, r1);
    }
}

struct MaxOp {
    __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); }
};
struct SumOp {
    __device__ __forceinline__ float operator()(float a, float b) const { return a + b; }
};

template <int S, int G, int R, typename Op>
__device__ __forceinline__ void allreduce_step(float (&v)[R], Op op) {
    if constexpr (S < G) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float a, b;
            exchange<S>(v[r], a, b);
            v[r] = op(a, b);
        }
        allreduce_step<S * 2, G, R>(v, op);
    }
}

// All-reduce of R independent values over aligned groups of G lanes (G a power
// of two, 1..64).  The R chains of each step are issued together.
template <int G, int R, typename Op>
__device__ __forceinline__ void group_allreduce(float (&v)[R], Op op) {
    allreduce_step<1, G, R>(v, op);
}

// ---- exact unsigned division by a runtime constant -------------------------
// q = n / d for 0 <= n < 2^31, d >= 1, via one multiply-high, one add and one
// shift (round-up magic number: m = floor(2^32 (2^s - d) / d) + 1, s = ceil(log2 d)).
struct FastDiv {
    unsigned mul;
    unsigned shift;
    unsigned d;
};

inline FastDiv make_fastdiv(unsigned d) {
    FastDiv f;
    f.d = d;
    unsigned s = 0;
    while ((1ull << s) < d) ++s;
    f.shift = s;
    f.mul = (unsigned)(((1ull << 32) * ((1ull << s) - d)) / d + 1);
    return f;
}

__host__ __device__ __forceinline__ unsigned fastdiv(unsigned n, const FastDiv& f) {
#if defined(__HIP_DEVICE_COMPILE__)
    unsigned hi = __umulhi(n, f.mul);
#else
    unsigned hi = (unsigned)(((unsigned long long)n * f.mul) >> 32);
#endif
    return (hi + n) >> f.shift;
}

}  // namespace turbo
