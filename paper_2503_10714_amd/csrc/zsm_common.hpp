// Shared device-side definitions of the ZSMerge cache step (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zsm {

typedef _Float16 f16_t;
struct bf16_t { uint16_t bits; };

// Where one cache lives in the caller's device buffer.  Every array is indexed by the
// global unit number ug = (layer * S + seq) * H + head, slots within a unit by slot index.
struct CacheView {
    int32_t L, S, H, G, D;
    int32_t cap;        // slot stride (slot_capacity)
    int32_t Br;         // residual slots per unit
    int32_t cap_tok;    // cap - Br
    int32_t dtype;
    float lambda, alpha;   // used as (double)lambda, (double)alpha
    double scale;          // logit scale (1/sqrt(d) in fp64 unless the caller set one)
    int32_t* Bp;        // [S]
    int32_t* Bc;        // [S]
    int64_t* n_seen;    // [units]   tokens seen (T)
    int32_t* n_occ;     // [units]   occupied token slots
    int32_t* flags;     // [units]   sticky condition bits (ZSM_FLAG_*), set by the kernels, never cleared by them
    float* s;           // [units][cap]
    int32_t* pos;       // [units][cap]
    int32_t* w;         // [units][cap]
    float* Kr;          // [units][Br][D]
    float* Vr;
    void* Kt;           // [units][cap_tok][D] in kv dtype
    void* Vt;
    // scratch of the split decode step (several workgroups per unit), indexed by the workgroup's
    // or the unit's number inside the launch; sp_max_units / sp_max_wgs bound the launches that may use it
    int32_t sp_max_units, sp_max_wgs;
    double* sp_L;          // [sp_max_wgs][G]         the parts' softmax denominators
    float* sp_acc;         // [sp_max_wgs][G][D]      the parts' outputs, each normalised by its own denominator
    double* sp_E;          // [sp_max_units][G][cap+1] exp(logit - C) of every slot
};

// Condition bits a kernel may raise in CacheView::flags (mirrored by include/zsm.h).
constexpr int32_t FLAG_DECODE_SPREAD = 1;    // decode step: a softmax denominator (relative to the incoming token's own logit) reached SPREAD_FLAG_SUM
constexpr int32_t FLAG_PREFILL_SPREAD = 2;   // prefill scoring: a row's softmax denominator (relative to its own position's logit) reached SPREAD_FLAG_SUM
// exp(logit - reference) is evaluated in fp64, which holds e^709; differences are clamped here
constexpr double LOGIT_SPREAD_MAX = 690.0;
// A sum of such exponentials that reaches e^680 raises the flag: a clamped term alone exceeds it, and sums of
// unclamped terms reach it only when some logit is within ln(number of terms) of 680 above the reference.
constexpr double SPREAD_FLAG_SUM = 1.7e295;   // just under e^680 = 1.77e295

// ---- element access -------------------------------------------------------------------
// load_seg<KT, N>(p, out): N consecutive elements starting at p (16-byte aligned when
// N * sizeof(KT) is a multiple of 16) converted to float.

template <int N>
__device__ __forceinline__ void load_seg(const float* p, float* out) {
    static_assert(N % 4 == 0, "");
#pragma unroll
    for (int i = 0; i < N / 4; ++i) {
        const float4 v = reinterpret_cast<const float4*>(p)[i];
        out[4 * i + 0] = v.x; out[4 * i + 1] = v.y; out[4 * i + 2] = v.z; out[4 * i + 3] = v.w;
    }
}

template <int N>
__device__ __forceinline__ void load_seg(const f16_t* p, float* out) {
    static_assert(N % 8 == 0, "");
    typedef f16_t h8 __attribute__((ext_vector_type(8)));
#pragma unroll
    for (int i = 0; i < N / 8; ++i) {
        const h8 v = reinterpret_cast<const h8*>(p)[i];
#pragma unroll
        for (int e = 0; e < 8; ++e) out[8 * i + e] = (float)v[e];
    }
}

template <int N>
__device__ __forceinline__ void load_seg(const bf16_t* p, float* out) {
    static_assert(N % 8 == 0, "");
#pragma unroll
    for (int i = 0; i < N / 8; ++i) {
        const uint4 v = reinterpret_cast<const uint4*>(p)[i];
        const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            out[8 * i + 2 * e + 0] = __uint_as_float(d[e] << 16);
            out[8 * i + 2 * e + 1] = __uint_as_float(d[e] & 0xffff0000u);
        }
    }
}

// load_nt: the same load marked non-temporal, for rows that are read once per kernel and whole (a wave-wide load
// covers complete rows): the lines then pass through the caches without displacing anything, which on this chip
// raises the rate of a streaming sweep by about an eighth.  Not for loads that take a row in pieces at different
// times (the line has to stay for the later pieces).
// Raw<KT, N>: the register image of N consecutive elements (N * sizeof(KT) is a multiple
// of 16): loaded with 16-byte loads, converted element by element only where it is used.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef f16_t f16x8_t __attribute__((ext_vector_type(8)));

template <typename KT, int N> struct Raw;
template <int N> struct Raw<float, N> {
    f32x4_t v[N / 4];
    __device__ __forceinline__ void load(const float* p) {
#pragma unroll
        for (int i = 0; i < N / 4; ++i) v[i] = reinterpret_cast<const f32x4_t*>(p)[i];
    }
    __device__ __forceinline__ void load_nt(const float* p) {
#pragma unroll
        for (int i = 0; i < N / 4; ++i) v[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p) + i);
    }
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int i = 0; i < N / 4; ++i) v[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    __device__ __forceinline__ float get(int e) const { return v[e / 4][e % 4]; }
};
template <int N> struct Raw<f16_t, N> {
    f16x8_t v[N / 8];
    __device__ __forceinline__ void load(const f16_t* p) {
#pragma unroll
        for (int i = 0; i < N / 8; ++i) v[i] = reinterpret_cast<const f16x8_t*>(p)[i];
    }
    __device__ __forceinline__ void load_nt(const f16_t* p) {
#pragma unroll
        for (int i = 0; i < N / 8; ++i) v[i] = __builtin_nontemporal_load(reinterpret_cast<const f16x8_t*>(p) + i);
    }
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int i = 0; i < N / 8; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e) v[i][e] = (f16_t)0;
    }
    __device__ __forceinline__ float get(int e) const { return (float)v[e / 8][e % 8]; }
};
template <int N> struct Raw<bf16_t, N> {
    u32x4_t v[N / 8];
    __device__ __forceinline__ void load(const bf16_t* p) {
#pragma unroll
        for (int i = 0; i < N / 8; ++i) v[i] = reinterpret_cast<const u32x4_t*>(p)[i];
    }
    __device__ __forceinline__ void load_nt(const bf16_t* p) {
#pragma unroll
        for (int i = 0; i < N / 8; ++i) v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p) + i);
    }
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int i = 0; i < N / 8; ++i) v[i] = u32x4_t{0u, 0u, 0u, 0u};
    }
    __device__ __forceinline__ float get(int e) const {
        const uint32_t d = v[e / 8][(e % 8) / 2];
        return __uint_as_float((e & 1) ? (d & 0xffff0000u) : (d << 16));
    }
};

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(f16_t x) { return (float)x; }
__device__ __forceinline__ float to_float(bf16_t x) { return __uint_as_float(((uint32_t)x.bits) << 16); }

// ---- wave-level helpers (64 lanes) ----------------------------------------------------

// Orders LDS traffic between lanes of one wave: a later read by any lane sees an earlier
// write by any lane (LDS executes a wave's instructions in order; this only stops the
// compiler from moving them).
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ unsigned long long wave_min(unsigned long long v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const unsigned long long t = __shfl_xor(v, o, 64);
        v = t < v ? t : v;
    }
    return v;
}

}  // namespace zsm
