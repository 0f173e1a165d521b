// Host side of the C ABI declared in include/zsm.h: argument checks, cache layout,
// launches.  No device memory is allocated or freed here.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/zsm.h"
#include "zsm_common.hpp"
#include "zsm_decode.hpp"
#include "zsm_prefill.hpp"

using namespace zsm;

struct zsm_cache {
    zsm_config_t cfg;
    CacheView cv;
    std::vector<int32_t> Bp, Bc;
    size_t bytes;
    int max_btok;   // max over sequences of B_p + B_c
    int32_t* dbg;   // device: one counter for the optional state checks
    int parts;      // workgroups per unit in the decode step: 0 = chosen per launch, 1 = never split, n = n
};

namespace {

thread_local char g_hip_msg[256] = "no HIP error recorded";

int hip_fail(hipError_t e, const char* what) {
    std::snprintf(g_hip_msg, sizeof(g_hip_msg), "%s: %s", what, hipGetErrorString(e));
    return ZSM_E_HIP;
}

size_t esize(int dtype) { return dtype == ZSM_F32 ? 4 : 2; }
size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

bool config_ok(const zsm_config_t* c) {
    if (!c) return false;
    if (c->n_layers < 1 || c->n_seqs < 1 || c->n_kv_heads < 1) return false;
    if (c->q_per_kv < 1 || c->q_per_kv > ZSM_MAX_Q_PER_KV) return false;
    if (!(c->head_dim == 64 || c->head_dim == 128)) return false;
    if (c->n_residual < 0 || c->slot_capacity < c->n_residual + 1) return false;
    if (!(c->lambda >= 0.f && c->lambda <= 1.f) || !(c->alpha >= 0.f && c->alpha <= 1.f)) return false;
    if (!(c->scale >= 0.f)) return false;
    if ((int64_t)c->n_layers * c->n_seqs * c->n_kv_heads > (int64_t)0x7fffffff) return false;
    return true;
}

// Launches of the decode step that may be split over several workgroups per unit: at most
// SP_MAX_UNITS units and SP_MAX_WGS workgroups (their partial results live in the cache buffer).
constexpr int SP_MAX_UNITS = 1024;
constexpr int SP_MAX_WGS = 8192;
constexpr int SP_MAX_PARTS = 64;
constexpr int SP_TARGET_WGS = 512;    // what an automatically split launch aims at (2 per compute unit: measured best)

// Section offsets inside the caller's buffer.
struct Layout {
    size_t Bp, Bc, n_seen, n_occ, flags, dbg, s, pos, w, Kr, Vr, Kt, Vt, sp_L, sp_acc, sp_E, total;
    int sp_max_units, sp_max_wgs;
};

// Scratch of a split decode launch of n_wgs workgroups over n_units units: offsets from a
// 256-byte aligned base, and the total.
struct SplitScratch { size_t L, acc, E, total; };
// (e_slices: arrays of cap + 1 doubles per unit in E; G of them for a split launch, one per share of heads for a
// step over more than eight query heads)
SplitScratch split_scratch(size_t n_wgs, size_t n_units, size_t G, size_t D, size_t cap, size_t e_slices = 0) {
    SplitScratch x{};
    size_t o = 0;
    x.L = o; o += up256(sizeof(double) * n_wgs * G);
    x.acc = o; o += up256(sizeof(float) * n_wgs * G * D);
    x.E = o; o += up256(sizeof(double) * n_units * (e_slices > G ? e_slices : G) * (cap + 1));
    x.total = o;
    return x;
}

// heads per workgroup of a step over more than eight query heads per KV head: 8, 4, or 0 where neither fits the LDS
int pool_share_heads(int dtype, int D, int cap) {
    switch (dtype) {
        case ZSM_F32: return decode_pool_share_heads_f32(D, cap + 1);
        case ZSM_F16: return decode_pool_share_heads_f16(D, cap + 1);
        default: return decode_pool_share_heads_bf16(D, cap + 1);
    }
}

// slices of pooled per-slot sums a unit needs (0: at most eight query heads, no pooled step)
size_t pool_slices(const zsm_config_t& c) {
    if (c.q_per_kv <= 8) return 0;
    const int gs = pool_share_heads(c.kv_dtype, c.head_dim, c.slot_capacity);
    return gs > 0 ? (size_t)(c.q_per_kv + gs - 1) / gs : 0;
}

Layout make_layout(const zsm_config_t& c) {
    const size_t units = (size_t)c.n_layers * c.n_seqs * c.n_kv_heads;
    const size_t cap = c.slot_capacity, Br = c.n_residual, D = c.head_dim;
    Layout l{};
    size_t o = 0;
    l.Bp = o; o += up256(sizeof(int32_t) * c.n_seqs);
    l.Bc = o; o += up256(sizeof(int32_t) * c.n_seqs);
    l.n_seen = o; o += up256(sizeof(int64_t) * units);
    l.n_occ = o; o += up256(sizeof(int32_t) * units);
    l.flags = o; o += up256(sizeof(int32_t) * units);
    l.dbg = o; o += 256;                                  // one counter for the optional state checks
    l.s = o; o += up256(sizeof(float) * units * cap);
    l.pos = o; o += up256(sizeof(int32_t) * units * cap);
    l.w = o; o += up256(sizeof(int32_t) * units * cap);
    l.Kr = o; o += up256(sizeof(float) * units * Br * D);
    l.Vr = o; o += up256(sizeof(float) * units * Br * D);
    l.Kt = o; o += up256(esize(c.kv_dtype) * units * (cap - Br) * D);
    l.Vt = o; o += up256(esize(c.kv_dtype) * units * (cap - Br) * D);
    l.sp_max_units = (int)(units < (size_t)SP_MAX_UNITS ? units : (size_t)SP_MAX_UNITS);
    l.sp_max_wgs = l.sp_max_units * SP_MAX_PARTS < SP_MAX_WGS ? l.sp_max_units * SP_MAX_PARTS : SP_MAX_WGS;
    const SplitScratch sp = split_scratch(l.sp_max_wgs, l.sp_max_units, decode_compiled_heads(c.q_per_kv), D, cap,
                                          pool_slices(c));
    l.sp_L = o + sp.L; l.sp_acc = o + sp.acc; l.sp_E = o + sp.E;
    o += sp.total;
    l.total = o;
    return l;
}

// ---- small kernels ---------------------------------------------------------------------

__global__ void fill_i32_kernel(int32_t* p, size_t n, int32_t v) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// after an import: count the occupied token slots of every unit of one layer
__global__ void recount_kernel(CacheView cv, int unit0) {
    const int ug = unit0 + blockIdx.x;
    const int b = (ug / cv.H) % cv.S;
    const int ntok = cv.Bp[b] + cv.Bc[b];
    const int32_t* pos = cv.pos + (size_t)ug * cv.cap + cv.Br;
    int n = 0;
    for (int j = threadIdx.x; j < ntok; j += blockDim.x) n += pos[j] >= 0;
    __shared__ int red[4];
    for (int o = 32; o > 0; o >>= 1) n += __shfl_xor(n, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = n;
    __syncthreads();
    if (threadIdx.x == 0) cv.n_occ[ug] = red[0] + red[1] + red[2] + red[3];
}

__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t n16, float* sink) {
    float acc = 0.f;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n16; i += stride) {
        const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src) + i);   // read once: the fastest plain read on this chip
        acc += __uint_as_float(v[0] ^ v[1] ^ v[2] ^ v[3]);
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0 && acc == 123.456f) sink[0] = acc;   // practically never taken; keeps the loads live
}

__global__ __launch_bounds__(256) void stream_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// ---- optional state checks (zsm_set_debug_checks) ------------------------------------------
std::atomic<int> g_debug_checks{0};

// counts the units of one layer that are not empty (a token seen, or an occupied slot)
__global__ void check_empty_kernel(CacheView cv, int unit0, int32_t* bad) {
    const int ug = unit0 + blockIdx.x;
    int n = 0;
    if (threadIdx.x == 0) n += cv.n_seen[ug] != 0 || cv.n_occ[ug] != 0;
    for (int j = threadIdx.x; j < cv.cap; j += blockDim.x)
        n += cv.w[(size_t)ug * cv.cap + j] != 0 || cv.pos[(size_t)ug * cv.cap + j] != -1;
    if (n) atomicAdd(bad, 1);
}

// counts the slots of one layer that break what zsm_cache_import asks of a state; an array the
// caller does not pass is taken from the cache (the state after the import is what is checked)
__global__ void check_import_kernel(CacheView cv, int unit0, const int32_t* pos_u, const int32_t* w_u,
                                    const int64_t* n_seen_u, int32_t* bad) {
    const int lu = blockIdx.x, ug = unit0 + lu;
    const int b = (ug / cv.H) % cv.S;
    const int B = cv.Bp[b] + cv.Bc[b] + cv.Br;
    const int32_t* pos = pos_u ? pos_u + (size_t)lu * cv.cap : cv.pos + (size_t)ug * cv.cap;
    const int32_t* w = w_u ? w_u + (size_t)lu * cv.cap : cv.w + (size_t)ug * cv.cap;
    const long long T = n_seen_u ? n_seen_u[lu] : cv.n_seen[ug];
    int n = threadIdx.x == 0 && T < 0;
    for (int j = threadIdx.x; j < cv.cap; j += blockDim.x) {
        const int p = pos[j], c = w[j];
        bool ok = c >= 0 && p >= -1 && (c == 0) == (p == -1);   // empty exactly where no position is recorded
        if (p >= 0) ok = ok && (long long)p < T;                  // positions lie below the tokens seen
        if (j >= cv.Br) ok = ok && c <= 1;          // a token slot holds one token
        if (j >= B) ok = ok && c == 0;              // slots past the sequence's budget stay empty
        n += !ok;
    }
    if (n) atomicAdd(bad, n);
}

// runs one of the checks: clears the counter, launches, waits for the stream, reads the counter back
template <typename Launch>
int run_state_check(zsm_cache_t* c, hipStream_t st, Launch launch, const char* what) {
    hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(64), 0, st, c->dbg, (size_t)1, 0);
    launch();
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, what);
    int32_t bad = 0;
    e = hipMemcpyAsync(&bad, c->dbg, sizeof(bad), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_fail(e, what);
    return bad ? ZSM_E_STATE : ZSM_OK;
}

// Workgroups per unit for a decode launch of n_units units (and the token rows one part's LDS
// must hold), or a negative status when no permitted cut fits the LDS.
int pool_share_heads(const CacheView& v) { return pool_share_heads(v.dtype, v.D, v.cap); }

int choose_parts(const zsm_cache_t* cache, int n_units, int* part_rows) {
    const CacheView& v = cache->cv;
    if (v.G > 8) {   // shares of eight heads, each one workgroup per unit: never cut over workgroups
        *part_rows = 0;
        return pool_share_heads(v) > 0 ? 1 : ZSM_E_SHAPE;   // shares of eight heads, else of four
    }
    auto lds_of = [&](int nz) {
        switch (v.dtype) {
            case ZSM_F32: return decode_lds_f32(v.D, v.G, nz);
            case ZSM_F16: return decode_lds_f16(v.D, v.G, nz);
            default: return decode_lds_bf16(v.D, v.G, nz);
        }
    };
    // a launch of few units is cut into parts so that it still fills the chip
    const int R = decode_tile_rows(v.D, (int)esize(v.dtype));
    const int ntiles = (cache->max_btok + R - 1) / R;
    const bool can_split = n_units <= v.sp_max_units;
    int hi = can_split ? v.sp_max_wgs / n_units : 1;              // most parts this launch may have
    hi = hi < SP_MAX_PARTS ? hi : SP_MAX_PARTS;
    hi = hi < ntiles ? hi : ntiles;
    hi = hi > 1 ? hi : 1;
    int parts = cache->parts;
    if (parts == 0) {
        parts = SP_TARGET_WGS / n_units;
        const int by_work = ntiles / (2 * DECODE_NW);             // at least two tiles per wave and part
        parts = parts < by_work ? parts : by_work;
    }
    parts = parts < hi ? parts : hi;
    parts = parts > 1 ? parts : 1;
    auto rows_of = [&](int p) { return (ntiles + p - 1) / p * R; };
    auto lds_need = [&](int p) { return p > 1 ? lds_of(rows_of(p) + v.Br + 1) : lds_of(v.cap + 1); };
    if (cache->parts == 0 && lds_need(parts) > 160 * 1024) {
        // a capacity one workgroup's LDS cannot hold: more parts, and then as many as let the compute unit hold the
        // workgroups its registers allow (4 of a single query head, 3 of four heads, 2 otherwise)
        while (lds_need(parts) > 160 * 1024 && parts < hi) ++parts;
        const size_t want = v.G == 1 ? 4 : (decode_compiled_heads(v.G) == 4 ? 3 : 2);
        while (160 * 1024 / lds_need(parts) < want && parts < hi && parts < ntiles / (2 * DECODE_NW)) ++parts;
    }
    if (lds_need(parts) > 160 * 1024) return ZSM_E_SHAPE;
    *part_rows = parts > 1 ? rows_of(parts) : 0;
    return parts;
}

int check_layer(const zsm_cache_t* c, int layer) {
    if (!c) return ZSM_E_NULL;
    if (layer < 0 || layer >= c->cfg.n_layers) return ZSM_E_RANGE;
    return ZSM_OK;
}

}  // namespace

extern "C" {

size_t zsm_cache_bytes(const zsm_config_t* cfg) {
    if (!config_ok(cfg) || cfg->kv_dtype < ZSM_F32 || cfg->kv_dtype > ZSM_BF16) return 0;
    return make_layout(*cfg).total;
}

int zsm_cache_alloc(const zsm_config_t* cfg, const int32_t* B_p, const int32_t* B_c, void* dev_buf,
                    size_t dev_bytes, void* stream, zsm_cache_t** out) {
    if (!cfg || !B_p || !B_c || !dev_buf || !out) return ZSM_E_NULL;
    if (cfg->kv_dtype < ZSM_F32 || cfg->kv_dtype > ZSM_BF16) return ZSM_E_DTYPE;
    if (!config_ok(cfg)) return ZSM_E_SHAPE;
    int max_btok = 0;
    for (int b = 0; b < cfg->n_seqs; ++b) {
        if (B_p[b] < 1 || B_c[b] < 0) return ZSM_E_SHAPE;
        if ((int64_t)B_p[b] + B_c[b] + cfg->n_residual > cfg->slot_capacity) return ZSM_E_SHAPE;
        max_btok = B_p[b] + B_c[b] > max_btok ? B_p[b] + B_c[b] : max_btok;
    }
    if ((reinterpret_cast<uintptr_t>(dev_buf) & 255) != 0) return ZSM_E_ALIGN;
    const Layout lay = make_layout(*cfg);
    if (dev_bytes < lay.total) return ZSM_E_NOMEM;

    zsm_cache_t* c = new (std::nothrow) zsm_cache_t();
    if (!c) return ZSM_E_NOMEM;
    c->cfg = *cfg;
    c->Bp.assign(B_p, B_p + cfg->n_seqs);
    c->Bc.assign(B_c, B_c + cfg->n_seqs);
    c->bytes = lay.total;
    c->max_btok = max_btok;
    char* base = static_cast<char*>(dev_buf);
    CacheView& v = c->cv;
    v.L = cfg->n_layers; v.S = cfg->n_seqs; v.H = cfg->n_kv_heads; v.G = cfg->q_per_kv; v.D = cfg->head_dim;
    v.cap = cfg->slot_capacity; v.Br = cfg->n_residual; v.cap_tok = v.cap - v.Br; v.dtype = cfg->kv_dtype;
    v.lambda = cfg->lambda; v.alpha = cfg->alpha;
    v.scale = cfg->scale > 0.f ? (double)cfg->scale : 1.0 / std::sqrt((double)cfg->head_dim);
    v.Bp = reinterpret_cast<int32_t*>(base + lay.Bp);
    v.Bc = reinterpret_cast<int32_t*>(base + lay.Bc);
    v.n_seen = reinterpret_cast<int64_t*>(base + lay.n_seen);
    v.n_occ = reinterpret_cast<int32_t*>(base + lay.n_occ);
    v.flags = reinterpret_cast<int32_t*>(base + lay.flags);
    c->dbg = reinterpret_cast<int32_t*>(base + lay.dbg);
    v.s = reinterpret_cast<float*>(base + lay.s);
    v.pos = reinterpret_cast<int32_t*>(base + lay.pos);
    v.w = reinterpret_cast<int32_t*>(base + lay.w);
    v.Kr = reinterpret_cast<float*>(base + lay.Kr);
    v.Vr = reinterpret_cast<float*>(base + lay.Vr);
    v.Kt = base + lay.Kt;
    v.Vt = base + lay.Vt;
    v.sp_max_units = lay.sp_max_units; v.sp_max_wgs = lay.sp_max_wgs;
    v.sp_L = reinterpret_cast<double*>(base + lay.sp_L);
    v.sp_acc = reinterpret_cast<float*>(base + lay.sp_acc);
    v.sp_E = reinterpret_cast<double*>(base + lay.sp_E);
    c->parts = 0;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t units = (size_t)v.L * v.S * v.H;
    hipError_t e;
    // budgets: pageable host -> device copies are staged by the runtime before the call returns
    e = hipMemcpyAsync(v.Bp, c->Bp.data(), sizeof(int32_t) * v.S, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync(v.Bc, c->Bc.data(), sizeof(int32_t) * v.S, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) { delete c; return hip_fail(e, "zsm_cache_alloc budgets"); }
    // empty state: pos = -1, everything else 0 (fill kernels, no memset nodes)
    const size_t n_zero_words = (lay.pos - lay.n_seen) / 4;   // n_seen, n_occ, flags, check counter, s
    hipLaunchKernelGGL(fill_i32_kernel, dim3(1024), dim3(256), 0, st, reinterpret_cast<int32_t*>(base + lay.n_seen), n_zero_words, 0);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(1024), dim3(256), 0, st, v.pos, units * v.cap, -1);
    const size_t n_rest_words = (lay.total - lay.w) / 4;      // w, Kr, Vr, Kt, Vt, split scratch
    hipLaunchKernelGGL(fill_i32_kernel, dim3(1024), dim3(256), 0, st, v.w, n_rest_words, 0);
    e = hipGetLastError();
    if (e != hipSuccess) { delete c; return hip_fail(e, "zsm_cache_alloc init"); }
    *out = c;
    return ZSM_OK;
}

int zsm_cache_free(zsm_cache_t* cache) {
    if (!cache) return ZSM_E_NULL;
    delete cache;
    return ZSM_OK;
}

// Shared body of the decode entry points.  `scratch` = NULL: a split launch keeps its partial results in the
// cache buffer's own scratch section; otherwise in the `scratch_bytes` bytes at `scratch` (256-byte aligned).
static int decode_step_impl(zsm_cache_t* cache, int32_t layer_begin, int32_t layer_end, const void* q,
                            const void* k_new, const void* v_new, float* out, int32_t* write_slot,
                            int32_t* evicted_pos, int32_t* merged_slot, void* stream, char* scratch,
                            size_t scratch_bytes) {
    if (!cache || !q || !k_new || !v_new || !out) return ZSM_E_NULL;
    if (layer_begin < 0 || layer_end > cache->cfg.n_layers || layer_begin >= layer_end) return ZSM_E_RANGE;
    if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(out)) return ZSM_E_ALIGN;
    const CacheView& v = cache->cv;
    const int n_units = (layer_end - layer_begin) * v.S * v.H;
    int part_rows = 0;
    const int parts = choose_parts(cache, n_units, &part_rows);
    if (parts < 0) return parts;
    DecodeArgs a;
    a.cv = v;
    if (scratch && parts > 1) {
        const SplitScratch sp = split_scratch((size_t)n_units * parts, n_units, decode_compiled_heads(v.G), v.D, v.cap);
        if (sp.total > scratch_bytes) return ZSM_E_NOMEM;
        a.cv.sp_L = reinterpret_cast<double*>(scratch + sp.L);
        a.cv.sp_acc = reinterpret_cast<float*>(scratch + sp.acc);
        a.cv.sp_E = reinterpret_cast<double*>(scratch + sp.E);
    }
    a.unit0 = layer_begin * v.S * v.H;
    a.n_units = n_units;
    a.parts = parts;
    a.part_rows = part_rows;
    a.q = q; a.k_new = k_new; a.v_new = v_new; a.out = out;
    a.write_slot = write_slot; a.evicted_pos = evicted_pos; a.merged_slot = merged_slot;
    a.pool = nullptr; a.q_heads = v.G; a.n_shares = 1;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (v.G > 8) {
        // Groups of more than eight query heads: one workgroup per unit and share of eight (or four) heads, the
        // shares' per-slot sums in the scratch section of the cache buffer, in launches of as many units as that
        // holds.
        const size_t es = esize(v.dtype);
        const int gs = pool_share_heads(v);   // > 0: choose_parts has checked
        a.n_shares = (v.G + gs - 1) / gs;
        const int per_launch = v.sp_max_units;   // the scratch holds n_shares slices for each of that many units
        for (int u0 = 0; u0 < n_units; u0 += per_launch) {
            DecodeArgs b = a;
            b.unit0 = a.unit0 + u0;
            b.n_units = n_units - u0 < per_launch ? n_units - u0 : per_launch;
            b.pool = v.sp_E;
            b.q = static_cast<const char*>(q) + (size_t)u0 * v.G * v.D * es;
            b.k_new = static_cast<const char*>(k_new) + (size_t)u0 * v.D * es;
            b.v_new = static_cast<const char*>(v_new) + (size_t)u0 * v.D * es;
            b.out = out + (size_t)u0 * v.G * v.D;
            b.write_slot = write_slot ? write_slot + u0 : nullptr;
            b.evicted_pos = evicted_pos ? evicted_pos + u0 : nullptr;
            b.merged_slot = merged_slot ? merged_slot + u0 : nullptr;
            switch (v.dtype) {
                case ZSM_F32: e = launch_decode_pooled_f32(b, st); break;
                case ZSM_F16: e = launch_decode_pooled_f16(b, st); break;
                default: e = launch_decode_pooled_bf16(b, st); break;
            }
            if (e != hipSuccess) return hip_fail(e, "zsm_decode_step launch (pooled heads)");
        }
        return ZSM_OK;
    }
    switch (v.dtype) {
        case ZSM_F32: e = launch_decode_f32(a, st); break;
        case ZSM_F16: e = launch_decode_f16(a, st); break;
        default: e = launch_decode_bf16(a, st); break;
    }
    if (e != hipSuccess) return hip_fail(e, "zsm_decode_step launch");
    return ZSM_OK;
}

int zsm_decode_step(zsm_cache_t* cache, int32_t layer_begin, int32_t layer_end, const void* q,
                    const void* k_new, const void* v_new, float* out, int32_t* write_slot,
                    int32_t* evicted_pos, int32_t* merged_slot, void* stream) {
    return decode_step_impl(cache, layer_begin, layer_end, q, k_new, v_new, out, write_slot, evicted_pos, merged_slot,
                            stream, nullptr, 0);
}

// ---- the decode step for callers that cannot allocate: scratch held by the library -----------
// One array per GPU, alive until the process ends.  In host code the array's name is only a handle
// for hipGetSymbolAddress; the device address it resolves to (per device) is what kernels get.
static __device__ __align__(256) unsigned char scratch[ZSM_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
char* g_scratch_ptr[MAX_DEVICES] = {};

// device address of `scratch` on the current device (resolved once per device)
int static_scratch_ptr(char** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "zsm_decode_step_static hipGetDevice");
    if (dev < 0 || dev >= MAX_DEVICES) return ZSM_E_RANGE;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(e, "zsm_decode_step_static hipGetSymbolAddress");
        g_scratch_ptr[dev] = static_cast<char*>(p);
    }
    *out = g_scratch_ptr[dev];
    return ZSM_OK;
}
}  // namespace

int zsm_decode_step_static(zsm_cache_t* cache, int32_t layer_begin, int32_t layer_end, const void* q,
                           const void* k_new, const void* v_new, float* out, int32_t* write_slot,
                           int32_t* evicted_pos, int32_t* merged_slot, void* stream) {
    char* ptr = nullptr;
    int rc = static_scratch_ptr(&ptr);
    if (rc) return rc;
    rc = decode_step_impl(cache, layer_begin, layer_end, q, k_new, v_new, out, write_slot, evicted_pos, merged_slot,
                          stream, ptr, ZSM_STATIC_SCRATCH_BYTES);
    return rc == ZSM_E_NOMEM ? ZSM_E_SCRATCH : rc;
}

int zsm_cache_set_decode_parts(zsm_cache_t* cache, int32_t parts) {
    if (!cache) return ZSM_E_NULL;
    if (parts < 0 || parts > SP_MAX_PARTS) return ZSM_E_RANGE;
    cache->parts = parts;
    return ZSM_OK;
}

int zsm_decode_parts(const zsm_cache_t* cache, int32_t layer_begin, int32_t layer_end) {
    if (!cache) return ZSM_E_NULL;
    if (layer_begin < 0 || layer_end > cache->cfg.n_layers || layer_begin >= layer_end) return ZSM_E_RANGE;
    int part_rows = 0;
    return choose_parts(cache, (layer_end - layer_begin) * cache->cv.S * cache->cv.H, &part_rows);
}

size_t zsm_prefill_workspace_bytes(const zsm_cache_t* cache, int32_t n_layers, int32_t T_max, int32_t W) {
    if (!cache || n_layers < 1 || n_layers > cache->cfg.n_layers || T_max < 1 || W < 1) return 0;
    return prefill_workspace_bytes(cache->cv, n_layers, T_max, W);
}

int zsm_prefill_compress(zsm_cache_t* cache, int32_t layer_begin, int32_t layer_end, const void* Q, int32_t W,
                         const void* K, const void* V, const int32_t* seq_lens, int32_t T_max, void* workspace,
                         size_t ws_bytes, void* stream) {
    if (!cache || !Q || !K || !V || !seq_lens || !workspace) return ZSM_E_NULL;
    if (layer_begin < 0 || layer_end > cache->cfg.n_layers || layer_begin >= layer_end) return ZSM_E_RANGE;
    if (T_max < 1 || W < 1) return ZSM_E_SHAPE;
    if (cache->cfg.n_residual > 64) return ZSM_E_SHAPE;
    const CacheView& cv = cache->cv;
    const int n_layers = layer_end - layer_begin;
    const int gl = prefill_group_layers(cv, n_layers);
    if (gl < 1) return ZSM_E_SHAPE;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V)) return ZSM_E_ALIGN;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return ZSM_E_ALIGN;
    if (ws_bytes < prefill_workspace_bytes(cv, n_layers, T_max, W)) return ZSM_E_NOMEM;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int lu = cv.S * cv.H;
    if (g_debug_checks.load(std::memory_order_relaxed)) {
        int rc = run_state_check(cache, st, [&] {
            hipLaunchKernelGGL(check_empty_kernel, dim3(n_layers * lu), dim3(256), 0, st, cv, layer_begin * lu, cache->dbg);
        }, "zsm_prefill_compress state check");
        if (rc) return rc;
    }
    const size_t es = esize(cv.dtype);
    for (int l0 = 0; l0 < n_layers; l0 += gl) {   // groups of whole layers, each one set of launches
        const int nl = n_layers - l0 < gl ? n_layers - l0 : gl;
        PrefillArgs a;
        a.cv = cv;
        a.unit0 = (layer_begin + l0) * lu;
        a.n_units = nl * lu;
        a.Q = static_cast<const char*>(Q) + (size_t)l0 * lu * cv.G * W * cv.D * es;
        a.K = static_cast<const char*>(K) + (size_t)l0 * lu * T_max * cv.D * es;
        a.V = static_cast<const char*>(V) + (size_t)l0 * lu * T_max * cv.D * es;
        a.seq_lens = seq_lens; a.W = W; a.T_max = T_max;
        a.ws = static_cast<char*>(workspace);
        hipError_t e = launch_prefill(a, st);
        if (e != hipSuccess) return hip_fail(e, "zsm_prefill_compress launch");
    }
    return ZSM_OK;
}

static int xfer(const zsm_cache_t* c, int layer, void* K, void* V, float* Kr, float* Vr, float* s,
                int32_t* pos, int32_t* w, int64_t* n_seen, hipStream_t st, bool to_cache) {
    const CacheView& v = c->cv;
    const size_t lu = (size_t)v.S * v.H, u0 = (size_t)layer * lu;
    const size_t es = esize(v.dtype);
    struct Seg { void* user; char* mine; size_t bytes; };
    const Seg segs[] = {
        {K, static_cast<char*>(v.Kt) + u0 * v.cap_tok * v.D * es, lu * v.cap_tok * v.D * es},
        {V, static_cast<char*>(v.Vt) + u0 * v.cap_tok * v.D * es, lu * v.cap_tok * v.D * es},
        {Kr, reinterpret_cast<char*>(v.Kr + u0 * v.Br * v.D), lu * v.Br * v.D * sizeof(float)},
        {Vr, reinterpret_cast<char*>(v.Vr + u0 * v.Br * v.D), lu * v.Br * v.D * sizeof(float)},
        {s, reinterpret_cast<char*>(v.s + u0 * v.cap), lu * v.cap * sizeof(float)},
        {pos, reinterpret_cast<char*>(v.pos + u0 * v.cap), lu * v.cap * sizeof(int32_t)},
        {w, reinterpret_cast<char*>(v.w + u0 * v.cap), lu * v.cap * sizeof(int32_t)},
        {n_seen, reinterpret_cast<char*>(v.n_seen + u0), lu * sizeof(int64_t)},
    };
    for (const Seg& g : segs) {
        if (!g.user || g.bytes == 0) continue;
        if (!aligned16(g.user)) return ZSM_E_ALIGN;
    }
    for (const Seg& g : segs) {
        if (!g.user || g.bytes == 0) continue;
        const size_t n16 = g.bytes / 16, rem = g.bytes % 16;
        char* dst = to_cache ? g.mine : static_cast<char*>(g.user);
        const char* src = to_cache ? static_cast<const char*>(g.user) : g.mine;
        if (n16) {
            const int blocks = (int)((n16 + 255) / 256 > 4096 ? 4096 : (n16 + 255) / 256);
            hipLaunchKernelGGL(stream_copy_kernel, dim3(blocks), dim3(256), 0, st, reinterpret_cast<uint4*>(dst),
                               reinterpret_cast<const uint4*>(src), n16);
        }
        if (rem) {
            hipError_t e = hipMemcpyAsync(dst + n16 * 16, src + n16 * 16, rem, hipMemcpyDeviceToDevice, st);
            if (e != hipSuccess) return hip_fail(e, "zsm_cache transfer tail");
        }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "zsm_cache transfer");
    return ZSM_OK;
}

int zsm_cache_export(const zsm_cache_t* cache, int32_t layer, void* K, void* V, float* Kr, float* Vr,
                     float* s, int32_t* pos, int32_t* w, int64_t* n_seen, void* stream) {
    int rc = check_layer(cache, layer);
    if (rc) return rc;
    return xfer(cache, layer, K, V, Kr, Vr, s, pos, w, n_seen, static_cast<hipStream_t>(stream), false);
}

int zsm_cache_import(zsm_cache_t* cache, int32_t layer, const void* K, const void* V, const float* Kr,
                     const float* Vr, const float* s, const int32_t* pos, const int32_t* w,
                     const int64_t* n_seen, void* stream) {
    int rc = check_layer(cache, layer);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (g_debug_checks.load(std::memory_order_relaxed)) {
        if ((pos && !aligned16(pos)) || (w && !aligned16(w)) || (n_seen && !aligned16(n_seen))) return ZSM_E_ALIGN;
        const int lu0 = cache->cv.S * cache->cv.H;
        rc = run_state_check(cache, st, [&] {
            hipLaunchKernelGGL(check_import_kernel, dim3(lu0), dim3(256), 0, st, cache->cv, layer * lu0, pos, w, n_seen, cache->dbg);
        }, "zsm_cache_import state check");
        if (rc) return rc;
    }
    rc = xfer(cache, layer, const_cast<void*>(K), const_cast<void*>(V), const_cast<float*>(Kr),
              const_cast<float*>(Vr), const_cast<float*>(s), const_cast<int32_t*>(pos),
              const_cast<int32_t*>(w), const_cast<int64_t*>(n_seen), st, true);
    if (rc) return rc;
    const int lu = cache->cv.S * cache->cv.H;
    hipLaunchKernelGGL(recount_kernel, dim3(lu), dim3(256), 0, st, cache->cv, layer * lu);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "zsm_cache_import recount");
    return ZSM_OK;
}

__global__ void flags_out_kernel(int32_t* flags, int32_t* out, int n, int clear) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    if (out) out[i] = flags[i];
    if (clear) flags[i] = 0;
}

int zsm_cache_flags(zsm_cache_t* cache, int32_t layer, int32_t* flags, int32_t clear, void* stream) {
    int rc = check_layer(cache, layer);
    if (rc) return rc;
    if (!flags && !clear) return ZSM_E_NULL;
    const int lu = cache->cv.S * cache->cv.H;
    hipLaunchKernelGGL(flags_out_kernel, dim3((lu + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                       cache->cv.flags + (size_t)layer * lu, flags, lu, clear ? 1 : 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "zsm_cache_flags");
    return ZSM_OK;
}

int zsm_set_debug_checks(int32_t on) {
    return g_debug_checks.exchange(on ? 1 : 0);
}

int zsm_stream_read(const void* src, size_t bytes, float* sink, void* stream) {
    if (!src || !sink) return ZSM_E_NULL;
    if (!aligned16(src)) return ZSM_E_ALIGN;
    if (bytes % 16) return ZSM_E_SHAPE;
    if (bytes == 0) return ZSM_OK;
    // 8 workgroups per compute unit: the fastest of the grid sizes tried (1024 to 8192) for a 1.5 GB buffer
    hipLaunchKernelGGL(stream_read_kernel, dim3(256 * 8), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(src), bytes / 16, sink);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "zsm_stream_read");
    return ZSM_OK;
}

int zsm_stream_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!src || !dst) return ZSM_E_NULL;
    if (!aligned16(src) || !aligned16(dst)) return ZSM_E_ALIGN;
    if (bytes % 16) return ZSM_E_SHAPE;
    if (bytes == 0) return ZSM_OK;
    hipLaunchKernelGGL(stream_copy_kernel, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint4*>(dst), static_cast<const uint4*>(src), bytes / 16);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "zsm_stream_copy");
    return ZSM_OK;
}

const char* zsm_strerror(int status) {
    switch (status) {
        case ZSM_OK: return "ok";
        case ZSM_E_NULL: return "a required pointer is NULL";
        case ZSM_E_SHAPE: return "unsupported or inconsistent sizes";
        case ZSM_E_DTYPE: return "unknown kv_dtype";
        case ZSM_E_ALIGN: return "device pointer not sufficiently aligned";
        case ZSM_E_NOMEM: return "buffer or workspace too small";
        case ZSM_E_RANGE: return "layer index or range outside the cache";
        case ZSM_E_STATE: return "the cache state breaks the call's precondition (found by the optional state checks)";
        case ZSM_E_SCRATCH: return "the launch needs more than ZSM_STATIC_SCRATCH_BYTES of library-held scratch";
        case ZSM_E_HIP: return g_hip_msg;
        default: return "unknown status";
    }
}

}  // extern "C"
