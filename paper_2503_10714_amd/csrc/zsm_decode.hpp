// Fused decode step of the ZSMerge cache (Alg. 1 loop body with the attention of Eq. 4).
//
// One workgroup per unit, two streaming passes inside it, K and V each read exactly once:
//   pass 1 streams K: every wave takes tiles of rows with 16-byte loads (a row of d*e
//     bytes is spread over LPR consecutive lanes, a wave-wide load covers RPL = 64/LPR
//     whole rows), forms the logits and stores exp(logit - C) per slot in LDS, C being the
//     incoming token's own logit (any reference works in fp64: see below);
//   one barrier gives every wave the softmax denominator L;
//   pass 2 streams V and accumulates p * v with p = exp(.)/L read back from LDS.
// After that: score update (Eq. 3), eviction choice, residual merge (Eq. 5, Eq. 6) and the
// write of the incoming token, all from the per-slot values kept in LDS plus 12 bytes of
// metadata per slot.
//
// Precision.  Everything that feeds a stored score or a decision (logits, exp, L, Eq. 5's
// dot products, Eq. 6's mean) is evaluated in fp64 and rounded once to the fp32 storage
// type; products of two fp16/bf16/fp32 values are exact in fp64, so the logits are the
// exactly rounded dot products and the eviction choice does not depend on the summation
// order of this kernel.  The attention output uses fp32 probabilities and accumulators.
// With fp64 exponentials no running maximum is needed: exp(z - C) cannot overflow unless a
// logit exceeds the incoming token's by more than 690, at which the difference is clamped.
#pragma once

#include "zsm_common.hpp"

namespace zsm {

struct DecodeArgs {
    CacheView cv;
    int32_t unit0;      // first global unit of the launch (layer_begin * S * H)
    int32_t n_units;
    const void* q;
    const void* k_new;
    const void* v_new;
    float* out;
    int32_t* write_slot;
    int32_t* evicted_pos;
    int32_t* merged_slot;
};

template <typename T, int D, int G, int NW>
struct DecodeShape {
    static constexpr int EPL = 16 / sizeof(T);   // elements per lane (one 16-byte load)
    static constexpr int LPR = D / EPL;          // lanes per row
    static constexpr int RPL = 64 / LPR;         // rows per wave-wide load
    static constexpr int UT = 4;                 // wave-wide loads per tile (two tiles are in flight)
    static constexpr int UH = 4;                 // loads per reduction granule
    static constexpr int R = UT * RPL;           // rows per wave tile
    static constexpr int PART = UH * RPL * (LPR + 1);   // doubles of partial-dot staging per wave
    static constexpr int NT = NW * 64;
    static constexpr bool QLDS = G > 2;          // queries live in LDS instead of registers
    static_assert(LPR >= 1 && LPR <= 64 && 64 % LPR == 0, "row must split over a wave");

    // dynamic LDS bytes for a slot capacity `cap` (same formula on host and device)
    __host__ __device__ static size_t lds_bytes(int cap) {
        size_t n = 0;
        n += sizeof(double) * G * (size_t)(cap + 1);   // et
        n += sizeof(double) * NW * PART;               // part
        n += sizeof(double) * NW * G;                  // red64
        n += sizeof(double) * (QLDS ? G * D : 0);      // qlds
        n += sizeof(unsigned long long) * NW;          // keyw
        n += sizeof(double) * NW;                      // dotw
        n += sizeof(float) * NW * G * D;               // accw
        n += sizeof(int) * (4 + NW);                   // misc
        return (n + 15) & ~(size_t)15;
    }
};

// The G query vectors, fp64: this lane's segment in registers, or all of them in LDS.
template <int G, int EPL, bool QLDS>
struct Query {
    double r[QLDS ? 1 : G][EPL];
    const double* lds;    // [G][D] when QLDS
    __device__ __forceinline__ void get(int g, int seg, int D, double* out) const {
        if (QLDS) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) out[e] = lds[g * D + seg * EPL + e];
        } else {
#pragma unroll
            for (int e = 0; e < EPL; ++e) out[e] = r[QLDS ? 0 : g][e];
        }
    }
};

// Branch-free load of UU wave-wide loads of rows [row0, row0 + UU*RPL) of a row array whose
// rows all exist and are occupied up to nrows: a row index past the end is clamped to the last
// row (its result is discarded by the compute step).
template <typename KT, int UU, int D, int EPL, int LPR, int RPL>
__device__ __forceinline__ void tile_load(Raw<KT, EPL>* dst, const KT* __restrict__ base, int row0, int nrows,
                                          int lane) {
    const int grp = lane / LPR, seg = lane % LPR;
    if (row0 + UU * RPL <= nrows) {
        const KT* p = base + ((size_t)(row0 + grp) * D + seg * EPL);
#pragma unroll
        for (int u = 0; u < UU; ++u) dst[u].load(p + (size_t)u * RPL * D);
    } else {
#pragma unroll
        for (int u = 0; u < UU; ++u) {
            const int r = row0 + u * RPL + grp;
            dst[u].load(base + (size_t)(r < nrows ? r : nrows - 1) * D + seg * EPL);
        }
    }
}

// Pass 1 on UU loaded wave-wide loads of K rows [row0, row0 + UU*RPL); rows >= nrows do not
// exist.  For every existing row the holder lane stores exp(logit - C) (0 for an empty row) at
// et[g][zidx0 + row] and adds it to lsum[g] (and, when mz is given, keeps the largest logit - C
// in mz[g]).  posb / wb (MASKED only) mark empty rows (pos < 0, w == 0); wb also adds
// alpha*log(w) to the logit (Eq. 4).
template <typename KT, int UU, bool MASKED, int D, int G, int EPL, int LPR, int RPL, bool QLDS>
__device__ __forceinline__ void k_compute(const Raw<KT, EPL>* kr, int row0, int nrows, int zidx0,
                                          const int32_t* __restrict__ posb, const int32_t* __restrict__ wb,
                                          double alpha, double scale, const Query<G, EPL, QLDS>& qq,
                                          const double* C, double* lsum, float* mz, double* et, int Bz,
                                          double* part_w, int lane) {
    constexpr int UH = UU < 4 ? UU : 4;
    const int grp = lane / LPR, seg = lane % LPR;
#pragma unroll
    for (int h = 0; h < UU; h += UH) {
        // lane x < UH*RPL "holds" row row0 + h*RPL + x: it finishes that row's logit
        const int hr = row0 + h * RPL + lane;
        const bool hexist = lane < UH * RPL && hr < nrows;
        bool hvalid = hexist;
        double addend = 0.0;
        if (MASKED) {
            if (hvalid && posb) hvalid = posb[hr] >= 0;
            if (hvalid && wb) {
                const int wv = wb[hr];
                hvalid = wv > 0;
                if (wv > 1) addend = alpha * log((double)wv);
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            double qv[EPL];
            qq.get(g, seg, D, qv);
#pragma unroll
            for (int u = 0; u < UH; ++u) {
                double p = 0.0;
#pragma unroll
                for (int e = 0; e < EPL; ++e) p = fma(qv[e], (double)kr[h + u].get(e), p);
                part_w[(u * RPL + grp) * (LPR + 1) + seg] = p;
            }
            wave_sync();
            if (hexist) {
                double ev = 0.0;
                if (hvalid) {
                    double a = 0.0;
#pragma unroll
                    for (int i = 0; i < LPR; ++i) a += part_w[lane * (LPR + 1) + i];
                    const double z = a * scale + addend;
                    ev = exp(fmin(z - C[g], 690.0));
                    lsum[g] += ev;
                    if (mz) mz[g] = fmaxf(mz[g], (float)(z - C[g]));
                }
                et[(size_t)g * Bz + zidx0 + hr] = ev;
            }
            wave_sync();
        }
    }
}

// Pass 1 for rows that may be empty: load only the occupied ones (an empty slot may hold any
// bit pattern), then k_compute.
template <typename KT, int UU, int D, int G, int EPL, int LPR, int RPL, bool QLDS>
__device__ __forceinline__ void k_tile_masked(const KT* __restrict__ Kb, int row0, int nrows, int zidx0,
                                              const int32_t* __restrict__ posb, const int32_t* __restrict__ wb,
                                              double alpha, double scale, const Query<G, EPL, QLDS>& qq,
                                              const double* C, double* lsum, float* mz, double* et, int Bz,
                                              double* part_w, int lane) {
    const int grp = lane / LPR, seg = lane % LPR;
    Raw<KT, EPL> kr[UU];
#pragma unroll
    for (int u = 0; u < UU; ++u) {
        const int r = row0 + u * RPL + grp;
        if (r < nrows && (posb == nullptr || posb[r] >= 0) && (wb == nullptr || wb[r] > 0))
            kr[u].load(Kb + (size_t)r * D + seg * EPL);
        else
            kr[u].zero();
    }
    k_compute<KT, UU, true, D, G, EPL, LPR, RPL, QLDS>(kr, row0, nrows, zidx0, posb, wb, alpha, scale, qq, C, lsum, mz,
                                                       et, Bz, part_w, lane);
}

// Pass 2 on UU loaded wave-wide loads of V rows: acc[g] += p * v with p = et * rL (fp32).
template <typename KT, int UU, int D, int G, int EPL, int LPR, int RPL>
__device__ __forceinline__ void v_compute(const Raw<KT, EPL>* vr, int row0, int nrows, int zidx0,
                                          const double* rL, float (*acc)[EPL], const double* et, int Bz,
                                          int lane) {
    const int grp = lane / LPR;
#pragma unroll
    for (int u = 0; u < UU; ++u) {
        const int r = row0 + u * RPL + grp;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const double ev = r < nrows ? et[(size_t)g * Bz + zidx0 + r] : 0.0;
            const float p = (float)(ev * rL[g]);
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, vr[u].get(e), acc[g][e]);
        }
    }
}

// Pass 2 for rows that may be empty: rows whose probability is exactly 0 (empty slots among
// them) are not loaded.
template <typename KT, int UU, int D, int G, int EPL, int LPR, int RPL>
__device__ __forceinline__ void v_tile_masked(const KT* __restrict__ Vb, int row0, int nrows, int zidx0,
                                              const double* rL, float (*acc)[EPL], const double* et, int Bz,
                                              int lane) {
    const int grp = lane / LPR, seg = lane % LPR;
    Raw<KT, EPL> vr[UU];
#pragma unroll
    for (int u = 0; u < UU; ++u) {
        const int r = row0 + u * RPL + grp;
        bool any = false;
        if (r < nrows) {
#pragma unroll
            for (int g = 0; g < G; ++g) any = any || (et[(size_t)g * Bz + zidx0 + r] != 0.0);
        }
        if (any) vr[u].load(Vb + (size_t)r * D + seg * EPL);
        else vr[u].zero();
    }
    v_compute<KT, UU, D, G, EPL, LPR, RPL>(vr, row0, nrows, zidx0, rL, acc, et, Bz, lane);
}

// A wave that is behind gets the issue priority: the workgroups that share a compute unit
// then advance together instead of oldest-first, which keeps all of them streaming to the
// end of the sweep.  `done` of `total` work items are finished.
__device__ __forceinline__ void prio_from_progress(int done, int total) {
    const int q = (4 * done) / (total > 0 ? total : 1);
    if (q >= 3) __builtin_amdgcn_s_setprio(0);
    else if (q == 2) __builtin_amdgcn_s_setprio(1);
    else if (q == 1) __builtin_amdgcn_s_setprio(2);
    else __builtin_amdgcn_s_setprio(3);
}

// Everything of a unit's cache that the end of a step touches.
template <typename T>
struct UnitRefs {
    T* Kt; T* Vt;              // token slots
    float* Kr; float* Vr;      // residual slots
    float* s; int32_t* pos; int32_t* w;
    const T* knew; const T* vnew;
};

constexpr int DECODE_MCH = 8;   // slots per thread whose score and position are requested ahead

// D3-D6 of one unit, by the whole workgroup: score update (Eq. 3) from the per-slot
// exp(logit - C) values in `et` (stride Bz per query head; LDS or global) and 1/L in rL,
// eviction choice, residual absorption (Eq. 5, Eq. 6) and the write of the incoming token.
// pj / sj hold the positions and scores of slots k*NT + tid, k < DECODE_MCH, loaded by the caller.
template <typename T, int D, int G, int NW>
__device__ __forceinline__ void decode_finish(const DecodeArgs& a, const CacheView& cv, const UnitRefs<T>& u, int lu,
                                              int ug, int Bp, int Br, int B, long long Tseen, int nocc, bool full,
                                              const double* et, int Bz, const double* rL, int* pj, float* sj,
                                              unsigned long long* keyw, double* dotw, int* misc) {
    constexpr int NT = NW * 64, MCH = DECODE_MCH;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    T* Kt = u.Kt; T* Vt = u.Vt;
    float* Kr = u.Kr; float* Vr = u.Vr;
    float* s = u.s; int32_t* pos = u.pos; int32_t* w = u.w;
    const T* knew = u.knew; const T* vnew = u.vnew;
    // ---- D3: score update (Eq. 3) and D4: eviction choice ------------------------------
    const double lam = (double)cv.lambda;
    const long long cand_hi = Tseen - Bp;   // evictable: position <= T - B_p (outside the latest B_p)
    unsigned long long best = ~0ull;
    int best_slot = -1;
    for (int base = 0; base < B; base += NT * MCH) {
        if (base > 0) {
#pragma unroll
            for (int k = 0; k < MCH; ++k) {
                const int j = base + k * NT + tid;
                pj[k] = j < B ? pos[j] : -1;
                sj[k] = j < B ? s[j] : 0.f;
            }
        }
#pragma unroll
        for (int k = 0; k < MCH; ++k) {
            const int j = base + k * NT + tid;
            if (j >= B) continue;
            if (pj[k] >= 0) {   // occupied (a residual slot carries the position of its first token)
                double pm = 0.0;
#pragma unroll
                for (int g = 0; g < G; ++g) pm += et[(size_t)g * Bz + j] * rL[g];
                pm /= (double)G;
                const float sn = (float)(lam * (double)sj[k] + pm);
                s[j] = sn;
                if (full && j >= Br && (long long)pj[k] <= cand_hi) {
                    const unsigned long long key = ((unsigned long long)__float_as_uint(sn) << 32) | (uint32_t)pj[k];
                    if (key < best) { best = key; best_slot = j; }
                }
            } else if (!full && j >= Br) {
                const unsigned long long key = (unsigned long long)j;   // lowest free token slot
                if (key < best) { best = key; best_slot = j; }
            }
        }
    }
    {
        const unsigned long long wb = wave_min(best);
        if (lane == 0) keyw[wave] = wb;
    }
    __syncthreads();
    unsigned long long bmin = keyw[0];
#pragma unroll
    for (int x = 1; x < NW; ++x) bmin = keyw[x] < bmin ? keyw[x] : bmin;
    if (best == bmin && best_slot >= 0) misc[0] = best_slot;
    __syncthreads();
    const int c = misc[0];        // slot that receives the incoming token
    if (c < Br || c >= B) return;  // corrupt imported state (no candidate at all): touch nothing
    const int ct = c - Br;
    const int ev_pos = full ? (int)(uint32_t)(bmin & 0xffffffffull) : -1;
    const float ev_s = __uint_as_float((uint32_t)(bmin >> 32));

    // ---- D5: absorb the evicted token into the residual set (Eq. 5, Eq. 6) ------------
    int merged = -1;
    int r_empty = -1;
    if (full && Br > 0) {
        for (int r = 0; r < Br; ++r)
            if (w[r] == 0) { r_empty = r; break; }
    }
    __syncthreads();   // every thread has taken its view of w before anyone changes it
    if (full && Br > 0) {
        if (r_empty >= 0) {
            if (tid < D) {
                Kr[r_empty * D + tid] = to_float(Kt[(size_t)ct * D + tid]);
                Vr[r_empty * D + tid] = to_float(Vt[(size_t)ct * D + tid]);
            }
            if (tid == 0) { w[r_empty] = 1; pos[r_empty] = ev_pos; s[r_empty] = ev_s; }
            merged = r_empty;
        } else {
            double bd = -INFINITY;
            int br = 0x7fffffff;
            for (int r = wave; r < Br; r += NW) {
                double p = 0.0;
                for (int ch = lane; ch < D; ch += 64)
                    p = fma((double)Kr[r * D + ch], (double)to_float(Kt[(size_t)ct * D + ch]), p);
                p = wave_sum(p);
                if (p > bd) { bd = p; br = r; }
            }
            if (lane == 0) { dotw[wave] = bd; misc[4 + wave] = br; }
            __syncthreads();
            bd = -INFINITY; br = 0x7fffffff;
#pragma unroll
            for (int x = 0; x < NW; ++x) {
                const double dx = dotw[x];
                const int rx = misc[4 + x];
                if (rx != 0x7fffffff && (br == 0x7fffffff || dx > bd || (dx == bd && rx < br))) { bd = dx; br = rx; }
            }
            merged = br;
            const int wv = w[br];
            if (tid < D) {
                const double wd = (double)wv;
                const double ke = (double)to_float(Kt[(size_t)ct * D + tid]);
                const double ve = (double)to_float(Vt[(size_t)ct * D + tid]);
                Kr[br * D + tid] = (float)((wd * (double)Kr[br * D + tid] + ke) / (wd + 1.0));
                Vr[br * D + tid] = (float)((wd * (double)Vr[br * D + tid] + ve) / (wd + 1.0));
            }
            __syncthreads();
            if (tid == 0) w[br] = wv + 1;
        }
    }
    __syncthreads();   // the evicted row has been read by everyone who needs it

    // ---- D6: the incoming token takes the freed slot ----------------------------------
    if (tid < D) {
        Kt[(size_t)ct * D + tid] = knew[tid];
        Vt[(size_t)ct * D + tid] = vnew[tid];
    }
    if (tid == 0) {
        double pm = 0.0;
#pragma unroll
        for (int g = 0; g < G; ++g) pm += et[(size_t)g * Bz + B] * rL[g];
        pm /= (double)G;
        pos[c] = (int32_t)Tseen;
        w[c] = 1;
        s[c] = (float)pm;
        cv.n_seen[ug] = Tseen + 1;
        if (!full) cv.n_occ[ug] = nocc + 1;
        if (a.write_slot) a.write_slot[lu] = c;
        if (a.evicted_pos) a.evicted_pos[lu] = ev_pos;
        if (a.merged_slot) a.merged_slot[lu] = merged;
    }
}

// Occupancy target: 4 waves per SIMD for G = 1 (four workgroups per compute unit, LDS permitting);
// the per-head state of grouped queries needs more registers and its LDS footprint caps the
// residency anyway.
template <typename T, int D, int G, int NW>
__global__ __launch_bounds__(NW * 64, (G == 1 ? 4 : 2)) void decode_kernel(DecodeArgs a) {
    using Sh = DecodeShape<T, D, G, NW>;
    constexpr int EPL = Sh::EPL, LPR = Sh::LPR, RPL = Sh::RPL, R = Sh::R, PART = Sh::PART, NT = Sh::NT, UT = Sh::UT;
    constexpr bool QLDS = Sh::QLDS;
    const CacheView& cv = a.cv;
    const int lu = blockIdx.x;
    const int ug = a.unit0 + lu;
    const int b = (ug / cv.H) % cv.S;
    const int Bp = cv.Bp[b], Bc = cv.Bc[b], Br = cv.Br;
    const int ntok = Bp + Bc, B = ntok + Br;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = lane / LPR, seg = lane % LPR;

    extern __shared__ __align__(16) unsigned char smem[];
    const int Bz = cv.cap + 1;
    double* et = reinterpret_cast<double*>(smem);                 // [G][Bz] exp(logit - C) per slot
    double* part = et + (size_t)G * Bz;                           // [NW][PART]
    double* red64 = part + NW * PART;                             // [NW][G]
    double* qlds = red64 + NW * G;                                // [G][D] (QLDS only)
    unsigned long long* keyw = reinterpret_cast<unsigned long long*>(qlds + (QLDS ? G * D : 0));   // [NW]
    double* dotw = reinterpret_cast<double*>(keyw + NW);          // [NW]
    float* accw = reinterpret_cast<float*>(dotw + NW);            // [NW][G][D]
    int* misc = reinterpret_cast<int*>(accw + NW * G * D);        // [4 + NW]

    T* Kt = reinterpret_cast<T*>(cv.Kt) + (size_t)ug * cv.cap_tok * D;
    T* Vt = reinterpret_cast<T*>(cv.Vt) + (size_t)ug * cv.cap_tok * D;
    float* Kr = cv.Kr + (size_t)ug * Br * D;
    float* Vr = cv.Vr + (size_t)ug * Br * D;
    float* s = cv.s + (size_t)ug * cv.cap;
    int32_t* pos = cv.pos + (size_t)ug * cv.cap;
    int32_t* w = cv.w + (size_t)ug * cv.cap;
    const T* qp = reinterpret_cast<const T*>(a.q) + (size_t)lu * G * D;
    const T* knew = reinterpret_cast<const T*>(a.k_new) + (size_t)lu * D;
    const T* vnew = reinterpret_cast<const T*>(a.v_new) + (size_t)lu * D;
    const long long Tseen = cv.n_seen[ug];
    const int nocc = cv.n_occ[ug];
    const bool full = nocc == ntok;
    const double scale = cv.scale;
    const double alpha = (double)cv.alpha;

    if (tid == 0) misc[0] = -1;
    Query<G, EPL, QLDS> qq;
    qq.lds = qlds;
    if (QLDS) {
        for (int i = tid; i < G * D; i += NT) qlds[i] = (double)to_float(qp[i]);
        __syncthreads();
    } else {
#pragma unroll
        for (int g = 0; g < (QLDS ? 1 : G); ++g) {
            float qf[EPL];
            load_seg<EPL>(qp + g * D + seg * EPL, qf);
#pragma unroll
            for (int e = 0; e < EPL; ++e) qq.r[g][e] = (double)qf[e];
        }
    }
    // reference logit C[g]: the incoming token against itself (every lane of every wave)
    double C[G], lsum[G];
    {
        float kf[EPL];
        load_seg<EPL>(knew + seg * EPL, kf);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            double qv[EPL];
            qq.get(g, seg, D, qv);
            double p = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) p = fma(qv[e], (double)kf[e], p);
#pragma unroll
            for (int o = 1; o < LPR; o <<= 1) p += __shfl_xor(p, o, 64);
            C[g] = p * scale;
            lsum[g] = 0.0;
        }
    }
    double* part_w = part + wave * PART;

    // ---- pass 1 (D1): logits of all slots, exp(logit - C) into LDS ---------------------
    // Fast path (every token slot occupied): tiles are double-buffered in registers, the loads
    // of the wave's next tile (or of its first V tile) are in flight while it works on this one.
    const int ntiles = (ntok + R - 1) / R;
    Raw<T, EPL> bufA[UT], bufB[UT];
    if (full) {
        int t = wave;
        if (t < ntiles) tile_load<T, UT, D, EPL, LPR, RPL>(bufA, Kt, t * R, ntok, lane);
        while (t < ntiles) {
            const int tn = t + NW;
            prio_from_progress(t, 2 * ntiles);
            if (tn < ntiles) tile_load<T, UT, D, EPL, LPR, RPL>(bufB, Kt, tn * R, ntok, lane);
            else tile_load<T, UT, D, EPL, LPR, RPL>(bufB, Vt, wave * R, ntok, lane);   // wave < ntiles here
            k_compute<T, UT, false, D, G, EPL, LPR, RPL, QLDS>(bufA, t * R, ntok, Br, nullptr, nullptr, alpha, scale, qq,
                                                               C, lsum, nullptr, et, Bz, part_w, lane);
#pragma unroll
            for (int u = 0; u < UT; ++u) bufA[u] = bufB[u];
            t = tn;
        }
    } else {
        for (int t = wave; t * RPL < ntok; t += NW)
            k_tile_masked<T, 1, D, G, EPL, LPR, RPL, QLDS>(Kt, t * RPL, ntok, Br, pos + Br, nullptr, alpha, scale, qq, C,
                                                           lsum, nullptr, et, Bz, part_w, lane);
    }
    // residual slots (fp32 rows, log-count term) and the incoming token itself
    for (int t = wave; t * RPL < Br; t += NW)
        k_tile_masked<float, 1, D, G, EPL, LPR, RPL, QLDS>(Kr, t * RPL, Br, 0, nullptr, w, alpha, scale, qq, C, lsum,
                                                           nullptr, et, Bz, part_w, lane);
    if (wave == NW - 1)
        k_tile_masked<T, 1, D, G, EPL, LPR, RPL, QLDS>(knew, 0, 1, B, nullptr, nullptr, alpha, scale, qq, C, lsum, nullptr,
                                                       et, Bz, part_w, lane);
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const double t = wave_sum(lsum[g]);
        if (lane == 0) red64[wave * G + g] = t;
    }
    __syncthreads();
    double rL[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        double t = 0.0;
#pragma unroll
        for (int x = 0; x < NW; ++x) t += red64[x * G + g];
        rL[g] = 1.0 / t;
    }

    // ---- pass 2 (D2): out = sum p * v --------------------------------------------------
    float acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    if (full) {
        int t = wave;   // bufA already holds this wave's first V tile
        while (t < ntiles) {
            const int tn = t + NW;
            prio_from_progress(ntiles + t, 2 * ntiles);
            if (tn < ntiles) tile_load<T, UT, D, EPL, LPR, RPL>(bufB, Vt, tn * R, ntok, lane);
            v_compute<T, UT, D, G, EPL, LPR, RPL>(bufA, t * R, ntok, Br, rL, acc, et, Bz, lane);
#pragma unroll
            for (int u = 0; u < UT; ++u) bufA[u] = bufB[u];
            t = tn;
        }
    } else {
        for (int t = wave; t * RPL < ntok; t += NW)
            v_tile_masked<T, 1, D, G, EPL, LPR, RPL>(Vt, t * RPL, ntok, Br, rL, acc, et, Bz, lane);
    }
    __builtin_amdgcn_s_setprio(0);
    for (int t = wave; t * RPL < Br; t += NW)
        v_tile_masked<float, 1, D, G, EPL, LPR, RPL>(Vr, t * RPL, Br, 0, rL, acc, et, Bz, lane);
    if (wave == NW - 1)
        v_tile_masked<T, 1, D, G, EPL, LPR, RPL>(vnew, 0, 1, B, rL, acc, et, Bz, lane);

    // Scores and positions of this thread's first batch of slots: requested now, used after the
    // output has been combined, so that their latency is hidden.
    constexpr int MCH = DECODE_MCH;
    int pj[MCH];
    float sj[MCH];
#pragma unroll
    for (int k = 0; k < MCH; ++k) {
        const int j = k * NT + tid;
        pj[k] = j < B ? pos[j] : -1;
        sj[k] = j < B ? s[j] : 0.f;
    }
    // ---- combine the waves' partial outputs -> out -------------------------------------
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            float v = acc[g][e];
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) v += __shfl_xor(v, o, 64);
            if (grp == 0) accw[(wave * G + g) * D + seg * EPL + e] = v;
        }
    }
    __syncthreads();
    for (int idx = tid; idx < G * D; idx += NT) {
        float o = 0.f;
#pragma unroll
        for (int x = 0; x < NW; ++x) o += accw[x * G * D + idx];
        a.out[(size_t)lu * G * D + idx] = o;
    }

    UnitRefs<T> u{Kt, Vt, Kr, Vr, s, pos, w, knew, vnew};
    decode_finish<T, D, G, NW>(a, cv, u, lu, ug, Bp, Br, B, Tseen, nocc, full, et, Bz, rL, pj, sj, keyw, dotw, misc);
}

// Host side: pick the instantiation for (D, G) and launch one workgroup per unit.
constexpr int DECODE_NW = 4;

template <typename T, int D, int G>
inline hipError_t launch_decode_dg(const DecodeArgs& a, hipStream_t stream) {
    using Sh = DecodeShape<T, D, G, DECODE_NW>;
    const size_t lds = Sh::lds_bytes(a.cv.cap);
    auto kern = decode_kernel<T, D, G, DECODE_NW>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(a.n_units), dim3(DECODE_NW * 64), lds, stream, a);
    return hipGetLastError();
}

template <typename T, int D, int G>
inline size_t decode_lds_dg(int cap) { return DecodeShape<T, D, G, DECODE_NW>::lds_bytes(cap); }

template <typename T>
inline hipError_t launch_decode_t(const DecodeArgs& a, hipStream_t stream) {
    const int D = a.cv.D, G = a.cv.G;
#define ZSM_CASE(DD, GG) if (D == DD && G == GG) return launch_decode_dg<T, DD, GG>(a, stream);
    ZSM_CASE(64, 1) ZSM_CASE(64, 2) ZSM_CASE(64, 4) ZSM_CASE(64, 8)
    ZSM_CASE(128, 1) ZSM_CASE(128, 2) ZSM_CASE(128, 4) ZSM_CASE(128, 8)
#undef ZSM_CASE
    return hipErrorInvalidValue;
}

template <typename T>
inline size_t decode_lds_t(int D, int G, int cap) {
#define ZSM_CASE(DD, GG) if (D == DD && G == GG) return decode_lds_dg<T, DD, GG>(cap);
    ZSM_CASE(64, 1) ZSM_CASE(64, 2) ZSM_CASE(64, 4) ZSM_CASE(64, 8)
    ZSM_CASE(128, 1) ZSM_CASE(128, 2) ZSM_CASE(128, 4) ZSM_CASE(128, 8)
#undef ZSM_CASE
    return (size_t)-1;
}

// one translation unit per dtype provides these
hipError_t launch_decode_f32(const DecodeArgs& a, hipStream_t stream);
hipError_t launch_decode_f16(const DecodeArgs& a, hipStream_t stream);
hipError_t launch_decode_bf16(const DecodeArgs& a, hipStream_t stream);
size_t decode_lds_f32(int D, int G, int cap);
size_t decode_lds_f16(int D, int G, int cap);
size_t decode_lds_bf16(int D, int G, int cap);

}  // namespace zsm
