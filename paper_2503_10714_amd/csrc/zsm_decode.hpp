// Fused decode step of the ZSMerge cache (Alg. 1 loop body with the attention of Eq. 4).
//
// One workgroup per unit.  Each wave streams its own tiles of K and V rows with 16-byte
// loads (a row of d*e bytes is spread over LPR consecutive lanes, so a wave-wide load
// covers RPL = 64/LPR whole rows) and keeps a private online softmax, so there is no
// block-wide barrier inside the sweep and K and V are read exactly once.
//
// Two precisions run side by side:
//   * the attention output uses fp32 probabilities and fp32 accumulators;
//   * everything that feeds a stored score or a decision (logits, the softmax that updates
//     s, Eq. 5's dot products, Eq. 6's mean) is evaluated in fp64 and rounded once to the
//     fp32 storage type.  Products of two fp16/bf16/fp32 values are exact in fp64, so the
//     logits are the exactly rounded dot products and the eviction choice does not depend
//     on the summation order of this kernel.
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

template <typename T, int D, int G, int NW, int U>
struct DecodeShape {
    static constexpr int EPL = 16 / sizeof(T);   // elements per lane (one 16-byte load)
    static constexpr int LPR = D / EPL;          // lanes per row
    static constexpr int RPL = 64 / LPR;         // rows per wave-wide load
    static constexpr int R = U * RPL;            // rows per wave tile
    static constexpr int PART = R * (LPR + 1);   // doubles of partial-dot staging per wave
    static constexpr int NT = NW * 64;
    static_assert(LPR >= 1 && LPR <= 64 && 64 % LPR == 0, "row must split over a wave");

    // dynamic LDS bytes for a slot capacity `cap` (same formula on host and device)
    __host__ __device__ static size_t lds_bytes(int cap) {
        size_t n = 0;
        n += sizeof(double) * G * (size_t)(cap + 1);   // zt
        n += sizeof(double) * NW * PART;               // part
        n += sizeof(double) * NW * G;                  // red64
        n += sizeof(double) * G;                       // l64
        n += sizeof(unsigned long long) * NW;          // keyw
        n += sizeof(double) * NW;                      // dotw
        n += sizeof(float) * NW * G * D;               // accw
        n += sizeof(float) * NW * R;                   // pbuf
        n += sizeof(float) * NW * G * 2;               // mw, lw
        n += sizeof(float) * G;                        // Mg
        n += sizeof(int) * (4 + NW);                   // misc
        return (n + 15) & ~(size_t)15;
    }
};

// State a wave carries through its sweep.
template <int G, int EPL>
struct WaveState {
    double qd[G][EPL];   // this lane's segment of every query head, fp64
    float m[G];          // running maximum (wave-uniform)
    float l[G];          // running sum of exp(z - m) for the rows this lane holds
    float acc[G][EPL];   // running sum of p * v for this lane's channel segment
};

// Process UU wave-wide loads of rows [row0, row0 + UU*RPL) of the row arrays Kb / Vb
// (element type KT, row length D).  Rows >= nrows do not exist.
// MASKED = false: every existing row is occupied; the loads are branch-free (a row index
// past the end is clamped to the last row and its result discarded).
// MASKED = true: posb / wb, when given, mark empty rows (pos < 0, w == 0), which take no
// part and are never loaded (an empty slot may hold any bit pattern); wb also adds
// alpha*log(w) to the logit (Eq. 4).
template <typename KT, int UU, bool MASKED, int D, int G, int EPL, int LPR, int RPL>
__device__ __forceinline__ void decode_tile(const KT* __restrict__ Kb, const KT* __restrict__ Vb,
                                            int row0, int nrows, int zidx0,
                                            const int32_t* __restrict__ posb,
                                            const int32_t* __restrict__ wb, double alpha,
                                            double scale, WaveState<G, EPL>& st, double* zt,
                                            int Bz, double* part_w, float* pbuf_w, int lane) {
    constexpr int RR = UU * RPL;
    const int grp = lane / LPR, seg = lane % LPR;
    Raw<KT, EPL> kr[UU], vr[UU];
#pragma unroll
    for (int u = 0; u < UU; ++u) {
        const int r = row0 + u * RPL + grp;
        if (MASKED) {
            if (r < nrows && (posb == nullptr || posb[r] >= 0) && (wb == nullptr || wb[r] > 0)) {
                kr[u].load(Kb + (size_t)r * D + seg * EPL);
                vr[u].load(Vb + (size_t)r * D + seg * EPL);
            } else {
                kr[u].zero();
                vr[u].zero();
            }
        } else {
            const int rc = r < nrows ? r : nrows - 1;
            kr[u].load(Kb + (size_t)rc * D + seg * EPL);
            vr[u].load(Vb + (size_t)rc * D + seg * EPL);
        }
    }
    // lane h < RR "holds" row row0 + h: it finishes that row's logit and probability
    const int hr = row0 + lane;
    const bool hexist = lane < RR && hr < nrows;
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
#pragma unroll
        for (int u = 0; u < UU; ++u) {
            double p = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) p = fma(st.qd[g][e], (double)kr[u].get(e), p);
            part_w[(u * RPL + grp) * (LPR + 1) + seg] = p;
        }
        wave_sync();
        double z = -INFINITY;
        if (hvalid) {
            double a = 0.0;
#pragma unroll
            for (int i = 0; i < LPR; ++i) a += part_w[lane * (LPR + 1) + i];
            z = a * scale + addend;
        }
        if (hexist) zt[(size_t)g * Bz + zidx0 + hr] = z;
        const float zf = (float)z;
        const float tmax = wave_max(zf);
        if (tmax > -INFINITY) {   // wave-uniform
            const float m_new = fmaxf(st.m[g], tmax);
            const float corr = __expf(st.m[g] - m_new);
            const float p = hvalid ? __expf(zf - m_new) : 0.f;
            st.l[g] = st.l[g] * corr + p;
            st.m[g] = m_new;
            if (lane < RR) pbuf_w[(lane % RPL) * UU + lane / RPL] = p;
            wave_sync();
#pragma unroll
            for (int e = 0; e < EPL; ++e) st.acc[g][e] *= corr;
#pragma unroll
            for (int u = 0; u < UU; ++u) {
                const float pu = pbuf_w[grp * UU + u];
#pragma unroll
                for (int e = 0; e < EPL; ++e) st.acc[g][e] = fmaf(pu, vr[u].get(e), st.acc[g][e]);
            }
        }
        wave_sync();
    }
}

template <typename T, int D, int G, int NW, int U>
__global__ __launch_bounds__(NW * 64, (G == 1 ? 4 : (G == 2 ? 2 : 1))) void decode_kernel(DecodeArgs a) {
    using Sh = DecodeShape<T, D, G, NW, U>;
    constexpr int EPL = Sh::EPL, LPR = Sh::LPR, RPL = Sh::RPL, R = Sh::R, PART = Sh::PART, NT = Sh::NT;
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
    double* zt = reinterpret_cast<double*>(smem);                 // [G][Bz] logits, later exp(z - M)
    double* part = zt + (size_t)G * Bz;                           // [NW][PART]
    double* red64 = part + NW * PART;                             // [NW][G]
    double* l64 = red64 + NW * G;                                 // [G]
    unsigned long long* keyw = reinterpret_cast<unsigned long long*>(l64 + G);   // [NW]
    double* dotw = reinterpret_cast<double*>(keyw + NW);          // [NW]
    float* accw = reinterpret_cast<float*>(dotw + NW);            // [NW][G][D]
    float* pbuf = accw + NW * G * D;                              // [NW][R]
    float* mw = pbuf + NW * R;                                    // [NW][G]
    float* lw = mw + NW * G;                                      // [NW][G]
    float* Mg = lw + NW * G;                                      // [G]
    int* misc = reinterpret_cast<int*>(Mg + G);                   // [4 + NW]

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

    WaveState<G, EPL> st;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float qf[EPL];
        load_seg<EPL>(qp + g * D + seg * EPL, qf);
#pragma unroll
        for (int e = 0; e < EPL; ++e) { st.qd[g][e] = (double)qf[e]; st.acc[g][e] = 0.f; }
        st.m[g] = -INFINITY;
        st.l[g] = 0.f;
    }
    if (tid == 0) misc[0] = -1;
    double* part_w = part + wave * PART;
    float* pbuf_w = pbuf + wave * R;

    // ---- D1 + D2: one sweep over the token slots -------------------------------------
    const int ntiles = (ntok + R - 1) / R;
    if (full) {
        for (int t = wave; t < ntiles; t += NW)
            decode_tile<T, U, false, D, G, EPL, LPR, RPL>(Kt, Vt, t * R, ntok, Br, nullptr, nullptr, alpha, scale,
                                                          st, zt, Bz, part_w, pbuf_w, lane);
    } else {
        for (int t = wave; t * RPL < ntok; t += NW)
            decode_tile<T, 1, true, D, G, EPL, LPR, RPL>(Kt, Vt, t * RPL, ntok, Br, pos + Br, nullptr, alpha, scale,
                                                         st, zt, Bz, part_w, pbuf_w, lane);
    }
    // residual slots (fp32 rows, log-count term) and the incoming token itself
    for (int t = wave; t * RPL < Br; t += NW)
        decode_tile<float, 1, true, D, G, EPL, LPR, RPL>(Kr, Vr, t * RPL, Br, 0, nullptr, w, alpha, scale,
                                                         st, zt, Bz, part_w, pbuf_w, lane);
    if (wave == NW - 1)
        decode_tile<T, 1, false, D, G, EPL, LPR, RPL>(knew, vnew, 0, 1, B, nullptr, nullptr, alpha, scale,
                                                      st, zt, Bz, part_w, pbuf_w, lane);

    // ---- combine the waves' partial softmaxes -> out ---------------------------------
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float ls = wave_sum(st.l[g]);
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            float v = st.acc[g][e];
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) v += __shfl_xor(v, o, 64);
            if (grp == 0) accw[(wave * G + g) * D + seg * EPL + e] = v;
        }
        if (lane == 0) { mw[wave * G + g] = st.m[g]; lw[wave * G + g] = ls; }
    }
    __syncthreads();
    for (int idx = tid; idx < G * D; idx += NT) {
        const int g = idx / D, c = idx % D;
        float M = -INFINITY;
#pragma unroll
        for (int x = 0; x < NW; ++x) M = fmaxf(M, mw[x * G + g]);
        float L = 0.f, o = 0.f;
#pragma unroll
        for (int x = 0; x < NW; ++x) {
            const float mx = mw[x * G + g];
            const float f = mx > -INFINITY ? __expf(mx - M) : 0.f;
            L += f * lw[x * G + g];
            o += f * accw[(x * G + g) * D + c];
        }
        a.out[(size_t)lu * G * D + idx] = o / L;
        if (c == 0) Mg[g] = M;
    }
    __syncthreads();

    // ---- D3: fp64 softmax over the stored logits, score update ------------------------
    {
        double lsum[G];
#pragma unroll
        for (int g = 0; g < G; ++g) lsum[g] = 0.0;
        for (int j = tid; j <= B; j += NT) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const double z = zt[(size_t)g * Bz + j];
                const double e = z == -INFINITY ? 0.0 : exp(z - (double)Mg[g]);
                zt[(size_t)g * Bz + j] = e;
                lsum[g] += e;
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const double t = wave_sum(lsum[g]);
            if (lane == 0) red64[wave * G + g] = t;
        }
        __syncthreads();
        if (tid < G) {
            double t = 0.0;
            for (int x = 0; x < NW; ++x) t += red64[x * G + tid];
            l64[tid] = t;
        }
        __syncthreads();
    }
    const double lam = (double)cv.lambda;
    const long long cand_hi = Tseen - Bp;   // evictable: position <= T - B_p (outside the latest B_p)
    unsigned long long best = ~0ull;
    int best_slot = -1;
    for (int j = tid; j < B; j += NT) {
        const int pj = pos[j];
        const bool occ = j < Br ? (w[j] > 0) : (pj >= 0);
        if (occ) {
            double pm = 0.0;
#pragma unroll
            for (int g = 0; g < G; ++g) pm += zt[(size_t)g * Bz + j] / l64[g];
            pm /= (double)G;
            const float sn = (float)(lam * (double)s[j] + pm);
            s[j] = sn;
            if (full && j >= Br && (long long)pj <= cand_hi) {
                const unsigned long long key = ((unsigned long long)__float_as_uint(sn) << 32) | (uint32_t)pj;
                if (key < best) { best = key; best_slot = j; }
            }
        } else if (!full && j >= Br) {
            const unsigned long long key = (unsigned long long)j;   // lowest free token slot
            if (key < best) { best = key; best_slot = j; }
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
        for (int g = 0; g < G; ++g) pm += zt[(size_t)g * Bz + B] / l64[g];
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

// Host side: pick the instantiation for (D, G) and launch one workgroup per unit.
template <typename T, int D, int G>
inline hipError_t launch_decode_dg(const DecodeArgs& a, hipStream_t stream) {
    constexpr int NW = 4, U = 4;
    using Sh = DecodeShape<T, D, G, NW, U>;
    const size_t lds = Sh::lds_bytes(a.cv.cap);
    auto kern = decode_kernel<T, D, G, NW, U>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(a.n_units), dim3(NW * 64), lds, stream, a);
    return hipGetLastError();
}

template <typename T, int D, int G>
inline size_t decode_lds_dg(int cap) { return DecodeShape<T, D, G, 4, 4>::lds_bytes(cap); }

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
