// Prefill compression kernels (see zsm_prefill.hpp).  All score arithmetic is fp64 (exact
// products, one rounding to the fp32 score at the end) so that the top-B_c selection does
// not depend on the summation order used here.
#include "zsm_prefill.hpp"

#include <type_traits>

namespace zsm {
namespace {

__device__ __forceinline__ double shfl_xor_d(double v, int o) { return __shfl_xor(v, o, 64); }

// a call covers the units of one or more whole layers: local unit lu = (layer * S + sequence) * H + head
__device__ __forceinline__ int seq_of(const CacheView& cv, int lu) { return (lu / cv.H) % cv.S; }

// the lengths live in device memory and cannot be checked on the host: clamp them here
__device__ __forceinline__ int seq_len_of(const PrefillArgs& a, int b) {
    const int t = a.seq_lens[b];
    return t < 0 ? 0 : (t > a.T_max ? a.T_max : t);
}

__device__ __forceinline__ double wave_max_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, shfl_xor_d(v, o));
    return v;
}

// ---- Q -> fp64 in the order the scoring kernels stage it, rows padded to a multiple of PF_MR with zeros
// Per (head, 32-row block): [row block rb of 16][matrix step c][lane l] = Q[row 16*rb + l%16][channel
// (4*(c/EPL) + l/16)*EPL + c%EPL]: lane l's A operand of step c (see pf_score_mfma), so that a workgroup
// stages a block with one contiguous 16-byte-per-lane copy.
template <typename T>
__global__ void pf_convert_q(const T* __restrict__ Q, double* __restrict__ Qd, int W, int Wp, int D, size_t n_heads) {
    constexpr int EPL = 16 / sizeof(T);
    const int nstep = D / 4;
    const size_t total = n_heads * Wp * D;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int l = (int)(i & 63);
        const int c = (int)((i >> 6) % nstep);
        const int rb = (int)((i / (64 * (size_t)nstep)) % (PF_MR / 16));
        const size_t blk = i / ((size_t)PF_MR * D);          // (head, 32-row block), Wp / PF_MR blocks per head
        const size_t h = blk / (Wp / PF_MR);
        const int r = (int)(blk % (Wp / PF_MR)) * PF_MR + 16 * rb + (l & 15);
        const int ch = (4 * (c / EPL) + (l >> 4)) * EPL + c % EPL;
        Qd[i] = r < W ? (double)to_float(Q[(h * W + r) * D + ch]) : 0.0;
    }
}

// ---- reference logit of every query row: the row's own key (Eq. 1 with t = i) -------------
// With fp64 exponentials a softmax row needs no running maximum, only a reference that keeps
// exp() in range; the query's logit against its own position is one.  A key whose logit is more
// than LOGIT_SPREAD_MAX (690) above it is clamped there; pf_row_combine raises the unit's
// FLAG_PREFILL_SPREAD when a row's denominator reaches SPREAD_FLAG_SUM, so the clamp never acts unseen.
template <typename T, int D>
__global__ __launch_bounds__(64) void pf_self_logit(PrefillArgs a, PrefillWs ws) {
    const CacheView& cv = a.cv;
    const int lu = blockIdx.y;
    const int b = seq_of(cv, lu);
    const int Tb = seq_len_of(a, b);
    const int nb = a.W < Tb ? a.W : Tb;
    const int G = cv.G;
    const int idx = blockIdx.x;             // g * Wp + r
    const int g = idx / ws.Wp, r = idx % ws.Wp;
    if (g >= G || r >= nb) return;
    const int lane = threadIdx.x;
    const T* q = reinterpret_cast<const T*>(a.Q) + (((size_t)lu * G + g) * a.W + r) * D;
    const T* k = reinterpret_cast<const T*>(a.K) + ((size_t)lu * a.T_max + (Tb - nb + r)) * D;
    double p = 0.0;
    for (int c = lane; c < D; c += 64) p = fma((double)to_float(q[c]), (double)to_float(k[c]), p);
    p = wave_sum(p);
    if (lane == 0) reinterpret_cast<double*>(a.ws + ws.rowm)[((size_t)lu * G + g) * ws.Wp + r] = p * cv.scale;
}

// ---- P1 / P2: logits of the window queries against the keys, on the fp64 matrix cores ------
// D = A x B with v_mfma_f64_16x16x4_f64: A = 16 query rows x 4 channels, B = 4 channels x 16
// keys, D = 16 x 16 logits accumulated over the D/4 channel steps.  Lane l supplies
// A[row l%16][channel l/16] and B[channel l/16][key l%16] and receives D[row l/16 + 4r][key l%16]
// in result register r.  Products of two values of the storage type are exact in fp64, so the
// logits are fp64 dot products whatever the summation order.
//   Keys: lane (key j = l%16, quarter q = l/16) loads the 16-byte pieces q, q+4, q+8, ... of its
//   key row; step c = u*EPL + e uses element e of piece 4u+q, i.e. channel (4u+q)*EPL + e.
//   Queries: the 32 rows of the pass live in LDS as fp64, permuted to that channel order, one
//   conflict-free 8-byte read per lane and step.
// A workgroup owns a range of keys of one unit; its four waves take wave tiles of 16*KB keys.
// MODE 0: l_i = sum over keys t <= i of exp(z_it - C_i) (the softmax denominator of Eq. 1), partial
//         per (row, workgroup) to the workspace.
// MODE 1: s_t = sum over rows of roww_i * exp(z_it - C_i)  (Eq. 3 unrolled over the window); with
//         one 32-row pass per unit the score is written at once, otherwise the passes add into sacc.
// MODE 2: MODE 0, and every exp(z_it - C_i) of a key that exists is stored at ev[t][row]; pf_score_from_ev
//         then forms s_t from there and K is swept once instead of twice.
typedef double d4_t __attribute__((ext_vector_type(4)));
typedef double d2_t __attribute__((ext_vector_type(2)));

template <typename T, int D, int MODE>
__global__ __launch_bounds__(256, MODE == 2 ? 3 : 4) void pf_score_mfma(PrefillArgs a, PrefillWs ws, const double* __restrict__ Qd,
                                                        const double* __restrict__ rowm,
                                                        const double* __restrict__ roww, double* __restrict__ pl,
                                                        double* __restrict__ sacc, float* __restrict__ sc,
                                                        double* __restrict__ evs) {
    constexpr int EPL = 16 / sizeof(T);            // elements per 16-byte piece
    constexpr int NSTEP = D / 4;                   // matrix steps (4 channels each) per tile
    constexpr int NLD = NSTEP / EPL;               // 16-byte pieces per lane and key
    constexpr int KB = sizeof(T) == 4 ? 1 : 2;     // 16-key blocks per wave tile
    constexpr int RB = PF_MR / 16;                 // 16-row blocks per pass
    constexpr int TK = 16 * KB;
    constexpr int NWV = 4;
    static_assert(PF_KQ % (NWV * 32) == 0, "");
    const CacheView& cv = a.cv;
    const int lu = (MODE == 2 ? ws.lu0 : 0) + blockIdx.y;   // MODE 2 launches cover units lu0, lu0 + 1, ...
    const int b = seq_of(cv, lu);
    const int Tb = seq_len_of(a, b);
    const int W = a.W, G = cv.G, Wp = ws.Wp;
    const int nb = W < Tb ? W : Tb;
    const int qpos0 = Tb - nb;                 // position of query row 0
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: tile numbers stay in scalar registers
    const int j = lane & 15, q = lane >> 4;
    const T* Kbase = reinterpret_cast<const T*>(a.K) + (size_t)lu * a.T_max * D;
    const double scale = cv.scale;
    __shared__ double Qs[RB * NSTEP * 64];
    __shared__ double rm[PF_MR], rw[PF_MR];
    __shared__ double red[NWV][PF_MR];

    // passes = (query head, 32-row block) pairs; this workgroup takes every rz-th one
    const int nblk = (nb + PF_MR - 1) / PF_MR;
    double* sacc_z = sacc + (size_t)blockIdx.z * gridDim.y * a.T_max;
    for (int half = 0; half < (ws.fold ? 2 : 1); ++half) {
    // key range of this round: x, then (folded launches) its mirror image nsums-1-x
    const int chunk = half == 0 ? (int)blockIdx.x : ws.nsums - 1 - (int)blockIdx.x;
    if (half == 1 && chunk <= (int)blockIdx.x) break;
    const int k0 = chunk * ws.chunk_keys;
    if (k0 >= Tb) continue;
    const int k1 = k0 + ws.chunk_keys < Tb ? k0 + ws.chunk_keys : Tb;
    for (int pass = blockIdx.z; pass < G * nblk; pass += gridDim.z) {
        const int g = pass / nblk;
        const size_t head = (size_t)lu * G + g;
        {
            const int r0 = (pass % nblk) * PF_MR;
            const int rlast = (r0 + PF_MR < nb ? r0 + PF_MR : nb) - 1;
            const size_t rowbase = head * Wp + r0;
            // keys past the last row's position are in the future of every row of this pass
            const int kend = k1 < qpos0 + rlast + 1 ? k1 : qpos0 + rlast + 1;
            if (k0 >= kend) {
                if (MODE != 1 && tid < PF_MR) pl[(rowbase + tid) * ws.nsums + chunk] = 0.0;
                continue;
            }
            __syncthreads();   // the previous pass has finished reading Qs / rm / rw
            {   // the block's query operands are stored in staging order: a contiguous copy
                const double2* src = reinterpret_cast<const double2*>(Qd + rowbase * D);   // rowbase is a multiple of 32
                double2* dst = reinterpret_cast<double2*>(Qs);
#pragma unroll
                for (int x = 0; x < RB * NSTEP * 64 / 2 / 256; ++x) dst[x * 256 + tid] = src[x * 256 + tid];
            }
            if (tid < PF_MR) {
                rm[tid] = rowm[rowbase + tid];
                rw[tid] = MODE == 1 ? roww[rowbase + tid] : 0.0;
            }
            __syncthreads();
            double lsum[RB][4];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int r = 0; r < 4; ++r) lsum[rb][r] = 0.0;

            // this lane's pieces of the wave's current tile; the next tile's pieces replace them one
            // by one as soon as the last step that needs them has been issued
            Raw<T, EPL> key[KB][NLD];
            auto piece = [&](int t0, int kb, int u) {
                const int t = t0 + 16 * kb + j;
                return Kbase + (size_t)(t < Tb ? t : Tb - 1) * D + (4 * u + q) * EPL;
            };
            int t0 = k0 + wave * TK;
            if (t0 < kend) {
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int u = 0; u < NLD; ++u) key[kb][u].load(piece(t0, kb, u));
            }
            for (; t0 < kend; t0 += NWV * TK) {
                const int tn = t0 + NWV * TK;
                d4_t acc[RB][KB];
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int kb = 0; kb < KB; ++kb) acc[rb][kb] = d4_t{0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int u = 0; u < NLD; ++u) {
#pragma unroll
                    for (int e = 0; e < EPL; ++e) {
                        const int c = u * EPL + e;
                        double av[RB], bv[KB];
#pragma unroll
                        for (int rb = 0; rb < RB; ++rb) av[rb] = Qs[(rb * NSTEP + c) * 64 + lane];
#pragma unroll
                        for (int kb = 0; kb < KB; ++kb) bv[kb] = (double)key[kb][u].get(e);
#pragma unroll
                        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                            for (int kb = 0; kb < KB; ++kb)
                                acc[rb][kb] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[rb], bv[kb], acc[rb][kb], 0, 0, 0);
                    }
                    if (tn < kend) {
#pragma unroll
                        for (int kb = 0; kb < KB; ++kb) key[kb][u].load(piece(tn, kb, u));
                    }
                    // keep each group of steps together: hoisting the later groups' LDS reads and
                    // conversions above this point costs more registers than there are
                    __builtin_amdgcn_sched_barrier(0);
                }
                // this lane holds the logits of rows 16*rb + q + 4*r against keys t0 + 16*kb + j
                double sp[KB];
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) sp[kb] = 0.0;
                // MODE 2: ev is [unit][key][G * Wp rows]; row 16*rb + 4*r of this lane sits a constant away from ep[kb]
                double* ep[KB];
                if (MODE == 2) {
#pragma unroll
                    for (int kb = 0; kb < KB; ++kb)
                        ep[kb] = evs + ((size_t)blockIdx.y * a.T_max + (t0 + 16 * kb + j)) * ((size_t)G * Wp) + (g * Wp + r0 + q);
                }
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int i = 16 * rb + q + 4 * r;
                        const bool valid = r0 + i < nb;
                        const int qp = qpos0 + r0 + i;     // the row's own position: keys up to it count (Eq. 1)
                        const double rmv = rm[i], rwv = rw[i];
#pragma unroll
                        for (int kb = 0; kb < KB; ++kb) {
                            const int t = t0 + 16 * kb + j;
                            const bool ok = valid && t <= qp;
                            const double ev = exp(fmin(acc[rb][kb][r] * scale - rmv, LOGIT_SPREAD_MAX));
                            if (MODE != 1) lsum[rb][r] += ok ? ev : 0.0;
                            else sp[kb] += ok ? rwv * ev : 0.0;
                            if (MODE == 2 && t < Tb) ep[kb][16 * rb + 4 * r] = ev;   // masked entries are never read back
                        }
                    }
                }
                if (MODE == 1) {
#pragma unroll
                    for (int kb = 0; kb < KB; ++kb) {
                        double v = sp[kb];
                        v += shfl_xor_d(v, 16);
                        v += shfl_xor_d(v, 32);
                        const int t = t0 + 16 * kb + j;
                        if (q == 0 && t < kend) {
                            const size_t o = (size_t)lu * a.T_max + t;
                            if (ws.multi) sacc_z[o] += v;   // this wave is the only one that touches key t in this group's array
                            else sc[o] = (float)v;
                        }
                    }
                }
            }
            if (MODE != 1) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        double v = lsum[rb][r];
#pragma unroll
                        for (int o = 1; o < 16; o <<= 1) v += shfl_xor_d(v, o);
                        if (j == 0) red[wave][16 * rb + q + 4 * r] = v;
                    }
                }
                __syncthreads();
                if (tid < PF_MR) {
                    double l = 0.0;
                    for (int x = 0; x < NWV; ++x) l += red[x][tid];
                    pl[(rowbase + tid) * ws.nsums + chunk] = l;
                }
            }
        }
    }
    }
}

// ---- P2 from the stored exponentials: s_t = sum over the window rows at or after t of roww_i * ev[t][i] ----
// Sixteen lanes per key: a key's G * Wp exponentials are contiguous, each lane takes two of every 32
// (one 16-byte load, the wave reads 1 KB in one piece) and the sixteen partial sums meet by shuffles.
__global__ __launch_bounds__(256) void pf_score_from_ev(PrefillArgs a, PrefillWs ws, const double* __restrict__ roww,
                                                        const double* __restrict__ evs, float* __restrict__ sc) {
    const CacheView& cv = a.cv;
    const int lu = ws.lu0 + blockIdx.y;
    const int Tb = seq_len_of(a, seq_of(cv, lu));
    const int nb = a.W < Tb ? a.W : Tb;
    const int qpos0 = Tb - nb;
    const int Wp = ws.Wp;
    const int rows = cv.G * Wp;                  // a multiple of 32
    const double* rw = roww + (size_t)lu * rows;
    const int sub = threadIdx.x & 15, kl = threadIdx.x >> 4;
    constexpr int KU = 4;                        // keys per 16-lane group and round: that many loads in flight
    for (int tb = blockIdx.x * 16 * KU; tb < Tb; tb += gridDim.x * 16 * KU) {
        double v[KU];
        int i0[KU];
        const double2* e[KU];
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            const int t = tb + u * 16 + kl;
            const int tc = t < Tb ? t : Tb - 1;
            e[u] = reinterpret_cast<const double2*>(evs + ((size_t)blockIdx.y * a.T_max + tc) * rows);
            i0[u] = tc > qpos0 ? tc - qpos0 : 0;   // first row whose position is at or after key t (Eq. 1: keys up to the row's own)
            v[u] = 0.0;
        }
        for (int c = 0; c < rows; c += 32) {
            const int r = c + 2 * sub, i = r % Wp;    // rows r and r + 1 belong to the same head (Wp is even)
            const double2 w = *reinterpret_cast<const double2*>(rw + r);
            d2_t x[KU];
#pragma unroll
            for (int u = 0; u < KU; ++u) x[u] = __builtin_nontemporal_load(reinterpret_cast<const d2_t*>(e[u]) + (r >> 1));   // read once, whole lines
#pragma unroll
            for (int u = 0; u < KU; ++u) {            // values outside the causal window were never written: not touched
                if (i >= i0[u] && i < nb) v[u] = fma(w.x, x[u].x, v[u]);
                if (i + 1 >= i0[u] && i + 1 < nb) v[u] = fma(w.y, x[u].y, v[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            double s = v[u];
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) s += shfl_xor_d(s, o);
            const int t = tb + u * 16 + kl;
            if (sub == 0 && t < Tb) sc[(size_t)lu * a.T_max + t] = (float)s;
        }
    }
}

// scores that passed through the fp64 accumulator (more than one pass per unit) -> fp32
__global__ void pf_sacc_to_sc(PrefillArgs a, const double* __restrict__ sacc, int rz, float* __restrict__ sc) {
    const int lu = blockIdx.y;
    const int Tb = seq_len_of(a, seq_of(a.cv, lu));
    const size_t zs = (size_t)gridDim.y * a.T_max;   // stride between the pass groups' arrays
    for (int t = blockIdx.x * blockDim.x + threadIdx.x; t < Tb; t += gridDim.x * blockDim.x) {
        double v = 0.0;
        for (int z = 0; z < rz; ++z) v += sacc[z * zs + (size_t)lu * a.T_max + t];
        sc[(size_t)lu * a.T_max + t] = (float)v;
    }
}

__global__ void pf_fill_f64(double* p, size_t n, double v) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// ---- P1b: combine the workgroups' partial denominators per query row ---------------------
__global__ void pf_row_combine(PrefillArgs a, PrefillWs ws) {
    const CacheView& cv = a.cv;
    const int lu = ws.lu0 + blockIdx.x;
    const int b = seq_of(cv, lu);
    const int Tb = seq_len_of(a, b);
    const int nb = a.W < Tb ? a.W : Tb;
    const int G = cv.G, Wp = ws.Wp;
    const double* pl = reinterpret_cast<const double*>(a.ws + ws.pl);
    double* roww = reinterpret_cast<double*>(a.ws + ws.roww);
    const int nt = (Tb + ws.chunk_keys - 1) / ws.chunk_keys;
    const double lam = (double)cv.lambda;
    for (int idx = threadIdx.x; idx < G * nb; idx += blockDim.x) {
        const int g = idx / nb, r = idx % nb;
        const size_t row = ((size_t)lu * G + g) * Wp + r;
        double L = 0.0;
        for (int x = 0; x < nt; ++x) L += pl[row * ws.nsums + x];
        if (L >= SPREAD_FLAG_SUM) atomicOr(cv.flags + a.unit0 + lu, FLAG_PREFILL_SPREAD);   // practically never taken
        roww[row] = pow(lam, (double)(nb - 1 - r)) / ((double)G * L);
    }
    // rows that pad the last 32-row pass carry no weight
    for (int idx = threadIdx.x; idx < G * (Wp - nb); idx += blockDim.x) {
        const int g = idx / (Wp - nb), r = nb + idx % (Wp - nb);
        roww[((size_t)lu * G + g) * Wp + r] = 0.0;
    }
}

// ---- P3: top-B_c selection and slot order ------------------------------------------------
// Radix select on the fp32 bit patterns (scores are >= 0, so the unsigned order is the value
// order), then an ordered compaction: kept = latest B_p, every score above the threshold,
// and the earliest positions among scores equal to it.
constexpr int SEL_NT = 1024;

__global__ __launch_bounds__(SEL_NT) void pf_select(PrefillArgs a, PrefillWs ws) {
    const CacheView& cv = a.cv;
    const int lu = blockIdx.x;
    const int ug = a.unit0 + lu;
    const int b = seq_of(cv, lu);
    const int Tb = seq_len_of(a, b);
    const int Bp = cv.Bp[b], Bc = cv.Bc[b];
    const int ntok = Bp + Bc;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t* sc = reinterpret_cast<const uint32_t*>(a.ws + ws.sc) + (size_t)lu * a.T_max;
    unsigned char* keep = reinterpret_cast<unsigned char*>(a.ws + ws.keep) + (size_t)lu * a.T_max;
    int32_t* kept_pos = reinterpret_cast<int32_t*>(a.ws + ws.kept_pos) + (size_t)lu * cv.cap_tok;
    int32_t* sel = reinterpret_cast<int32_t*>(a.ws + ws.sel) + (size_t)lu * 4;
    (void)ug;

    if (Tb <= ntok) {   // short prompt: everything is kept, in position order
        for (int t = tid; t < Tb; t += SEL_NT) { kept_pos[t] = t; keep[t] = 1; }
        if (tid == 0) { sel[0] = Tb; sel[1] = -1; }
        return;
    }
    const int N = Tb - Bp;   // candidates for the context set: positions [0, N)
    __shared__ int hist[256];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_k;
    uint32_t prefix = 0, mask = 0;
    int k = Bc;              // rank (from the top) still to find inside the prefix class
    if (Bc > 0) {
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            for (int t = tid; t < N; t += SEL_NT) {
                const uint32_t v = sc[t];
                if ((v & mask) == prefix) atomicAdd(&hist[(v >> shift) & 255], 1);
            }
            __syncthreads();
            if (tid == 0) {
                int kk = k, bin = 255;
                for (; bin > 0; --bin) {
                    if (hist[bin] >= kk) break;
                    kk -= hist[bin];
                }
                sh_prefix = prefix | ((uint32_t)bin << shift);
                sh_k = kk;
            }
            __syncthreads();
            prefix = sh_prefix;
            k = sh_k;
            mask |= 255u << shift;
            __syncthreads();
        }
    }
    // prefix = bit pattern of the B_c-th largest score; k = how many equal to it are kept
    const uint32_t thr = prefix;
    const int r_eq = Bc > 0 ? k : 0;
    __shared__ unsigned long long wsum[SEL_NT / 64];
    __shared__ unsigned long long carry_sh;
    __shared__ int first_drop;
    if (tid == 0) { carry_sh = 0; first_drop = 0x7fffffff; }
    __syncthreads();
    for (int c0 = 0; c0 < N; c0 += SEL_NT) {
        const int t = c0 + tid;
        uint32_t v = 0;
        bool gt = false, eq = false;
        if (t < N && Bc > 0) { v = sc[t]; gt = v > thr; eq = v == thr; }
        const unsigned long long mine = ((unsigned long long)gt << 32) | (unsigned long long)eq;
        // inclusive scan inside the wave, then across waves
        unsigned long long inc = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const unsigned long long up = __shfl_up(inc, o, 64);
            if (lane >= o) inc += up;
        }
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        unsigned long long base = carry_sh;
        for (int x = 0; x < wave; ++x) base += wsum[x];
        const unsigned long long exc = base + inc - mine;
        const int gt_before = (int)(exc >> 32), eq_before = (int)(exc & 0xffffffffull);
        if (t < N) {
            const bool kp = gt || (eq && eq_before < r_eq);
            keep[t] = kp ? 1 : 0;
            if (kp) kept_pos[gt_before + (eq_before < r_eq ? eq_before : r_eq)] = t;
            else atomicMin(&first_drop, t);
        }
        __syncthreads();
        if (tid == SEL_NT - 1) carry_sh = base + inc;
        __syncthreads();
    }
    for (int i = tid; i < Bp; i += SEL_NT) { kept_pos[Bc + i] = N + i; keep[N + i] = 1; }
    __syncthreads();
    if (tid == 0) { sel[0] = ntok; sel[1] = first_drop; }
}

// The same selection for prompts of up to SEL_NT * SEL_NPT candidates, with the scores held in
// registers (candidate k*SEL_NT + tid in register k): the B_c-th largest bit pattern is found
// bit by bit (31 counting steps of ballots, no histogram and no memory traffic), the ordered
// compaction takes one block scan over the (register, wave) ballot counts.
constexpr int SEL_NPT = 64;

__global__ __launch_bounds__(SEL_NT) void pf_select_reg(PrefillArgs a, PrefillWs ws) {
    const CacheView& cv = a.cv;
    const int lu = blockIdx.x;
    const int b = seq_of(cv, lu);
    const int Tb = seq_len_of(a, b);
    const int Bp = cv.Bp[b], Bc = cv.Bc[b];
    const int ntok = Bp + Bc;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int NWV = SEL_NT / 64;
    const uint32_t* sc = reinterpret_cast<const uint32_t*>(a.ws + ws.sc) + (size_t)lu * a.T_max;
    unsigned char* keep = reinterpret_cast<unsigned char*>(a.ws + ws.keep) + (size_t)lu * a.T_max;
    int32_t* kept_pos = reinterpret_cast<int32_t*>(a.ws + ws.kept_pos) + (size_t)lu * cv.cap_tok;
    int32_t* sel = reinterpret_cast<int32_t*>(a.ws + ws.sel) + (size_t)lu * 4;

    if (Tb <= ntok) {   // short prompt: everything is kept, in position order
        for (int t = tid; t < Tb; t += SEL_NT) { kept_pos[t] = t; keep[t] = 1; }
        if (tid == 0) { sel[0] = Tb; sel[1] = -1; }
        return;
    }
    const int N = Tb - Bp;   // candidates for the context set: positions [0, N)
    const int nk = (N + SEL_NT - 1) / SEL_NT;   // registers in use (<= SEL_NPT, checked by the host)
    uint32_t v[SEL_NPT];
#pragma unroll
    for (int k = 0; k < SEL_NPT; ++k) {
        // branch-free: a candidate index past the end reads the last candidate and is zeroed
        const int t = k * SEL_NT + tid;
        const uint32_t x = sc[min(t, N - 1)];
        v[k] = x & (uint32_t)((t - N) >> 31);   // all ones where t < N
        if (k % 16 == 15) __builtin_amdgcn_sched_barrier(0);   // sixteen loads in flight at a time
    }
    __shared__ int wcnt[2][NWV];
    __shared__ unsigned long long cnt2[SEL_NPT * NWV];   // per (register, wave): (greater << 32 | equal), then their exclusive scan
    __shared__ unsigned long long mgt[SEL_NPT * NWV], meq[SEL_NPT * NWV];   // the ballots themselves
    __shared__ unsigned long long wsum[NWV];
    __shared__ int first_drop;
    if (tid == 0) first_drop = 0x7fffffff;

    // number of candidates whose pattern is >= c (every thread gets the same answer)
    auto count_ge = [&](uint32_t c, int par) {
        int n = 0;   // this lane's count; registers past nk and candidates past N hold 0 and are not counted (c > 0)
#pragma unroll
        for (int k = 0; k < SEL_NPT; ++k) n += v[k] >= c ? 1 : 0;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) n += __shfl_xor(n, o, 64);
        if (lane == 0) wcnt[par][wave] = n;
        __syncthreads();
        int tot = 0;
#pragma unroll
        for (int x = 0; x < NWV; ++x) tot += wcnt[par][x];
        return tot;
    };
    uint32_t thr = 0xffffffffu;   // B_c = 0: nothing is above or equal
    int r_eq = 0;
    if (Bc > 0) {
        thr = 0;
        // scores are >= 0: bit 31 is clear, the unsigned order of the patterns is the value order
        int par = 0;
        for (int bit = 30; bit >= 0; --bit) {
            const uint32_t c = thr | (1u << bit);
            if (count_ge(c, par) >= Bc) thr = c;   // at least B_c candidates reach c: the B_c-th largest does too
            par ^= 1;
        }
        // thr = pattern of the B_c-th largest score; r_eq = how many equal to it are kept
        const int n_gt = thr == 0xffffffffu ? 0 : count_ge(thr + 1u, par);
        r_eq = Bc - n_gt;
    }
    __syncthreads();
    // ordered compaction: kept = every score above thr and the first r_eq equal to it, in position order
#pragma unroll
    for (int k = 0; k < SEL_NPT; ++k) {
        if (k < nk) {
            // registers of candidates past N hold 0: never above thr, and where they equal it (thr = 0)
            // they come after every real candidate in position order, so none of them is among the r_eq kept
            const unsigned long long bg = __ballot(v[k] > thr), be = __ballot(v[k] == thr);
            if (lane == 0) {
                cnt2[k * NWV + wave] = ((unsigned long long)__popcll(bg) << 32) | (unsigned long long)__popcll(be);
                mgt[k * NWV + wave] = bg;
                meq[k * NWV + wave] = be;
            }
        }
        __builtin_amdgcn_sched_barrier(0);   // one pair of ballots at a time: they live in scalar registers
    }
    __syncthreads();
    {   // exclusive scan of the nk * NWV counts in (register, wave) order = position order
        const int ne = nk * NWV;   // <= SEL_NT
        const unsigned long long mine = tid < ne ? cnt2[tid] : 0ull;
        unsigned long long inc = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const unsigned long long up = __shfl_up(inc, o, 64);
            if (lane >= o) inc += up;
        }
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        unsigned long long base = 0;
        for (int x = 0; x < wave; ++x) base += wsum[x];
        if (tid < ne) cnt2[tid] = base + inc - mine;
    }
    __syncthreads();
    int my_first_drop = 0x7fffffff;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    // The compiler would otherwise keep the 64 lane masks of "t < N" from the loads above alive in
    // scalar registers (and spill them); an opaque copy of N makes it compare again here.
    int Nv = N;
    asm volatile("" : "+s"(Nv));
#pragma unroll
    for (int k = 0; k < SEL_NPT; ++k) {
        if (k < nk) {
            const int t = k * SEL_NT + tid;
            const unsigned long long bg = mgt[k * NWV + wave], be = meq[k * NWV + wave];   // the ballots taken above
            const bool gt = (bg >> lane) & 1ull, eq = (be >> lane) & 1ull;
            const unsigned long long base = cnt2[k * NWV + wave];
            const int gt_before = (int)(base >> 32) + __popcll(bg & lt_mask);
            const int eq_before = (int)(base & 0xffffffffull) + __popcll(be & lt_mask);
            if (t < Nv) {
                const bool kp = gt || (eq && eq_before < r_eq);
                keep[t] = kp ? 1 : 0;
                if (kp) kept_pos[gt_before + (eq_before < r_eq ? eq_before : r_eq)] = t;
                else my_first_drop = t < my_first_drop ? t : my_first_drop;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    if (my_first_drop != 0x7fffffff) atomicMin(&first_drop, my_first_drop);
    for (int i = tid; i < Bp; i += SEL_NT) { kept_pos[Bc + i] = N + i; keep[N + i] = 1; }
    __syncthreads();
    if (tid == 0) { sel[0] = ntok; sel[1] = first_drop; }
}

// ---- P4: gather the kept rows into their slots, write all slot metadata ------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void pf_gather(PrefillArgs a, PrefillWs ws) {
    const CacheView& cv = a.cv;
    const int lu = blockIdx.y;
    const int ug = a.unit0 + lu;
    const int b = seq_of(cv, lu);
    const int Tb = seq_len_of(a, b);
    const int Br = cv.Br;
    const int32_t* kept_pos = reinterpret_cast<const int32_t*>(a.ws + ws.kept_pos) + (size_t)lu * cv.cap_tok;
    const int32_t* sel = reinterpret_cast<const int32_t*>(a.ws + ws.sel) + (size_t)lu * 4;
    const float* sc = reinterpret_cast<const float*>(a.ws + ws.sc) + (size_t)lu * a.T_max;
    const int nkept = sel[0];
    constexpr int EPL = 16 / sizeof(T), LPR = D / EPL, RPB = 256 / LPR;   // rows per block pass
    const T* Ksrc = reinterpret_cast<const T*>(a.K) + (size_t)lu * a.T_max * D;
    const T* Vsrc = reinterpret_cast<const T*>(a.V) + (size_t)lu * a.T_max * D;
    T* Kt = reinterpret_cast<T*>(cv.Kt) + (size_t)ug * cv.cap_tok * D;
    T* Vt = reinterpret_cast<T*>(cv.Vt) + (size_t)ug * cv.cap_tok * D;
    const int tid = threadIdx.x;
    const int j0 = blockIdx.x * RPB * 4;
    for (int p = 0; p < 4; ++p) {
        const int j = j0 + p * RPB + tid / LPR;
        if (j < nkept) {
            const int t = kept_pos[j];
            const int sg = (tid % LPR) * EPL;
            const uint4 kv = *reinterpret_cast<const uint4*>(Ksrc + (size_t)t * D + sg);
            const uint4 vv = *reinterpret_cast<const uint4*>(Vsrc + (size_t)t * D + sg);
            *reinterpret_cast<uint4*>(Kt + (size_t)j * D + sg) = kv;
            *reinterpret_cast<uint4*>(Vt + (size_t)j * D + sg) = vv;
        }
    }
    // metadata of every token slot in this block's range, and (block 0) unit header
    float* s = cv.s + (size_t)ug * cv.cap;
    int32_t* pos = cv.pos + (size_t)ug * cv.cap;
    int32_t* w = cv.w + (size_t)ug * cv.cap;
    for (int j = j0 + tid; j < j0 + RPB * 4 && j < cv.cap_tok; j += 256) {
        if (j < nkept) {
            const int t = kept_pos[j];
            pos[Br + j] = t; w[Br + j] = 1; s[Br + j] = sc[t];
        } else {
            pos[Br + j] = -1; w[Br + j] = 0; s[Br + j] = 0.f;
        }
    }
    if (blockIdx.x == 0 && tid == 0) {
        cv.n_seen[ug] = Tb;
        cv.n_occ[ug] = nkept;
    }
}

// ---- P5: sum of the rows that were not kept ------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void pf_residual_partial(PrefillArgs a, PrefillWs ws) {
    const CacheView& cv = a.cv;
    const int lu = blockIdx.y;
    const int b = seq_of(cv, lu);
    const int Tb = seq_len_of(a, b);
    const int chunk = blockIdx.x;
    const int t0 = chunk * PF_RC;
    double* rsum = reinterpret_cast<double*>(a.ws + ws.rsum) + ((size_t)lu * ws.nchunks + chunk) * 2 * D;
    const int tid = threadIdx.x;
    constexpr int EPL = 16 / sizeof(T), LPR = D / EPL, RPB = 256 / LPR;
    const int seg = tid % LPR, rg = tid / LPR;
    __shared__ double red[2][RPB][D + 1];
    double ak[EPL], av[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) { ak[e] = 0.0; av[e] = 0.0; }
    if (t0 < Tb) {
        const unsigned char* keep = reinterpret_cast<const unsigned char*>(a.ws + ws.keep) + (size_t)lu * a.T_max;
        const T* Ksrc = reinterpret_cast<const T*>(a.K) + (size_t)lu * a.T_max * D;
        const T* Vsrc = reinterpret_cast<const T*>(a.V) + (size_t)lu * a.T_max * D;
        const int t1 = t0 + PF_RC < Tb ? t0 + PF_RC : Tb;
        // Branch-free and four rows deep: most rows are absorbed, so every row is loaded (a row index
        // past the end reads the last row) and a kept row adds nothing; the loads of four rows are in
        // flight together.
        constexpr int UR = 4;
        for (int tb = t0 + rg; tb < t1; tb += UR * RPB) {
            Raw<T, EPL> kr[UR], vr[UR];
            bool use[UR];
#pragma unroll
            for (int x = 0; x < UR; ++x) {
                const int t = tb + x * RPB;
                const int tc = t < t1 ? t : t1 - 1;
                use[x] = t < t1 && keep[tc] == 0;
                kr[x].load_nt(Ksrc + (size_t)tc * D + seg * EPL);
                vr[x].load_nt(Vsrc + (size_t)tc * D + seg * EPL);
            }
#pragma unroll
            for (int x = 0; x < UR; ++x) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    ak[e] += use[x] ? (double)kr[x].get(e) : 0.0;
                    av[e] += use[x] ? (double)vr[x].get(e) : 0.0;
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) { red[0][rg][seg * EPL + e] = ak[e]; red[1][rg][seg * EPL + e] = av[e]; }
    __syncthreads();
    for (int i = tid; i < 2 * D; i += 256) {
        const int which = i / D, c = i % D;
        double t = 0.0;
        for (int r = 0; r < RPB; ++r) t += red[which][r][c];
        rsum[i] = t;
    }
}

template <int D>
__global__ __launch_bounds__(256) void pf_residual_final(PrefillArgs a, PrefillWs ws) {
    const CacheView& cv = a.cv;
    const int lu = blockIdx.x;
    const int ug = a.unit0 + lu;
    const int b = seq_of(cv, lu);
    const int Tb = seq_len_of(a, b);
    const int Br = cv.Br;
    const int32_t* sel = reinterpret_cast<const int32_t*>(a.ws + ws.sel) + (size_t)lu * 4;
    const int nkept = sel[0], first_drop = sel[1];
    const int ndrop = Tb - nkept;
    float* s = cv.s + (size_t)ug * cv.cap;
    int32_t* pos = cv.pos + (size_t)ug * cv.cap;
    int32_t* w = cv.w + (size_t)ug * cv.cap;
    float* Kr = cv.Kr + (size_t)ug * Br * D;
    float* Vr = cv.Vr + (size_t)ug * Br * D;
    const int tid = threadIdx.x;
    if (Br == 0) return;
    if (ndrop <= 0) {
        for (int i = tid; i < Br * D; i += 256) { Kr[i] = 0.f; Vr[i] = 0.f; }
        if (tid < Br) { w[tid] = 0; pos[tid] = -1; s[tid] = 0.f; }
        return;
    }
    const double* rsum = reinterpret_cast<const double*>(a.ws + ws.rsum) + (size_t)lu * ws.nchunks * 2 * D;
    const int nch = (Tb + PF_RC - 1) / PF_RC;
    for (int i = tid; i < 2 * D; i += 256) {
        double t = 0.0;
        int c = 0;
        for (; c + 8 <= nch; c += 8) {   // eight partial sums requested together, added in chunk order
            double x[8];
#pragma unroll
            for (int y = 0; y < 8; ++y) x[y] = rsum[(size_t)(c + y) * 2 * D + i];
#pragma unroll
            for (int y = 0; y < 8; ++y) t += x[y];
        }
        for (; c < nch; ++c) t += rsum[(size_t)c * 2 * D + i];
        const float m = (float)(t / (double)ndrop);
        if (i < D) Kr[i] = m; else Vr[i - D] = m;
    }
    if (tid == 0 && first_drop >= 0 && first_drop < Tb) {
        // the slot was opened by the first absorbed token and carries its position and score
        w[0] = ndrop; pos[0] = first_drop;
        s[0] = reinterpret_cast<const float*>(a.ws + ws.sc)[(size_t)lu * a.T_max + first_drop];
    }
}

// ---- P5 for B_r >= 2, block form ---------------------------------------------------------
// The same walk (Alg. 1's residual branch token by token, Eq. 5 and Eq. 6, one wave per unit),
// organised so that the work per token that has to wait for the previous token's merge is small:
//   * Per block of 16 positions the dot products of all 16 tokens with all residual keys are one
//     fp64 matrix product on the matrix cores (v_mfma_f64_16x16x4: tokens x channels times
//     channels x keys, 16 keys per column block), and so is the block's Gram matrix x_i . x_j.
//   * A merge changes one key: k' = (w k + x_i) / (w + 1), rounded to fp32.  For the later tokens
//     j of the block only that key's column changes, to k' . x_j = (w (k . x_j) + x_i . x_j) / (w + 1)
//     up to the rounding of k' to fp32, which moves the dot product by at most
//     2^-24 |k'| |x_j|.  So the column is updated from the Gram row in a few instructions, and
//     the error that the skipped re-evaluation leaves is bounded: each merge adds at most
//     2^-23 * n(k') * X to the column's error, n(k') = (w n(k) + |x_i|) / (w + 1) being a running
//     bound of the key's norm (a mean of tokens; exact when the last slot was opened) and X the
//     largest token norm of the block.  E is the largest such error over the columns.
//   * A choice is taken from these values only when the best exceeds the runner-up by more than
//     2E; otherwise the token's dot products are re-evaluated from the stored fp32 keys, as
//     they are while the residual slots are still being opened.  Choices are therefore the ones
//     an evaluation from the stored keys gives.  Best and runner-up come from two 16-lane
//     maxima over integer order keys of the dot products with the slot index in the low bits
//     (v_max_i32 / v_max_u32 with DPP operands: one instruction per exchange).
//   * Eq. 6's quotient is formed with the correctly rounded reciprocal of w + 1 and one
//     residual correction (q0 = n r, q = q0 + (n - q0 d) r), which is the correctly rounded
//     quotient n / d for integer d, so the stored means are what a division gives.
constexpr int PF_RMAX = 64;   // residual slots the wave can own
constexpr int PF_GB = 16;     // positions per block

// every pattern used here reads a lane that exists, so the destination needs no prior value (bound_ctrl)
template <int CTRL>
__device__ __forceinline__ int dpp_mov_i(int v) { return __builtin_amdgcn_mov_dpp(v, CTRL, 0xf, 0xf, true); }
template <int CTRL>
__device__ __forceinline__ double dpp_mov_d(double v) {
    return __hiloint2double(dpp_mov_i<CTRL>(__double2hiint(v)), dpp_mov_i<CTRL>(__double2loint(v)));
}
// the larger of two doubles that are never NaN (a compare and two selects: no canonicalisation)
__device__ __forceinline__ double max_d(double a, double b) { return a > b ? a : b; }
// Arg-max of (value, index) over the lanes of each 16-lane row by four DPP exchanges (lane pairs
// i^1, i^2, i <-> 7-i, i <-> 15-i: after them every lane of a row holds the row's winner), ties to
// the lower index; no LDS round trip and no compare chain.
template <int CTRL>
__device__ __forceinline__ void dpp_argmax_step(double& v, int& idx) {
    const double v2 = dpp_mov_d<CTRL>(v);
    const int i2 = dpp_mov_i<CTRL>(idx);
    const bool take = (v2 > v) | ((v2 == v) & (i2 < idx));
    v = take ? v2 : v;
    idx = take ? i2 : idx;
}
__device__ __forceinline__ void row_argmax(double& v, int& idx) {
    dpp_argmax_step<0xB1>(v, idx);    // quad_perm [1,0,3,2]
    dpp_argmax_step<0x4E>(v, idx);    // quad_perm [2,3,0,1]
    dpp_argmax_step<0x141>(v, idx);   // row_half_mirror
    dpp_argmax_step<0x140>(v, idx);   // row_mirror
}
__device__ __forceinline__ double row_max(double v) {
    v = max_d(v, dpp_mov_d<0xB1>(v));
    v = max_d(v, dpp_mov_d<0x4E>(v));
    v = max_d(v, dpp_mov_d<0x141>(v));
    v = max_d(v, dpp_mov_d<0x140>(v));
    return v;
}
// Order key of a dot product: two 32-bit words (hi compared signed, lo unsigned) that order as the doubles do,
// with the key's index in the six lowest bits of lo (which moves the value by less than 2^-46 of itself) so that
// the largest key names the arg-max, the lower index winning between equal dot products.
struct OrdKey { int hi; uint32_t lo; };
__device__ __forceinline__ OrdKey ord_key(double v, int idx) {
    const int h = __double2hiint(v);
    const int sgn = h >> 31;                                  // all ones for negative values
    OrdKey k;
    k.hi = h ^ (sgn & 0x7fffffff);
    k.lo = (((uint32_t)__double2loint(v) ^ (uint32_t)sgn) & ~63u) | (uint32_t)(63 - idx);
    return k;
}
__device__ __forceinline__ double ord_value(int hi, uint32_t lo) {   // the (tagged) double behind a key
    const int sgn = hi >> 31;
    return __hiloint2double(hi ^ (sgn & 0x7fffffff), (int)(lo ^ (uint32_t)sgn));
}
__device__ __forceinline__ bool ord_less(const OrdKey& a, const OrdKey& b) { return a.hi < b.hi || (a.hi == b.hi && a.lo < b.lo); }
// maximum over the 16 lanes of each row: the high words first, then the low words of the lanes that hold that high word
template <int CTRL>
__device__ __forceinline__ int dpp_max_i(int v) { const int o = dpp_mov_i<CTRL>(v); return o > v ? o : v; }
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_max_u(uint32_t v) { const uint32_t o = (uint32_t)dpp_mov_i<CTRL>((int)v); return o > v ? o : v; }
__device__ __forceinline__ OrdKey row_max_key(const OrdKey& k) {
    int h = k.hi;
    h = dpp_max_i<0xB1>(h); h = dpp_max_i<0x4E>(h); h = dpp_max_i<0x141>(h); h = dpp_max_i<0x140>(h);
    uint32_t l = k.hi == h ? k.lo : 0u;
    l = dpp_max_u<0xB1>(l); l = dpp_max_u<0x4E>(l); l = dpp_max_u<0x141>(l); l = dpp_max_u<0x140>(l);
    return OrdKey{h, l};
}
__device__ __forceinline__ double readlane_d(double v, int l) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), l), __builtin_amdgcn_readlane(__double2loint(v), l));
}

// State of the walk that lives in registers while whole blocks are absorbed.
template <int NCB>
struct BlockCols {
    double dv[NCB][4];  // dot products: lane l holds token 4r + l/16 against key 16cb + l%16 in dv[cb][r]
    double gram[4];     // x_a . x_b: token a = 4r + l/16, token b = l%16, in gram[r]
    int wreg[NCB];      // fusion count of key 16cb + l%16
    double knorm[NCB];  // upper bound of that key's norm
    double cerr[NCB];   // how far this block's updated dot products of that key may be from what the stored key gives
    double xnorm;       // norm of token l%16 (valid in the lane whose row group l/16 is that token's: l/16 = (l%16) % 4)
};

// bytes of LDS one wave (one unit) of pf_residual_blocks needs
template <typename T, int D>
inline size_t pf_residual_blocks_lds(int Br) {
    const size_t n = sizeof(float) * 2 * (size_t)Br * (D + 4) + sizeof(double) * D + sizeof(int) * PF_RMAX + 2 * PF_GB * D * sizeof(T);
    return (n + 15) & ~(size_t)15;
}

// One wave per unit, `blockDim.x / 64` units per workgroup.  The waves of a workgroup never meet (no barrier, a region
// of LDS each): they are put in one workgroup because its waves are dealt to the four SIMDs of a compute unit one
// each, while single-wave workgroups were seen to share SIMDs from the third per compute unit on (the walk of 1024
// units then took 55 ms instead of the 37 ms of 512 units: two waves on one SIMD take turns on its matrix core).
template <typename T, int D, int NCB>
__global__ __launch_bounds__(256, 1) void pf_residual_blocks(PrefillArgs a, PrefillWs ws, int lds_per_wave) {
    const CacheView& cv = a.cv;
    const int wave_in_wg = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int lu = blockIdx.x * ((int)blockDim.x >> 6) + wave_in_wg;
    if (lu >= a.n_units) return;
    const int ug = a.unit0 + lu;
    const int b = seq_of(cv, lu);
    const int Tb = seq_len_of(a, b);
    const int Br = cv.Br;
    const int lane = threadIdx.x & 63;
    constexpr int RS = D + 4;   // padded row stride (floats): lanes reading 16 bytes of different rows hit different banks
    constexpr int CPL = D / 64; // channels per lane in the merge: CPL * lane .. CPL * lane + CPL - 1
    constexpr int EPL = 16 / sizeof(T);
    constexpr int SPK = D / 4;                // matrix steps; lane (i = l%16, k = l/16) owns channels SPK*k .. SPK*k + SPK-1 of row i
    constexpr int NLD = SPK / EPL;            // 16-byte pieces per lane, row and array
    static_assert(SPK % EPL == 0 && NLD >= 1, "");
    extern __shared__ __align__(16) unsigned char smem[];
    float* Krs = reinterpret_cast<float*>(smem + (size_t)wave_in_wg * lds_per_wave);   // [Br][RS]
    float* Vrs = Krs + (size_t)Br * RS;                      // [Br][RS]
    double* ktok = reinterpret_cast<double*>(Vrs + (size_t)Br * RS);   // [D]
    int* wcs = reinterpret_cast<int*>(ktok + D);             // [PF_RMAX] fusion counts
    T* Kst = reinterpret_cast<T*>(wcs + PF_RMAX);            // [PF_GB][D] rows of the current block
    T* Vst = Kst + PF_GB * D;
    float* s = cv.s + (size_t)ug * cv.cap;
    int32_t* pos = cv.pos + (size_t)ug * cv.cap;
    int32_t* w = cv.w + (size_t)ug * cv.cap;
    float* Kr = cv.Kr + (size_t)ug * Br * D;
    float* Vr = cv.Vr + (size_t)ug * Br * D;
    const unsigned char* keep = reinterpret_cast<const unsigned char*>(a.ws + ws.keep) + (size_t)lu * a.T_max;
    const float* sc = reinterpret_cast<const float*>(a.ws + ws.sc) + (size_t)lu * a.T_max;
    const T* Ksrc = reinterpret_cast<const T*>(a.K) + (size_t)lu * a.T_max * D;
    const T* Vsrc = reinterpret_cast<const T*>(a.V) + (size_t)lu * a.T_max * D;
    const int ti = lane & 15, tk = lane >> 4;   // this lane's row of a block and its quarter of the channels

    for (int i = lane; i < Br * RS; i += 64) { Krs[i] = 0.f; Vrs[i] = 0.f; }
    for (int i = lane; i < PF_RMAX; i += 64) wcs[i] = 0;
    int n_open = 0;        // residual slots opened so far (wave-uniform)

    // ---- one token the slow way: its dot products from the stored keys (Eq. 5), lane r against key r
    auto exact_choice = [&](int i) -> int {
        wave_sync();
        for (int c = lane; c < D; c += 64) ktok[c] = (double)to_float(Kst[i * D + c]);
        wave_sync();
        double dot = -INFINITY;
        if (lane < Br) {
            double p0_ = 0.0, p1_ = 0.0, p2_ = 0.0, p3_ = 0.0;
            const float* kr = Krs + lane * RS;
#pragma unroll 4
            for (int c = 0; c < D; c += 4) {
                const float4 kv = *reinterpret_cast<const float4*>(kr + c);
                p0_ = fma((double)kv.x, ktok[c + 0], p0_);
                p1_ = fma((double)kv.y, ktok[c + 1], p1_);
                p2_ = fma((double)kv.z, ktok[c + 2], p2_);
                p3_ = fma((double)kv.w, ktok[c + 3], p3_);
            }
            dot = (p0_ + p1_) + (p2_ + p3_);
        }
        int rbest = lane;
        row_argmax(dot, rbest);
        // the four rows' winners meet in scalar registers; the lower row wins a tie (its indices are lower)
        double bd = readlane_d(dot, 0);
        int br = __builtin_amdgcn_readlane(rbest, 0);
#pragma unroll
        for (int row = 1; row < 4; ++row) {
            const double d2 = readlane_d(dot, 16 * row);
            const int r2 = __builtin_amdgcn_readlane(rbest, 16 * row);
            if (d2 > bd) { bd = d2; br = r2; }
        }
        return br;
    };

    // ---- Eq. 6 for token i of the block into residual slot r (count wi before the merge, rinv = 1 / (wi + 1))
    auto merge_into = [&](int i, int r, int wi, double rinv) {
        const double wd = (double)wi, dd = wd + 1.0;
        float kc[CPL], vc[CPL];
#pragma unroll
        for (int x = 0; x < CPL; ++x) {
            kc[x] = to_float(Kst[i * D + CPL * lane + x]);
            vc[x] = to_float(Vst[i * D + CPL * lane + x]);
        }
#pragma unroll
        for (int x = 0; x < CPL; ++x) {
            const int c = CPL * lane + x;
            const double nk = fma(wd, (double)Krs[r * RS + c], (double)kc[x]);   // w * k is exact in fp64: this is the rounded sum
            const double nv = fma(wd, (double)Vrs[r * RS + c], (double)vc[x]);
            double qk = nk * rinv, qv = nv * rinv;
            qk = fma(fma(-qk, dd, nk), rinv, qk);    // the correctly rounded quotient nk / dd
            qv = fma(fma(-qv, dd, nv), rinv, qv);
            Krs[r * RS + c] = (float)qk;
            Vrs[r * RS + c] = (float)qv;
        }
        if (lane == 0) wcs[r] = wi + 1;
    };

    // a block's rows and flags, requested one block ahead: lane (i, k) takes its quarter of row i
    Raw<T, EPL> kreg[NLD], vreg[NLD];
    int kflag = 1;
    auto request = [&](int p0) {   // positions [p0, p0 + PF_GB); rows past the prompt read its last row
        const int row = p0 + ti;
        const size_t off = (size_t)(row < Tb ? row : Tb - 1) * D + SPK * tk;
#pragma unroll
        for (int x = 0; x < NLD; ++x) {
            kreg[x].load(Ksrc + off + x * EPL);
            vreg[x].load(Vsrc + off + x * EPL);
        }
        const int t = p0 + lane;
        kflag = (lane < PF_GB && t < Tb) ? keep[t] : 1;   // 1 = not to be absorbed
    };

    BlockCols<NCB> st;
    bool fast = false;        // every residual slot is open: whole blocks go through the matrix cores

    if (Tb > 0) request(0);
    for (int p0 = 0; p0 < Tb; p0 += PF_GB) {
        wave_sync();   // the previous block's rows are no longer read
        double xd[SPK];       // this lane's channels of its row, fp64: the A operand (and, for the Gram matrix, the B operand)
#pragma unroll
        for (int x = 0; x < NLD; ++x) {
            *reinterpret_cast<Raw<T, EPL>*>(Kst + (size_t)ti * D + SPK * tk + x * EPL) = kreg[x];
            *reinterpret_cast<Raw<T, EPL>*>(Vst + (size_t)ti * D + SPK * tk + x * EPL) = vreg[x];
#pragma unroll
            for (int e = 0; e < EPL; ++e) xd[x * EPL + e] = (double)kreg[x].get(e);
        }
        const unsigned long long todo = __ballot(kflag == 0);   // bit i: position p0 + i is absorbed
        if (p0 + PF_GB < Tb) request(p0 + PF_GB);
        wave_sync();
        if (todo == 0ull) continue;

        if (!fast) {
            // the residual set still has room (Alg. 1: the token opens the next slot), or the block began that way
            unsigned long long td = todo;
            while (td) {
                const int i = __builtin_ctzll(td);
                td &= td - 1;
                if (n_open < Br) {
#pragma unroll
                    for (int x = 0; x < CPL; ++x) {
                        Krs[n_open * RS + CPL * lane + x] = to_float(Kst[i * D + CPL * lane + x]);
                        Vrs[n_open * RS + CPL * lane + x] = to_float(Vst[i * D + CPL * lane + x]);
                    }
                    if (lane == 0) {
                        wcs[n_open] = 1;
                        pos[n_open] = p0 + i;
                        s[n_open] = sc[p0 + i];
                    }
                    ++n_open;
                    wave_sync();
                    continue;
                }
                const int r = exact_choice(i);
                const int wi = wcs[r];
                wave_sync();   // every lane has read the count
                merge_into(i, r, wi, 1.0 / ((double)wi + 1.0));
                wave_sync();
            }
            if (n_open == Br) {
                // from the next block on: counts and reciprocals of this lane's columns, and the norm bound
                fast = true;
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) {
                    const int r = 16 * cb + ti;
                    st.wreg[cb] = r < Br ? wcs[r] : 1;
                    double n2 = 0.0;
                    const float* kr = Krs + (size_t)(r < Br ? r : Br - 1) * RS;
                    for (int c = 0; c < D; ++c) { const double x = (double)kr[c]; n2 = fma(x, x, n2); }
                    st.knorm[cb] = sqrt(n2) * (1.0 + 1e-12);
                }
            }
            continue;
        }

        // ---- whole block: all dot products and the Gram matrix on the matrix cores ----------
        {
            d4_t acc[NCB], gacc = d4_t{0.0, 0.0, 0.0, 0.0};
            const float* kb[NCB];
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                acc[cb] = d4_t{0.0, 0.0, 0.0, 0.0};
                const int r = 16 * cb + ti;
                kb[cb] = Krs + (size_t)(r < Br ? r : Br - 1) * RS + SPK * tk;   // a column past B_r repeats the last key; it is masked below
            }
#pragma unroll
            for (int s4 = 0; s4 < SPK; s4 += 4) {
                float4 kv[NCB];
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) kv[cb] = *reinterpret_cast<const float4*>(kb[cb] + s4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
#pragma unroll
                    for (int cb = 0; cb < NCB; ++cb) {
                        const float kf = e == 0 ? kv[cb].x : (e == 1 ? kv[cb].y : (e == 2 ? kv[cb].z : kv[cb].w));
                        acc[cb] = __builtin_amdgcn_mfma_f64_16x16x4f64(xd[s4 + e], (double)kf, acc[cb], 0, 0, 0);
                    }
                    gacc = __builtin_amdgcn_mfma_f64_16x16x4f64(xd[s4 + e], xd[s4 + e], gacc, 0, 0, 0);
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                st.gram[r] = gacc[r];
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) st.dv[cb][r] = acc[cb][r];
            }
        }
        // token norms (the Gram diagonal: token t against itself sits in lane 16 * (t % 4) + t, register t / 4) and the largest one
        double xmax = 0.0;
        {
            double n2 = 0.0;
#pragma unroll
            for (int r = 0; r < 4; ++r) n2 = (ti == 4 * r + tk) ? st.gram[r] : n2;   // x_t . x_t of token t = l%16, where it exists
            st.xnorm = sqrt(n2) * (1.0 + 1e-12);
            n2 = row_max(st.xnorm);
            xmax = max_d(max_d(readlane_d(n2, 0), readlane_d(n2, 16)), max_d(readlane_d(n2, 32), readlane_d(n2, 48)));
        }
        // 2^-24 |k'| |x| for the rounding of a merged key to fp32, doubled for the fp64 arithmetic around it
        const double err_unit = 1.1920928955078125e-07 * xmax;
        double emax = 0.0;    // largest error of a column so far in this block (wave-uniform)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) st.cerr[cb] = 0.0;

        // token I of the block (compile-time: it selects registers and lane patterns)
        auto token_step = [&](auto Ic) {
            constexpr int I = decltype(Ic)::value;
            constexpr int R = I / 4, RG = I % 4;
            if (!((todo >> I) & 1ull)) return;
            // this lane's best and second best over its columns (keys 16cb + l%16), then over the 16 lanes of the row
            const OrdKey none{(int)0x80000000, 0u};           // below every value
            OrdKey m1 = none, m2 = none;
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                const int idx = 16 * cb + ti;
                OrdKey v = ord_key(st.dv[cb][R], idx);
                if (idx >= Br) v = none;
                const bool up = ord_less(m1, v);
                const OrdKey lo = up ? m1 : v;                 // the smaller of the two
                m1 = up ? v : m1;
                m2 = ord_less(m2, lo) ? lo : m2;
            }
            const OrdKey w1 = row_max_key(m1);
            const bool mine = m1.hi == w1.hi && m1.lo == w1.lo;   // keys are distinct: equality names the winner's lane
            const OrdKey w2 = row_max_key(mine ? m2 : m1);
            const int h1 = __builtin_amdgcn_readlane(w1.hi, 16 * RG), h2 = __builtin_amdgcn_readlane(w2.hi, 16 * RG);
            const uint32_t l1 = (uint32_t)__builtin_amdgcn_readlane((int)w1.lo, 16 * RG), l2 = (uint32_t)__builtin_amdgcn_readlane((int)w2.lo, 16 * RG);
            const double d1 = ord_value(h1, l1), d2 = ord_value(h2, l2);
            int rbest = 63 - (int)(l1 & 63u);
            // every value is within emax of what the stored keys give, and the tag bits move it by less than 2^-46 of itself
            if (!(d1 - d2 > 2.0 * emax + 3e-14 * (fabs(d1) + fabs(d2)))) rbest = exact_choice(I);
            const int cbs = rbest >> 4, col = rbest & 15;
            const bool is_col = ti == col;
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                if (cb != cbs) continue;      // wave-uniform
                const int wi = __builtin_amdgcn_readlane(st.wreg[cb], col);   // the key's count, from a lane that owns the column
                const double wd = (double)wi, dd = wd + 1.0;
                // Eq. 6: the rows are requested first, the arithmetic that does not need them runs meanwhile
                float kc[CPL], vc[CPL], ko[CPL], vo[CPL];
#pragma unroll
                for (int x = 0; x < CPL; ++x) {
                    kc[x] = to_float(Kst[I * D + CPL * lane + x]);
                    vc[x] = to_float(Vst[I * D + CPL * lane + x]);
                    ko[x] = Krs[rbest * RS + CPL * lane + x];
                    vo[x] = Vrs[rbest * RS + CPL * lane + x];
                }
                const double ri = 1.0 / dd;                   // correctly rounded
                // the column's dot products with the block's later tokens: (w d + x_I . x_j) / (w + 1)
#pragma unroll
                for (int r = R; r < 4; ++r) {
                    const double gb = dpp_mov_d<0x150 + I>(st.gram[r]);   // row broadcast of lane I: x_(4r + l/16) . x_I
                    const double nd = fma(wd, st.dv[cb][r], gb) * ri;
                    st.dv[cb][r] = is_col ? nd : st.dv[cb][r];
                }
                // the merged key's norm bound, and what the skipped re-evaluation of its column may now be off by
                const double xn = readlane_d(st.xnorm, 16 * RG + I);
                const double kn = fma(wd, st.knorm[cb], xn) * ri * (1.0 + 2.4e-7);
                const double ce = st.cerr[cb] + err_unit * kn;
                st.knorm[cb] = is_col ? kn : st.knorm[cb];
                st.cerr[cb] = is_col ? ce : st.cerr[cb];
                st.wreg[cb] = is_col ? wi + 1 : st.wreg[cb];
                emax = max_d(emax, readlane_d(st.cerr[cb], col));
#pragma unroll
                for (int x = 0; x < CPL; ++x) {
                    const int c = CPL * lane + x;
                    const double nk = fma(wd, (double)ko[x], (double)kc[x]);   // w * k is exact in fp64: this is the rounded sum
                    const double nv = fma(wd, (double)vo[x], (double)vc[x]);
                    double qk = nk * ri, qv = nv * ri;
                    qk = fma(fma(-qk, dd, nk), ri, qk);    // the correctly rounded quotient nk / dd
                    qv = fma(fma(-qv, dd, nv), ri, qv);
                    Krs[rbest * RS + c] = (float)qk;
                    Vrs[rbest * RS + c] = (float)qv;
                }
                if (lane == 0) wcs[rbest] = wi + 1;
            }
        };
        token_step(std::integral_constant<int, 0>{});  token_step(std::integral_constant<int, 1>{});
        token_step(std::integral_constant<int, 2>{});  token_step(std::integral_constant<int, 3>{});
        token_step(std::integral_constant<int, 4>{});  token_step(std::integral_constant<int, 5>{});
        token_step(std::integral_constant<int, 6>{});  token_step(std::integral_constant<int, 7>{});
        token_step(std::integral_constant<int, 8>{});  token_step(std::integral_constant<int, 9>{});
        token_step(std::integral_constant<int, 10>{}); token_step(std::integral_constant<int, 11>{});
        token_step(std::integral_constant<int, 12>{}); token_step(std::integral_constant<int, 13>{});
        token_step(std::integral_constant<int, 14>{}); token_step(std::integral_constant<int, 15>{});
    }
    wave_sync();
    // write the residual slots back; slots never opened are empty
    for (int i = lane; i < Br * D; i += 64) {
        const int r = i / D, c = i % D;
        Kr[i] = Krs[r * RS + c];
        Vr[i] = Vrs[r * RS + c];
    }
    if (lane < Br) {
        const int wcnt = wcs[lane];
        w[lane] = wcnt;
        if (wcnt == 0) { pos[lane] = -1; s[lane] = 0.f; }
    }
}

template <typename T, int D>
hipError_t launch_prefill_td(const PrefillArgs& a, hipStream_t st) {
    const CacheView& cv = a.cv;
    const PrefillWs ws = prefill_ws_layout(cv, a.n_units, a.T_max, a.W);
    const size_t n_heads = (size_t)a.n_units * cv.G;
    hipLaunchKernelGGL((pf_convert_q<T>), dim3(1024), dim3(256), 0, st, reinterpret_cast<const T*>(a.Q),
                       reinterpret_cast<double*>(a.ws + ws.Qd), a.W, ws.Wp, D, n_heads);
    const dim3 gs(ws.fold ? (ws.nsums + 1) / 2 : ws.nsums, a.n_units, ws.rz);
    hipLaunchKernelGGL((pf_self_logit<T, D>), dim3(cv.G * ws.Wp, a.n_units), dim3(64), 0, st, a, ws);
    const double* Qd = reinterpret_cast<const double*>(a.ws + ws.Qd);
    const double* rowm = reinterpret_cast<const double*>(a.ws + ws.rowm);
    const double* roww = reinterpret_cast<const double*>(a.ws + ws.roww);
    double* pl = reinterpret_cast<double*>(a.ws + ws.pl);
    double* sacc = reinterpret_cast<double*>(a.ws + ws.sacc);
    float* sc = reinterpret_cast<float*>(a.ws + ws.sc);
    double* evs = reinterpret_cast<double*>(a.ws + ws.ev);
    if (ws.store_e) {
        const int tb16 = (a.T_max + 63) / 64;
        for (int u0 = 0; u0 < a.n_units; u0 += ws.ev_units) {   // batches of units whose exponentials fit the workspace
            const int nu = a.n_units - u0 < ws.ev_units ? a.n_units - u0 : ws.ev_units;
            PrefillWs wb = ws;
            wb.lu0 = u0;
            hipLaunchKernelGGL((pf_score_mfma<T, D, 2>), dim3(gs.x, nu, gs.z), dim3(256), 0, st, a, wb, Qd, rowm, roww, pl, sacc, sc, evs);
            hipLaunchKernelGGL(pf_row_combine, dim3(nu), dim3(256), 0, st, a, wb);
            hipLaunchKernelGGL(pf_score_from_ev, dim3(tb16 < 2048 ? tb16 : 2048, nu), dim3(256), 0, st, a, wb, roww, evs, sc);
        }
    } else {
        hipLaunchKernelGGL((pf_score_mfma<T, D, 0>), gs, dim3(256), 0, st, a, ws, Qd, rowm, roww, pl, sacc, sc, evs);
        hipLaunchKernelGGL(pf_row_combine, dim3(a.n_units), dim3(256), 0, st, a, ws);
        if (ws.multi) hipLaunchKernelGGL(pf_fill_f64, dim3(1024), dim3(256), 0, st, sacc, (size_t)ws.rz * a.n_units * a.T_max, 0.0);
        hipLaunchKernelGGL((pf_score_mfma<T, D, 1>), gs, dim3(256), 0, st, a, ws, Qd, rowm, roww, pl, sacc, sc, evs);
        if (ws.multi) hipLaunchKernelGGL(pf_sacc_to_sc, dim3((a.T_max + 255) / 256, a.n_units), dim3(256), 0, st, a, sacc, ws.rz, sc);
    }
    if (a.T_max <= SEL_NT * SEL_NPT) hipLaunchKernelGGL(pf_select_reg, dim3(a.n_units), dim3(SEL_NT), 0, st, a, ws);
    else hipLaunchKernelGGL(pf_select, dim3(a.n_units), dim3(SEL_NT), 0, st, a, ws);
    constexpr int EPL = 16 / sizeof(T), LPR = D / EPL, RPB = 256 / LPR;
    const int gblocks = (cv.cap_tok + RPB * 4 - 1) / (RPB * 4);
    hipLaunchKernelGGL((pf_gather<T, D>), dim3(gblocks > 0 ? gblocks : 1, a.n_units), dim3(256), 0, st, a, ws);
    if (cv.Br == 1) {
        // a single residual slot is the plain mean of everything absorbed: parallel sums
        hipLaunchKernelGGL((pf_residual_partial<T, D>), dim3(ws.nchunks, a.n_units), dim3(256), 0, st, a, ws);
        hipLaunchKernelGGL((pf_residual_final<D>), dim3(a.n_units), dim3(256), 0, st, a, ws);
    } else if (cv.Br > 1) {
        const size_t lds = pf_residual_blocks_lds<T, D>(cv.Br);
        const int wpg = 4 * lds <= 160 * 1024 ? 4 : (2 * lds <= 160 * 1024 ? 2 : 1);   // units per workgroup
        // column blocks of 16 residual keys
        void (*kern)(PrefillArgs, PrefillWs, int) = cv.Br > 48 ? pf_residual_blocks<T, D, 4>
                                                    : (cv.Br > 32 ? pf_residual_blocks<T, D, 3>
                                                       : (cv.Br > 16 ? pf_residual_blocks<T, D, 2> : pf_residual_blocks<T, D, 1>));
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3((a.n_units + wpg - 1) / wpg), dim3(64 * wpg), wpg * lds, st, a, ws, (int)lds);
    }
    return hipGetLastError();
}

template <typename T>
hipError_t launch_prefill_t(const PrefillArgs& a, hipStream_t st) {
    if (a.cv.D == 64) return launch_prefill_td<T, 64>(a, st);
    if (a.cv.D == 128) return launch_prefill_td<T, 128>(a, st);
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_prefill(const PrefillArgs& a, hipStream_t stream) {
    switch (a.cv.dtype) {
        case 0: return launch_prefill_t<float>(a, stream);
        case 1: return launch_prefill_t<f16_t>(a, stream);
        default: return launch_prefill_t<bf16_t>(a, stream);
    }
}

}  // namespace zsm
