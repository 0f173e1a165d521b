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
// Launch shapes: one workgroup per unit (4 waves; 8, 12 or 16 where the per-slot values of one workgroup fill a
// compute unit's LDS); several workgroups per unit plus decode_combine_kernel for launches of few units (SPLIT);
// for more than eight query heads per KV head, one workgroup per unit and share of eight or four heads plus
// decode_pool_finish_kernel (POOL).  Group sizes are compiled for 1, 2, 4 and 8 query heads; 3 and 5..7 run the
// next one with the surplus heads masked.
//
// Precision.  Everything that feeds a stored score or a decision (logits, exp, L, Eq. 5's
// dot products, Eq. 6's mean) is evaluated in fp64 and rounded once to the fp32 storage
// type; products of two fp16/bf16/fp32 values are exact in fp64, so the logits are the
// exactly rounded dot products and the eviction choice does not depend on the summation
// order of this kernel.  The attention output uses fp32 probabilities and accumulators.
// With fp64 exponentials no running maximum is needed: exp(z - C) cannot overflow unless a
// logit exceeds the incoming token's by more than LOGIT_SPREAD_MAX (690); there the difference
// is clamped (the slots beyond it tie).  A softmax denominator that reaches SPREAD_FLAG_SUM
// (e^680: one logit 680 above the reference, or many a little lower) raises the unit's
// FLAG_DECODE_SPREAD bit, so the clamp never acts unseen.
#pragma once

#include <atomic>
#include <type_traits>

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
    int32_t parts;      // workgroups per unit (1: the whole unit in one workgroup)
    int32_t part_rows;  // parts > 1: token rows the LDS of one part holds (a whole number of wave tiles)
    // Groups of more than eight query heads (decode_kernel's POOL): the unit's q_heads query heads are dealt to
    // n_shares workgroups, G (the kernel's compiled group size) each
    double* pool;       // [n_units][n_shares][cap + 1]: per share and slot (the incoming token last), the sum over the share's heads of e / L
    int32_t q_heads, n_shares;
};

template <typename T, int D, int G, int NW>
struct DecodeShape {
    static constexpr int EPL = 16 / sizeof(T);   // elements per lane (one 16-byte load)
    static constexpr int LPR = D / EPL;          // lanes per row
    static constexpr int RPL = 64 / LPR;         // rows per wave-wide load
    static constexpr int UT = 4;                 // wave-wide loads per tile (two tiles are in flight)
    static constexpr int UH = 4;                 // loads per reduction granule
    static constexpr int R = UT * RPL;           // rows per wave tile
    static constexpr int RU = 2;                 // wave-wide loads of residual rows a wave requests together
    static constexpr int NT = NW * 64;
    // pass 1 of full tiles on the 4x4x4 fp64 matrix instruction: four query heads, 16 keys of 16 pieces each per tile
    static constexpr bool MFMA4 = (G == 4 || G == 8) && sizeof(T) == 2 && D == 128;   // G / 4 groups of four heads
    // doubles of partial-dot staging per wave (the matrix path stages only its masked tiles: at most RU loads)
    static constexpr int PART = (MFMA4 ? RU : UH) * RPL * (LPR + 1);
    // queries live in LDS instead of registers (G * EPL doubles per lane); the matrix path keeps its own
    // operand registers and leaves the LDS copy, in fp32 (exact: the queries have the cache's element
    // type), to the masked tiles
    static constexpr bool QLDS = G > 4 || MFMA4;
    using QE = typename std::conditional<MFMA4, float, double>::type;
    static constexpr size_t QBYTES = QLDS ? sizeof(QE) * G * D : 0;
    // one LDS region serves the partial-dot staging and the queries of pass 1 and, after pass 2, the
    // waves' partial outputs
    // Normally every wave has a slot of its own there (out_slots = NW).  With eight query heads that is 16 KB, twice
    // what pass 1 needs, and at B = 1024 what keeps a second workgroup out of a compute unit's LDS: such a launch
    // runs with two slots, the waves handing their outputs over two at a time (NW / 2 rounds, a barrier each).
    static constexpr size_t STAGE_A = sizeof(double) * NW * PART;
    __host__ __device__ static constexpr size_t stage_bytes(int out_slots) {
        return STAGE_A + QBYTES > sizeof(float) * out_slots * G * D ? STAGE_A + QBYTES : sizeof(float) * out_slots * G * D;
    }
    static_assert(LPR >= 1 && LPR <= 64 && 64 % LPR == 0, "row must split over a wave");

    // dynamic LDS bytes when `nz` slots (the incoming token counted) keep their exp(logit - C) in LDS
    __host__ __device__ static size_t lds_bytes(int nz, int out_slots = NW) {
        size_t n = 0;
        n += sizeof(double) * G * (size_t)nz;          // et
        n += stage_bytes(out_slots);                   // part and queries (pass 1) / accw (after pass 2)
        n += sizeof(double) * NW * G;                  // red64
        n += sizeof(unsigned long long) * NW;          // keyw
        n += sizeof(double) * NW;                      // dotw
        n += sizeof(int) * (4 + NW);                   // misc
        return (n + 15) & ~(size_t)15;
    }
};

// The G query vectors, fp64: this lane's segment in registers, or all of them in LDS.
template <int G, int EPL, bool QLDS, typename QE = double>
struct Query {
    double r[QLDS ? 1 : G][EPL];
    const QE* lds;    // [G][D] when QLDS
    __device__ __forceinline__ void get(int g, int seg, int D, double* out) const {
        if (QLDS) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) out[e] = (double)lds[g * D + seg * EPL + e];
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
        for (int u = 0; u < UU; ++u) dst[u].load_nt(p + (size_t)u * RPL * D);
    } else {
#pragma unroll
        for (int u = 0; u < UU; ++u) {
            const int r = row0 + u * RPL + grp;
            dst[u].load_nt(base + (size_t)(r < nrows ? r : nrows - 1) * D + seg * EPL);
        }
    }
}

// Pass 1 on UU loaded wave-wide loads of K rows [row0, row0 + UU*RPL); rows >= nrows do not
// exist.  For every existing row the holder lane stores exp(logit - C) (0 for an empty row) at
// et[g][zidx0 + row] and adds it to lsum[g].  posb / wb (MASKED only) mark empty rows (pos < 0, w == 0); wb also adds
// alpha*log(w) to the logit (Eq. 4).
template <typename KT, int UU, bool MASKED, int D, int G, int EPL, int LPR, int RPL, bool QLDS, typename QQ>
__device__ __forceinline__ void k_compute(const Raw<KT, EPL>* kr, int row0, int nrows, int zidx0,
                                          const int32_t* __restrict__ posb, const int32_t* __restrict__ wb,
                                          double alpha, double scale, const QQ& qq,
                                          const double* C, double* lsum, double* et, int Bz,
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
                    ev = exp(fmin(z - C[g], LOGIT_SPREAD_MAX));
                    lsum[g] += ev;
                }
                et[(size_t)g * Bz + zidx0 + hr] = ev;
            }
            wave_sync();
        }
    }
}

// ---- pass 1 for grouped queries (G >= 2), full tiles only --------------------------------
// With G query heads a lane holds 4*G partial dot products per tile (4 rows x G heads), and the
// LPR lanes of a row group have to add theirs up.  Instead of staging them in LDS head by head
// (G rounds of writes, reads by a quarter of the lanes, and an exp at a quarter of the lanes),
// the lanes of the group exchange halves: at every step a lane keeps one half of its values,
// sends the other half to the lane whose number differs in one bit, and adds what it receives.
// After log2(LPR) steps every (row, head) sum sits in exactly one lane (or in LPR/(4G) lanes when
// there are fewer sums than lanes), so one exp per lane serves all heads at full width.
constexpr int ilog2_c(int x) { return x <= 1 ? 0 : 1 + ilog2_c(x / 2); }

// Lane numbering of that pass.  The two steps that move the most values should cross lane bits
// 5 and 4, where the exchange is a register swap between the wave's halves or between
// neighbouring 16-lane rows, so the two top bits of a lane's segment number come from lane bits
// 5 and 4, the other segment bits from the lowest lane bits, and the row group from the bits in
// between.  A wave-wide load still covers the same RPL whole rows, whatever lane reads which piece.
template <int LPR>
struct GqLane {
    static constexpr int LB = ilog2_c(LPR), LOW = LB - 2;
    static_assert(LB >= 2 && LB <= 5, "");
    __device__ static int seg(int lane) { return (((lane >> 4) & 3) << LOW) | (lane & ((1 << LOW) - 1)); }
    __device__ static int grp(int lane) { return (lane >> LOW) & (64 / LPR - 1); }
    // the number tile_load() takes: row group * LPR + segment
    __device__ static int as_row_major(int lane) { return grp(lane) * LPR + seg(lane); }
    // sum over the LPR lanes of a row group, left in all of them
    __device__ static double group_sum(double p) {
#pragma unroll
        for (int o = 1; o < (1 << LOW); o <<= 1) p += __shfl_xor(p, o, 64);
        p += __shfl_xor(p, 16, 64);
        p += __shfl_xor(p, 32, 64);
        return p;
    }
};

// a (kept by the lower lane of a pair, sent by the upper) and b (the reverse) -> own + received,
// the pair being lanes l and l ^ 32 (FAR) or l and l ^ 16
template <bool FAR>
__device__ __forceinline__ double swap_add(double a, double b) {
    const uint32_t al = (uint32_t)__double2loint(a), ah = (uint32_t)__double2hiint(a);
    const uint32_t bl = (uint32_t)__double2loint(b), bh = (uint32_t)__double2hiint(b);
    if constexpr (FAR) {
        const auto lo = __builtin_amdgcn_permlane32_swap(al, bl, false, false);
        const auto hi = __builtin_amdgcn_permlane32_swap(ah, bh, false, false);
        return __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
    } else {
        const auto lo = __builtin_amdgcn_permlane16_swap(al, bl, false, false);
        const auto hi = __builtin_amdgcn_permlane16_swap(ah, bh, false, false);
        return __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
    }
}

// DD: the segment bit of this step (LPR / 2 first); NV values per lane before it.
template <int NV, int DD, int LPR>
__device__ __forceinline__ void lane_group_reduce(double* pp, int seg) {
    if constexpr (DD >= 1) {
        constexpr int DIST = DD == LPR / 2 ? 32 : (DD == LPR / 4 ? 16 : DD);   // lane distance of the pair
        if constexpr (NV > 1) {
            constexpr int H = NV / 2;
            if constexpr (DIST >= 16) {
#pragma unroll
                for (int i = 0; i < H; ++i) pp[i] = swap_add<DIST == 32>(pp[i], pp[i + H]);
            } else {
                const bool hi = (seg & DD) != 0;
#pragma unroll
                for (int i = 0; i < H; ++i) {
                    const double keep = hi ? pp[i + H] : pp[i];
                    const double send = hi ? pp[i] : pp[i + H];
                    pp[i] = keep + __shfl_xor(send, DIST, 64);
                }
            }
            lane_group_reduce<H, DD / 2, LPR>(pp, seg);
        } else {
            pp[0] += __shfl_xor(pp[0], DIST, 64);
            lane_group_reduce<1, DD / 2, LPR>(pp, seg);
        }
    }
}

// Which sums a lane ends up with: values are numbered v = g*4 + u (head g, wave-wide load u).
template <int G, int LPR>
struct GqOwn {
    static constexpr int UH = 4, V = UH * G;
    static constexpr int NVF = V >= LPR ? V / LPR : 1;        // sums per lane at the end
    static constexpr int REP = V >= LPR ? 1 : LPR / V;        // lanes that hold the same sum
    static constexpr int K = ilog2_c(V / NVF), LB = ilog2_c(LPR);
    static_assert(NVF <= UH, "a lane's sums must belong to one head");
    __device__ static int first_value(int seg) { return (seg >> (LB - K)) * NVF; }
    __device__ static int head(int seg) { return first_value(seg) / UH; }
    __device__ static bool writes(int seg) { return (seg & (REP - 1)) == 0; }
};

// One full tile (4 wave-wide loads, every row occupied): exp(logit - C) of this lane's (row, head)
// sums into et, their total into lsum_own.  c_own = C[GqOwn::head(seg)].
template <typename KT, int D, int G, int EPL, int LPR, int RPL, bool QLDS, typename QQ>
__device__ __forceinline__ void k_compute_gq(const Raw<KT, EPL>* kr, int row0, int nrows, int zidx0, double scale,
                                             const QQ& qq, double c_own, double& lsum_own,
                                             double* et, int Bz, int lane) {
    using Own = GqOwn<G, LPR>;
    constexpr int UH = Own::UH;
    const int grp = GqLane<LPR>::grp(lane), seg = GqLane<LPR>::seg(lane);   // kr was loaded in this numbering
    double pp[Own::V];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        double qv[EPL];
        qq.get(g, seg, D, qv);
#pragma unroll
        for (int u = 0; u < UH; ++u) {
            double p = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) p = fma(qv[e], (double)kr[u].get(e), p);
            pp[g * UH + u] = p;
        }
    }
    lane_group_reduce<Own::V, LPR / 2, LPR>(pp, seg);
    const int v0 = Own::first_value(seg);
    const int g_own = v0 / UH;
    if (Own::writes(seg)) {
#pragma unroll
        for (int i = 0; i < Own::NVF; ++i) {
            const int row = row0 + ((v0 + i) % UH) * RPL + grp;
            if (row < nrows) {
                const double ev = exp(fmin(pp[i] * scale - c_own, LOGIT_SPREAD_MAX));
                lsum_own += ev;
                et[(size_t)g_own * Bz + zidx0 + row] = ev;
            }
        }
    }
}

// ---- pass 1 for four grouped query heads on the matrix cores (16-bit K, d = 128, full tiles) ----
// v_mfma_f64_4x4x4 multiplies, in each of four blocks, a 4x4 A by a 4x4 B.  Lane l supplies
// A[i = l % 4][k = l / 16] and B[k = l / 16][j = l % 4] of block (l / 4) % 4 and receives
// D[i = l / 16][j = l % 4] of that block (checked on the device with one-hot operands).  With
// i = query head, block and j = key (key l % 16 of the tile's 16) and k = one of four 16-byte
// pieces of the row, lane l loads pieces l/16, 4 + l/16, 8 + l/16, 12 + l/16 of key row l % 16
// (one per wave-wide load) and holds head l % 4's query values of the same pieces; the 32 steps
// (4 loads x 8 elements) contract all 128 channels, and lane l ends up with the exact-product
// fp64 logit of (head l / 16, key l % 16): no exchange between lanes, one exp per lane.
template <typename KT, int UU, int D, int EPL>
__device__ __forceinline__ void tile_load_mfma4(Raw<KT, EPL>* dst, const KT* __restrict__ base, int row0, int nrows, int lane) {
    const int r = row0 + (lane & 15);
    const KT* p = base + ((size_t)(r < nrows ? r : nrows - 1) * D + (lane >> 4) * EPL);
#pragma unroll
    for (int u = 0; u < UU; ++u) dst[u].load(p + u * 4 * EPL);
}

// NG groups of four heads (G = 4 * NG): group h uses qa[h] and gives lane l head 4h + l / 16.
template <typename KT, int UU, int EPL, int NG>
__device__ __forceinline__ void k_compute_mfma4(const Raw<KT, EPL>* kr, const double (*qa)[UU][EPL], int row0, int nrows,
                                                int zidx0, double scale, const double* c_own, double* lsum_own,
                                                double* et_own, int Bz, int lane) {
    double d0[NG], d1[NG];   // two accumulators per group: consecutive steps do not wait for each other
#pragma unroll
    for (int h = 0; h < NG; ++h) d0[h] = d1[h] = 0.0;
#pragma unroll
    for (int u = 0; u < UU; ++u) {
#pragma unroll
        for (int e = 0; e < EPL; e += 2) {
            const double b0 = (double)kr[u].get(e), b1 = (double)kr[u].get(e + 1);
#pragma unroll
            for (int h = 0; h < NG; ++h) {
                d0[h] = __builtin_amdgcn_mfma_f64_4x4x4f64(qa[h][u][e], b0, d0[h], 0, 0, 0);
                d1[h] = __builtin_amdgcn_mfma_f64_4x4x4f64(qa[h][u][e + 1], b1, d1[h], 0, 0, 0);
            }
        }
    }
    const int row = row0 + (lane & 15);
    if (row < nrows) {
#pragma unroll
        for (int h = 0; h < NG; ++h) {
            const double ev = exp(fmin((d0[h] + d1[h]) * scale - c_own[h], LOGIT_SPREAD_MAX));
            lsum_own[h] += ev;
            et_own[(size_t)4 * h * Bz + zidx0 + row] = ev;   // et_own = et + (lane / 16) * Bz
        }
    }
}

// Pass 1 for rows that may be empty: load only the occupied ones (an empty slot may hold any
// bit pattern), then k_compute.  LOADALL requests every row without waiting for its occupancy
// (one memory round trip instead of two); what an empty row yields is never used: k_compute
// stores 0 for it.
template <typename KT, int UU, int D, int G, int EPL, int LPR, int RPL, bool QLDS, bool LOADALL = false, typename QQ>
__device__ __forceinline__ void k_tile_masked(const KT* __restrict__ Kb, int row0, int nrows, int zidx0,
                                              const int32_t* __restrict__ posb, const int32_t* __restrict__ wb,
                                              double alpha, double scale, const QQ& qq,
                                              const double* C, double* lsum, double* et, int Bz,
                                              double* part_w, int lane) {
    const int grp = lane / LPR, seg = lane % LPR;
    Raw<KT, EPL> kr[UU];
    if constexpr (LOADALL) {
        tile_load<KT, UU, D, EPL, LPR, RPL>(kr, Kb, row0, nrows, lane);
    } else {
#pragma unroll
        for (int u = 0; u < UU; ++u) {
            const int r = row0 + u * RPL + grp;
            if (r < nrows && (posb == nullptr || posb[r] >= 0) && (wb == nullptr || wb[r] > 0))
                kr[u].load(Kb + (size_t)r * D + seg * EPL);
            else
                kr[u].zero();
        }
    }
    k_compute<KT, UU, true, D, G, EPL, LPR, RPL, QLDS>(kr, row0, nrows, zidx0, posb, wb, alpha, scale, qq, C, lsum, et,
                                                       Bz, part_w, lane);
}

// Pass 2 on UU loaded wave-wide loads of V rows: acc[g] += p * v with p = et * rL (fp32).
template <typename KT, int UU, int D, int G, int EPL, int LPR, int RPL>
__device__ __forceinline__ void v_compute(const Raw<KT, EPL>* vr, int row0, int nrows, int zidx0,
                                          const double* rL, float (*acc)[EPL], const double* et, int Bz,
                                          int lane) {
    const int grp = lane / LPR;
    if (row0 + UU * RPL <= nrows) {   // every row of the tile exists: no per-row test
#pragma unroll
        for (int u = 0; u < UU; ++u) {
            const int r = row0 + u * RPL + grp;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float p = (float)(et[(size_t)g * Bz + zidx0 + r] * rL[g]);
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, vr[u].get(e), acc[g][e]);
            }
        }
        return;
    }
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
    const int d4 = 4 * done;   // quarter of the way = floor(4 * done / total), by comparisons (both are wave-uniform)
    if (d4 >= 3 * total) __builtin_amdgcn_s_setprio(0);
    else if (d4 >= 2 * total) __builtin_amdgcn_s_setprio(1);
    else if (d4 >= total) __builtin_amdgcn_s_setprio(2);
    else __builtin_amdgcn_s_setprio(3);
}

// Query heads per KV head.  The kernels are compiled for G = 1, 2, 4, 8; a cache with another number Gr of query
// heads (3, 5, 6, 7) runs the next larger one: the heads past the last read the last head's query again, their
// 1/L is set to 0 (so they add nothing to Eq. 3's head mean) and their outputs are not written.
template <int G>
__device__ __forceinline__ int real_heads(const CacheView& cv) { return G == 1 ? 1 : cv.G; }

// mean over the Gr heads of a sum over them (appendix, grouped-query adaptation): the oracle's sum / Gr
template <int G>
__device__ __forceinline__ double head_mean(double sum, int Gr) {
    if constexpr (G == 1) return sum;
    return Gr == G ? sum / (double)G : sum / (double)Gr;   // a power of two: an exact multiplication
}

// Everything of a unit's cache that the end of a step touches.
template <typename T>
struct UnitRefs {
    T* Kt; T* Vt;              // token slots
    float* Kr; float* Vr;      // residual slots
    float* s; int32_t* pos; int32_t* w;
    const T* knew; const T* vnew;
};

constexpr int DECODE_MCH = 12;  // slots per thread whose score and position are requested ahead (3072 slots per workgroup)

// What the end of a step reads that does not depend on its decisions.  The caller requests it
// early (load()), so that the only memory round trip left between the eviction choice and the
// stores is the read of the evicted row.
template <typename T, int D, int NW, int GE = 0>
struct FinishPre {
    static constexpr int NT = NW * 64;
    int pj[DECODE_MCH];      // positions and scores of slots k*NT + tid
    float sj[DECODE_MCH];
    // GE = G: their exp(logit - C) too (values that live in global memory); of the first MCHE slots only where the
    // eight heads' values of all twelve would take 192 registers and leave one wave per SIMD
    static constexpr int MCHE = GE >= 8 ? DECODE_MCH / 2 : DECODE_MCH;
    double ej[GE > 0 ? MCHE : 1][GE > 0 ? GE : 1];
    int wres;                // fusion count of residual slot tid (tid < B_r), else 1
    T kn, vn;                // channel tid of the incoming token (tid < D)
    float kr0, vr0;          // B_r = 1: channel tid of the only residual slot
    int w0;                  // B_r = 1: its fusion count
    bool vec;                // slots are taken four at a time (16-byte loads and stores): the slot stride allows it
    // slot of this thread's k-th value, counted from the start of a batch of NT * DECODE_MCH slots
    __device__ __forceinline__ int slot_of(int k) const {
        const int tid = threadIdx.x;
        return vec ? (((k >> 2) * NT + tid) << 2) + (k & 3) : k * NT + tid;
    }
    // positions and scores of the batch that starts at slot `base`; slots >= lim read as empty.
    // Under load every memory instruction of a wave queues behind the other workgroups' sweeps,
    // so their number matters: four slots per instruction where the layout is 16-byte aligned.
    __device__ __forceinline__ void load_meta(const UnitRefs<T>& u, int base, int lim) {
        const int tid = threadIdx.x;
        if (vec) {
#pragma unroll
            for (int kk = 0; kk < DECODE_MCH / 4; ++kk) {
                const int j = base + ((kk * NT + tid) << 2);
                int4 p = make_int4(-1, -1, -1, -1);
                float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
                if (j < lim) {   // lim is a multiple of 4 here
                    p = *reinterpret_cast<const int4*>(u.pos + j);
                    x = *reinterpret_cast<const float4*>(u.s + j);
                }
                pj[4 * kk + 0] = p.x; pj[4 * kk + 1] = p.y; pj[4 * kk + 2] = p.z; pj[4 * kk + 3] = p.w;
                sj[4 * kk + 0] = x.x; sj[4 * kk + 1] = x.y; sj[4 * kk + 2] = x.z; sj[4 * kk + 3] = x.w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < DECODE_MCH; ++k) {
                const int j = base + k * NT + tid;
                pj[k] = j < lim ? u.pos[j] : -1;
                sj[k] = j < lim ? u.s[j] : 0.f;
            }
        }
    }
    __device__ __forceinline__ void load(const UnitRefs<T>& u, int cap, int Br, const double* et = nullptr, int Bz = 0) {
        const int tid = threadIdx.x;
        static_assert(DECODE_MCH % 4 == 0, "");
        vec = (cap & 3) == 0;   // every unit's score and position rows then start on a 16-byte boundary
        if (GE > 0) {
#pragma unroll
            for (int k = 0; k < (GE > 0 ? MCHE : 1); ++k) {
                const int j = slot_of(k);
#pragma unroll
                for (int g = 0; g < (GE > 0 ? GE : 1); ++g) ej[k][g] = j < cap ? et[(size_t)g * Bz + j] : 0.0;
            }
        }
        // slots between the unit's B and the slot stride are empty by construction (pos = -1)
        load_meta(u, 0, cap);
        wres = tid < Br ? u.w[tid] : 1;
        if (tid < D) { kn = u.knew[tid]; vn = u.vnew[tid]; }
        w0 = 1; kr0 = 0.f; vr0 = 0.f;
        if (Br == 1) {
            w0 = u.w[0];
            if (tid < D) { kr0 = u.Kr[tid]; vr0 = u.Vr[tid]; }
        }
    }
};

// D3-D6 of one unit, by the whole workgroup: score update (Eq. 3) from the per-slot
// exp(logit - C) values in `et` (stride Bz per query head; LDS or global) and 1/L in rL,
// eviction choice, residual absorption (Eq. 5, Eq. 6) and the write of the incoming token.
// misc[0] must hold -1 and misc[2] 0x7fffffff (set before a barrier the caller has passed).
template <typename T, int D, int G, int NW, int GE>
__device__ __forceinline__ void decode_finish(const DecodeArgs& a, const CacheView& cv, const UnitRefs<T>& u, int lu,
                                              int ug, int Bp, int Br, int B, long long Tseen, int nocc, bool full,
                                              const double* et, int Bz, const double* rL, FinishPre<T, D, NW, GE>& pre,
                                              unsigned long long* keyw, double* dotw, int* misc) {
    constexpr int NT = NW * 64, MCH = DECODE_MCH;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int Gr = real_heads<G>(cv);
    T* Kt = u.Kt; T* Vt = u.Vt;
    float* Kr = u.Kr; float* Vr = u.Vr;
    float* s = u.s; int32_t* pos = u.pos; int32_t* w = u.w;
    // the incoming token's own exp value (thread 0 needs it at the very end)
    double e_new[G];
    if (tid == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) e_new[g] = et[(size_t)g * Bz + B];
    }
    // lowest unused residual slot (they are opened in index order, Alg. 1) -> misc[2]
    if (full && Br > 0) {
        for (int r0 = 0; r0 < Br; r0 += NT) {
            const int wv = r0 == 0 ? pre.wres : (r0 + tid < Br ? w[r0 + tid] : 1);
            const unsigned long long m = __ballot(wv == 0);
            if (m != 0ull && lane == 0) atomicMin(&misc[2], r0 + wave * 64 + (int)__builtin_ctzll(m));
        }
    }
    // ---- D3: score update (Eq. 3) and D4: eviction choice ------------------------------
    const double lam = (double)cv.lambda;
    const long long cand_hi = Tseen - Bp;   // evictable: position <= T - B_p (outside the latest B_p)
    unsigned long long best = ~0ull;
    int best_slot = -1;
    for (int base = 0; base < B; base += NT * MCH) {
        if (base > 0) pre.load_meta(u, base, cv.cap);
#pragma unroll
        for (int kk = 0; kk < MCH / 4; ++kk) {
            float sn4[4];
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
                const int k = 4 * kk + c4;
                const int j = base + pre.slot_of(k);
                sn4[c4] = pre.sj[k];
                if (j >= B) continue;
                if (pre.pj[k] >= 0) {   // occupied (a residual slot carries the position of its first token)
                    double pm = 0.0;
#pragma unroll
                    for (int g = 0; g < G; ++g)
                        pm += ((GE > 0 && base == 0 && k < FinishPre<T, D, NW, GE>::MCHE) ? pre.ej[(GE > 0 && k < FinishPre<T, D, NW, GE>::MCHE) ? k : 0][GE > 0 ? g : 0]
                                                                                         : et[(size_t)g * Bz + j]) * rL[g];
                    pm = head_mean<G>(pm, Gr);
                    const float sn = (float)(lam * (double)pre.sj[k] + pm);
                    sn4[c4] = sn;
                    if (!pre.vec) s[j] = sn;
                    if (full && j >= Br && (long long)pre.pj[k] <= cand_hi) {
                        const unsigned long long key = ((unsigned long long)__float_as_uint(sn) << 32) | (uint32_t)pre.pj[k];
                        if (key < best) { best = key; best_slot = j; }
                    }
                } else if (!full && j >= Br) {
                    const unsigned long long key = (unsigned long long)j;   // lowest free token slot
                    if (key < best) { best = key; best_slot = j; }
                }
            }
            if (pre.vec) {   // four scores per store; a slot that was not updated gets back what was read
                const int j0 = base + pre.slot_of(4 * kk);
                if (j0 < B) *reinterpret_cast<float4*>(s + j0) = make_float4(sn4[0], sn4[1], sn4[2], sn4[3]);
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
    if (full && Br > 0) {
        const int r_empty = misc[2] < Br ? misc[2] : -1;
        float ke = 0.f, ve = 0.f;   // channel tid of the evicted token
        if (tid < D) {
            ke = to_float(Kt[(size_t)ct * D + tid]);
            ve = to_float(Vt[(size_t)ct * D + tid]);
        }
        if (r_empty >= 0) {
            if (tid < D) { Kr[r_empty * D + tid] = ke; Vr[r_empty * D + tid] = ve; }
            if (tid == 0) { w[r_empty] = 1; pos[r_empty] = ev_pos; s[r_empty] = ev_s; }
            merged = r_empty;
        } else {
            int br = 0, wv = pre.w0;
            float k0 = pre.kr0, v0 = pre.vr0;
            if (Br > 1) {
                // Eq. 5: the residual key with the largest dot product, lowest index on ties
                double bd = -INFINITY;
                br = 0x7fffffff;
                // A wave takes rows wave, wave + NW, ...; the rows of a batch are all requested
                // before the first is used, so a batch costs one memory round trip, not one per row.
                constexpr int CPL = (D + 63) / 64, RB = 8;
                float kt[CPL];
#pragma unroll
                for (int x = 0; x < CPL; ++x) {
                    const int ch = lane + 64 * x;
                    kt[x] = ch < D ? to_float(Kt[(size_t)ct * D + ch]) : 0.f;
                }
                for (int r0 = wave; r0 < Br; r0 += NW * RB) {
                    float kr[RB][CPL];
#pragma unroll
                    for (int y = 0; y < RB; ++y) {
                        const int r = r0 + y * NW < Br ? r0 + y * NW : Br - 1;
#pragma unroll
                        for (int x = 0; x < CPL; ++x) {
                            const int ch = lane + 64 * x;
                            kr[y][x] = ch < D ? Kr[r * D + ch] : 0.f;
                        }
                    }
#pragma unroll
                    for (int y = 0; y < RB; ++y) {
                        double p = 0.0;
#pragma unroll
                        for (int x = 0; x < CPL; ++x) p = fma((double)kr[y][x], (double)kt[x], p);
                        p = wave_sum(p);
                        if (r0 + y * NW < Br && p > bd) { bd = p; br = r0 + y * NW; }
                    }
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
                wv = w[br];
                if (tid < D) { k0 = Kr[br * D + tid]; v0 = Vr[br * D + tid]; }
                __syncthreads();   // every thread has read w[br] before thread 0 changes it
            }
            merged = br;
            if (tid < D) {
                const double wd = (double)wv;
                Kr[br * D + tid] = (float)((wd * (double)k0 + (double)ke) / (wd + 1.0));
                Vr[br * D + tid] = (float)((wd * (double)v0 + (double)ve) / (wd + 1.0));
            }
            if (tid == 0) w[br] = wv + 1;
        }
        __syncthreads();   // the evicted row has been read by everyone who needs it
    }

    // ---- D6: the incoming token takes the freed slot ----------------------------------
    if (tid < D) {
        Kt[(size_t)ct * D + tid] = pre.kn;
        Vt[(size_t)ct * D + tid] = pre.vn;
    }
    if (tid == 0) {
        double pm = 0.0;
#pragma unroll
        for (int g = 0; g < G; ++g) pm += e_new[g] * rL[g];
        pm = head_mean<G>(pm, Gr);
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

// Occupancy bound: 4 waves per SIMD for G = 1 (four workgroups per compute unit, LDS permitting).
// Grouped queries are bounded at 2 (up to 256 registers): their per-head state needs more than
// 128, and what they really use decides the residency (the matrix-core pass takes about 165, which
// gives three workgroups per compute unit; the LDS footprint of a large budget caps it further).
//
// SPLIT = false: one workgroup per unit does everything.
// SPLIT = true: a.parts workgroups per unit.  Part p sweeps a contiguous range of the token
//   slots' wave tiles (part 0 also takes the residual slots and the incoming token), normalises
//   by its own denominator L_p and leaves L_p, its output share and the exp(logit - C) of its
//   slots in the cache's scratch area; C is the same for every part, so no maxima are exchanged.
//   decode_combine_kernel, launched behind it, finishes every unit from there (the kernel
//   boundary is what makes one workgroup's scratch visible to another: fences inside one
//   kernel cost more here than the whole sweep of a small launch).
//
// AW: LDS slots for the waves' partial outputs after pass 2: one per wave, or fewer, the waves then handing
// their outputs over AW at a time.
// POOL: groups of more than eight query heads.  a.n_shares workgroups per unit, each with a share of G (eight, or
//   four where eight heads' per-slot values do not fit the LDS) of the unit's a.q_heads query heads.  A workgroup
//   writes its heads' outputs and leaves, per slot, the sum over its heads of e / L in its slice of a.pool; the
//   cache is not touched.  decode_pool_finish_kernel, launched behind it, adds the shares up in order, divides by
//   the number of heads (the head mean of Eq. 3's grouped-query form) and runs D3-D6.
template <typename T, int D, int G, int NW, bool SPLIT, int AW = NW, bool POOL = false>
__global__ __launch_bounds__(NW * 64, G == 1 ? 4 : (NW == 12 ? 3 : 2)) void decode_kernel(DecodeArgs a) {
    static_assert(!POOL || (!SPLIT && (G == 8 || G == 4)), "shares of a large group run the eight- or four-head kernel, one workgroup per unit");
    using Sh = DecodeShape<T, D, G, NW>;
    constexpr int EPL = Sh::EPL, LPR = Sh::LPR, RPL = Sh::RPL, R = Sh::R, PART = Sh::PART, NT = Sh::NT, UT = Sh::UT;
    constexpr bool QLDS = Sh::QLDS;
    const CacheView& cv = a.cv;
    // POOL: workgroup x of the grid is dispatched to XCD x % 8; the shares of one unit are given numbers that agree
    // modulo 8 and lie 8 apart, so that they run at about the same time on one XCD and meet in its L2 (the unit's K
    // and V come from memory once instead of once per share)
    const int pool_r = (int)blockIdx.x >> 3;
    const int share = POOL ? pool_r % a.n_shares : 0;
    const int Gr = POOL ? (a.q_heads - share * G < G ? a.q_heads - share * G : G) : real_heads<G>(cv);
    const int lu = SPLIT ? (int)blockIdx.x / a.parts : (POOL ? (pool_r / a.n_shares) * 8 + ((int)blockIdx.x & 7) : (int)blockIdx.x);
    if (POOL && lu >= a.n_units) return;   // the grid is rounded up to whole groups of eight units
    const int part = SPLIT ? (int)blockIdx.x % a.parts : 0;
    const int ug = a.unit0 + lu;
    const int b = (ug / cv.H) % cv.S;
    const int Bp = cv.Bp[b], Bc = cv.Bc[b], Br = cv.Br;
    const int ntok = Bp + Bc, B = ntok + Br;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: loop counters and tile numbers stay in scalar registers
    // Pass 1 of grouped queries numbers the lanes for its exchange (GqLane); every part of that pass
    // (queries in registers, masked tiles, the reference logit) uses the same numbering.  Pass 2 and
    // the output use the plain one.
    constexpr bool MF = Sh::MFMA4;
    const int klane = (G >= 2 && !MF) ? GqLane<LPR>::as_row_major(lane) : lane;
    const int grp = lane / LPR, seg = lane % LPR;
    const int kseg = klane % LPR;

    // this workgroup's wave tiles [tb, te) = token rows [row_b, row_e)
    const int ntiles = (ntok + R - 1) / R;
    int tb = 0, te = ntiles;
    if (SPLIT) {
        const int tpp = (ntiles + a.parts - 1) / a.parts;
        tb = part * tpp < ntiles ? part * tpp : ntiles;
        te = tb + tpp < ntiles ? tb + tpp : ntiles;
    }
    const int row_b = tb * R, row_e = te * R < ntok ? te * R : ntok;
    // LDS index of a slot's exp value: residual slot r -> r, token row x -> zt + x, incoming token -> znew
    const int Bz = SPLIT ? a.part_rows + Br + 1 : cv.cap + 1;
    const int zt = Br - row_b;
    const int znew = Br + (row_e - row_b);   // used where row_b = 0 and row_e = ntok (SPLIT: part 0 only, any row_e)

    extern __shared__ __align__(16) unsigned char smem[];
    double* et = reinterpret_cast<double*>(smem);                 // [G][Bz] exp(logit - C) per slot
    double* part_s = et + (size_t)G * Bz;                         // [NW][PART], pass 1 only
    using QE = typename Sh::QE;
    QE* qlds = reinterpret_cast<QE*>(part_s + NW * PART);         // [G][D] (QLDS only), pass 1 only
    float* accw = reinterpret_cast<float*>(part_s);               // [AW][G][D], after pass 2 (the memory of the two above)
    double* red64 = reinterpret_cast<double*>(reinterpret_cast<unsigned char*>(part_s) + Sh::stage_bytes(AW));   // [NW][G]
    unsigned long long* keyw = reinterpret_cast<unsigned long long*>(red64 + NW * G);   // [NW]
    double* dotw = reinterpret_cast<double*>(keyw + NW);          // [NW]
    int* misc = reinterpret_cast<int*>(dotw + NW);                // [4 + NW]

    T* Kt = reinterpret_cast<T*>(cv.Kt) + (size_t)ug * cv.cap_tok * D;
    T* Vt = reinterpret_cast<T*>(cv.Vt) + (size_t)ug * cv.cap_tok * D;
    float* Kr = cv.Kr + (size_t)ug * Br * D;
    float* Vr = cv.Vr + (size_t)ug * Br * D;
    float* s = cv.s + (size_t)ug * cv.cap;
    int32_t* pos = cv.pos + (size_t)ug * cv.cap;
    int32_t* w = cv.w + (size_t)ug * cv.cap;
    // The wave's first K tile is requested before anything else when its rows are known without
    // the budgets (one workgroup per unit: tile `wave`); rows past the unit's budget exist up to
    // the slot stride and are discarded by the compute step.
    Raw<T, EPL> bufA[UT], bufB[UT];
    if (!SPLIT) {
        if constexpr (MF) tile_load_mfma4<T, UT, D, EPL>(bufA, Kt, wave * R, cv.cap_tok, lane);
        else tile_load<T, UT, D, EPL, LPR, RPL>(bufA, Kt, wave * R, cv.cap_tok, klane);
    }
    const size_t head_off = POOL ? (size_t)lu * a.q_heads + share * G : (size_t)lu * Gr;   // this workgroup's first head in q and out
    const T* qp = reinterpret_cast<const T*>(a.q) + head_off * D;
    const T* knew = reinterpret_cast<const T*>(a.k_new) + (size_t)lu * D;
    const T* vnew = reinterpret_cast<const T*>(a.v_new) + (size_t)lu * D;
    const long long Tseen = cv.n_seen[ug];
    const int nocc = cv.n_occ[ug];
    const bool full = nocc == ntok;
    const double scale = cv.scale;
    const double alpha = (double)cv.alpha;

    if (tid == 0) { misc[0] = -1; misc[2] = 0x7fffffff; }
    Query<G, EPL, QLDS, QE> qq;
    qq.lds = qlds;
    if (QLDS) {
        for (int i = tid; i < G * D; i += NT) qlds[i] = (QE)to_float(qp[(i / D < Gr ? i / D : Gr - 1) * D + i % D]);
        __syncthreads();
    } else {
#pragma unroll
        for (int g = 0; g < (QLDS ? 1 : G); ++g) {
            float qf[EPL];
            load_seg<EPL>(qp + (g < Gr ? g : Gr - 1) * D + kseg * EPL, qf);
#pragma unroll
            for (int e = 0; e < EPL; ++e) qq.r[g][e] = (double)qf[e];
        }
    }
    // matrix path: head lane % 4's query values at the pieces this lane loads of a key row
    constexpr int NG = MF ? G / 4 : 1;
    double qa[NG][MF ? UT : 1][EPL];
    if constexpr (MF) {
#pragma unroll
        for (int h = 0; h < NG; ++h)
#pragma unroll
            for (int u = 0; u < UT; ++u) {
                float qf[EPL];
                const int hq = 4 * h + (lane & 3);
                load_seg<EPL>(qp + (hq < Gr ? hq : Gr - 1) * D + (4 * u + (lane >> 4)) * EPL, qf);
#pragma unroll
                for (int e = 0; e < EPL; ++e) qa[h][u][e] = (double)qf[e];
            }
    }
    // reference logit C[g]: the incoming token against itself (every lane of every wave)
    double C[G], lsum[G];
    {
        float kf[EPL];
        load_seg<EPL>(knew + kseg * EPL, kf);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            double qv[EPL];
            qq.get(g, kseg, D, qv);
            double p = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) p = fma(qv[e], (double)kf[e], p);
            if constexpr (G >= 2 && !MF) {
                p = GqLane<LPR>::group_sum(p);
            } else {
#pragma unroll
                for (int o = 1; o < LPR; o <<= 1) p += __shfl_xor(p, o, 64);
            }
            C[g] = p * scale;
            lsum[g] = 0.0;
        }
    }
    double* part_w = part_s + wave * PART;
    // grouped queries: the head whose sums this lane finishes in full tiles, its reference, its total
    // (matrix path: heads 4h + lane / 16, one per group of four heads)
    const int g_own = MF ? lane >> 4 : GqOwn<G, LPR>::head(GqLane<LPR>::seg(lane));
    double c_own = C[0], lsum_own = 0.0;
#pragma unroll
    for (int g = 1; g < G; ++g) c_own = g == g_own ? C[g] : c_own;
    double c_mf[NG], lsum_mf[NG];
#pragma unroll
    for (int h = 0; h < NG; ++h) {
        lsum_mf[h] = 0.0;
        c_mf[h] = C[MF ? 4 * h : 0];
        if constexpr (MF) {
#pragma unroll
            for (int i = 1; i < 4; ++i) c_mf[h] = i == g_own ? C[4 * h + i] : c_mf[h];
        }
    }

    // Residual rows are dealt to the waves RU wave-wide loads at a time (wave x takes loads RU*x ..
    // RU*x + RU - 1, then RU*NW further on): up to RU*NW*RPL residual slots cost each wave one
    // memory round trip per pass.
    constexpr int RU = Sh::RU;
    // ---- pass 1 (D1): logits of this workgroup's slots, exp(logit - C) into LDS ---------
    // Residual slots (fp32 rows, log-count term) and the incoming token itself come first: their
    // few rows are requested while the wave's first K tile is still on its way, so their round
    // trip hides behind that one instead of standing alone at the end of the pass.
    if (part == 0) {
        for (int t = RU * wave; t * RPL < Br; t += RU * NW)
            k_tile_masked<float, RU, D, G, EPL, LPR, RPL, QLDS, true>(Kr, t * RPL, Br, 0, nullptr, w, alpha, scale, qq, C,
                                                                      lsum, et, Bz, part_w, klane);
        if (wave == NW - 1)
            k_tile_masked<T, 1, D, G, EPL, LPR, RPL, QLDS>(knew, 0, 1, znew, nullptr, nullptr, alpha, scale, qq, C, lsum,
                                                           et, Bz, part_w, klane);
    }
    // Fast path (every token slot occupied): tiles are double-buffered in registers, the loads
    // of the wave's next tile (or of its first V tile) are in flight while it works on this one.
    if (full) {
        int t = tb + wave;
        if (SPLIT && t < te) {
            if constexpr (MF) tile_load_mfma4<T, UT, D, EPL>(bufA, Kt, t * R, ntok, lane);
            else tile_load<T, UT, D, EPL, LPR, RPL>(bufA, Kt, t * R, ntok, klane);
        }
        while (t < te) {
            const int tn = t + NW;
            prio_from_progress(t - tb, 2 * (te - tb));
            if (tn < te) {
                if constexpr (MF) tile_load_mfma4<T, UT, D, EPL>(bufB, Kt, tn * R, ntok, lane);
                else tile_load<T, UT, D, EPL, LPR, RPL>(bufB, Kt, tn * R, ntok, klane);
            } else {
                tile_load<T, UT, D, EPL, LPR, RPL>(bufB, Vt, (tb + wave) * R, ntok, lane);   // tb + wave < te here
            }
            if constexpr (G >= 2) __builtin_amdgcn_sched_barrier(0);   // the requests stay ahead of the tile's arithmetic
            if constexpr (MF)
                k_compute_mfma4<T, UT, EPL, NG>(bufA, qa, t * R, row_e, zt, scale, c_mf, lsum_mf, et + (size_t)g_own * Bz, Bz, lane);
            else if constexpr (G >= 2)
                k_compute_gq<T, D, G, EPL, LPR, RPL, QLDS>(bufA, t * R, row_e, zt, scale, qq, c_own, lsum_own, et, Bz, lane);
            else
                k_compute<T, UT, false, D, G, EPL, LPR, RPL, QLDS>(bufA, t * R, row_e, zt, nullptr, nullptr, alpha, scale, qq,
                                                                   C, lsum, et, Bz, part_w, lane);
#pragma unroll
            for (int u = 0; u < UT; ++u) bufA[u] = bufB[u];
            t = tn;
        }
    } else {
        for (int r0 = row_b + wave * RPL; r0 < row_e; r0 += NW * RPL)
            k_tile_masked<T, 1, D, G, EPL, LPR, RPL, QLDS>(Kt, r0, row_e, zt, pos + Br, nullptr, alpha, scale, qq, C, lsum,
                                                           et, Bz, part_w, klane);
    }
    // The wave's first tile of residual V rows and (last wave) the incoming token's V row are
    // requested before the barrier, so their round trip passes while the waves meet; rows whose
    // probability is exactly 0 (empty slots among them) are not loaded.  This wave wrote their
    // exponentials itself (the first of the loads pass 1 dealt to it).
    constexpr bool VPRE = G <= 4;   // eight query heads leave no registers for it: their rows are loaded where they are used
    constexpr bool VPRE2 = G <= 2;  // the wave's second load of residual rows is requested ahead too
    Raw<float, EPL> vres, vres2;
    Raw<T, EPL> vnw;
    vres.zero();
    vres2.zero();
    vnw.zero();
    if (VPRE && part == 0) {
        const int r = RU * wave * RPL + grp;
        bool any = false;
        if (r < Br) {
#pragma unroll
            for (int g = 0; g < G; ++g) any = any || (et[(size_t)g * Bz + r] != 0.0);
        }
        if (any) vres.load(Vr + (size_t)r * D + seg * EPL);
        if (wave == NW - 1 && grp == 0) vnw.load(vnew + seg * EPL);   // its probability is never 0: exp(0) / L
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
        double mine = (G >= 2 && !MF && g == g_own) ? lsum_own : 0.0;
        if constexpr (MF) mine = (g & 3) == g_own ? lsum_mf[g >> 2] : 0.0;
        const double t = wave_sum(lsum[g] + mine);
        if (lane == 0) red64[wave * G + g] = t;
    }
    __syncthreads();
    double rL[G];   // 1 / (this workgroup's softmax denominator)
#pragma unroll
    for (int g = 0; g < G; ++g) {
        double t = 0.0;
#pragma unroll
        for (int x = 0; x < NW; ++x) t += red64[x * G + g];
        rL[g] = SPLIT ? (t > 0.0 ? 1.0 / t : 0.0) : 1.0 / t;   // the unit's own denominator counts the incoming token: >= 1
        if (G > 1 && g >= Gr) rL[g] = 0.0;
        if (t >= SPREAD_FLAG_SUM && tid == 0) atomicOr(cv.flags + ug, FLAG_DECODE_SPREAD);   // practically never taken
    }

    // ---- pass 2 (D2): sum p * v over this workgroup's slots ------------------------------
    float acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    if (VPRE && part == 0) {
        // the wave's second load of residual V rows: requested now (every wave's exponentials are
        // visible after the barrier), used after the sweep of the token rows
        const int r2 = (RU * wave + 1) * RPL + grp;
        bool any2 = false;
        if (VPRE2 && r2 < Br) {
#pragma unroll
            for (int g = 0; g < G; ++g) any2 = any2 || (et[(size_t)g * Bz + r2] != 0.0);
        }
        if (any2) vres2.load(Vr + (size_t)r2 * D + seg * EPL);
        if (RU * wave * RPL < Br) v_compute<float, 1, D, G, EPL, LPR, RPL>(&vres, RU * wave * RPL, Br, 0, rL, acc, et, Bz, lane);
        if (wave == NW - 1) v_compute<T, 1, D, G, EPL, LPR, RPL>(&vnw, 0, 1, znew, rL, acc, et, Bz, lane);
    }
    if (full) {
        int t = tb + wave;   // bufA already holds this wave's first V tile
        while (t < te) {
            const int tn = t + NW;
            prio_from_progress(te - tb + t - tb, 2 * (te - tb));
            if (tn < te) tile_load<T, UT, D, EPL, LPR, RPL>(bufB, Vt, tn * R, ntok, lane);
            v_compute<T, UT, D, G, EPL, LPR, RPL>(bufA, t * R, row_e, zt, rL, acc, et, Bz, lane);
#pragma unroll
            for (int u = 0; u < UT; ++u) bufA[u] = bufB[u];
            t = tn;
        }
    } else {
        for (int r0 = row_b + wave * RPL; r0 < row_e; r0 += NW * RPL)
            v_tile_masked<T, 1, D, G, EPL, LPR, RPL>(Vt, r0, row_e, zt, rL, acc, et, Bz, lane);
    }
    __builtin_amdgcn_s_setprio(0);
    if (part == 0) {
        if (VPRE2 && (RU * wave + 1) * RPL < Br)
            v_compute<float, 1, D, G, EPL, LPR, RPL>(&vres2, (RU * wave + 1) * RPL, Br, 0, rL, acc, et, Bz, lane);
        // the residual loads not requested ahead
        for (int t = VPRE ? 0 : wave; t * RPL < Br; t += VPRE ? 1 : NW) {
            if (VPRE) {   // loads 0 .. RU*NW - 1 belong to wave t / RU; the later ones go round
                const int own = t < RU * NW ? t / RU : t % NW;
                if (own != wave || (t < RU * NW && (t % RU == 0 || (VPRE2 && t % RU == 1)))) continue;
            }
            v_tile_masked<float, 1, D, G, EPL, LPR, RPL>(Vr, t * RPL, Br, 0, rL, acc, et, Bz, lane);
        }
        if (!VPRE && wave == NW - 1)
            v_tile_masked<T, 1, D, G, EPL, LPR, RPL>(vnew, 0, 1, znew, rL, acc, et, Bz, lane);
    }

    // What the end of the step reads regardless of its decisions: requested now, used after the
    // output has been combined, so that part of the latency is hidden.  (Requested a pass earlier
    // the values do not fit the register budget and the spill makes every wave wait for them.)
    UnitRefs<T> u{Kt, Vt, Kr, Vr, s, pos, w, knew, vnew};
    FinishPre<T, D, NW> pre;
    if (!SPLIT && !POOL) pre.load(u, cv.cap, Br);
    // ---- combine the waves' partial outputs ----------------------------------------------
    // (fewer slots than waves: waves r*AW .. r*AW + AW - 1 take round r; the first round stores, the later ones add)
#pragma unroll
    for (int round = 0; round < NW / AW; ++round) {
        if (wave / AW == round) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    float v = acc[g][e];
#pragma unroll
                    for (int o = LPR; o < 64; o <<= 1) v += __shfl_xor(v, o, 64);
                    float* slot = &accw[((wave - round * AW) * G + g) * D + seg * EPL + e];
                    if (grp == 0) *slot = round == 0 ? v : *slot + v;
                }
            }
        }
        __syncthreads();
    }
    if (!SPLIT) {
        for (int idx = tid; idx < Gr * D; idx += NT) {
            float o = 0.f;
#pragma unroll
            for (int x = 0; x < AW; ++x) o += accw[x * G * D + idx];
            a.out[head_off * D + idx] = o;
        }
        if constexpr (POOL) {
            // slot j's exponentials sit at et[g][j], the incoming token's at et[g][B] (one workgroup per unit)
            double* pool = a.pool + ((size_t)lu * a.n_shares + share) * (cv.cap + 1);
            for (int j = tid; j <= B; j += NT) {
                double pm = 0.0;
#pragma unroll
                for (int g = 0; g < G; ++g) pm += et[(size_t)g * Bz + j] * rL[g];   // 1/L of the heads past the last is 0
                pool[j] = pm;
            }
        } else {
            decode_finish<T, D, G, NW, 0>(a, cv, u, lu, ug, Bp, Br, B, Tseen, nocc, full, et, Bz, rL, pre, keyw, dotw, misc);
        }
        return;
    }

    // ---- SPLIT: leave this part's share in scratch for decode_combine_kernel
    const int wg = blockIdx.x;
    const int BzG = cv.cap + 1;
    double* Eu = cv.sp_E + (size_t)lu * G * BzG;   // [G][cap + 1], indexed by slot (incoming token at B)
    for (int idx = tid; idx < G * D; idx += NT) {
        float o = 0.f;
#pragma unroll
        for (int x = 0; x < AW; ++x) o += accw[x * G * D + idx];
        cv.sp_acc[(size_t)wg * G * D + idx] = o;
    }
    if (tid < G) {
        double t = 0.0;
#pragma unroll
        for (int x = 0; x < NW; ++x) t += red64[x * G + tid];
        cv.sp_L[(size_t)wg * G + tid] = t;
    }
    for (int g = 0; g < G; ++g) {
        for (int i = tid; i < row_e - row_b; i += NT) Eu[(size_t)g * BzG + Br + row_b + i] = et[(size_t)g * Bz + Br + i];
        if (part == 0) {
            for (int i = tid; i < Br; i += NT) Eu[(size_t)g * BzG + i] = et[(size_t)g * Bz + i];
            if (tid == 0) Eu[(size_t)g * BzG + B] = et[(size_t)g * Bz + znew];
        }
    }
}

// Second kernel of a split step, one workgroup per unit: adds the parts' output shares up with
// weights L_p / L, writes the output and runs the score update, eviction, merge and token write
// from the per-slot values the parts left in scratch.  Latency-bound (a few dependent memory
// round trips), so everything whose address is known up front is requested up front.
template <typename T, int D, int G, int NW>
__global__ __launch_bounds__(NW * 64, G >= 8 ? 2 : 1) void decode_combine_kernel(DecodeArgs a) {
    constexpr int NT = NW * 64;
    constexpr int MAXP = 64;   // parts per unit (the host never asks for more)
    const CacheView& cv = a.cv;
    const int lu = blockIdx.x;
    const int ug = a.unit0 + lu;
    const int b = (ug / cv.H) % cv.S;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int Br = cv.Br, P = a.parts;
    const int Gr = real_heads<G>(cv);
    __shared__ unsigned long long keyw[NW];
    __shared__ double dotw[NW];
    __shared__ int misc[4 + NW];
    __shared__ double Lp[MAXP][G];
    __shared__ double Lsum[G];
    T* Kt = reinterpret_cast<T*>(cv.Kt) + (size_t)ug * cv.cap_tok * D;
    T* Vt = reinterpret_cast<T*>(cv.Vt) + (size_t)ug * cv.cap_tok * D;
    UnitRefs<T> u{Kt, Vt, cv.Kr + (size_t)ug * Br * D, cv.Vr + (size_t)ug * Br * D, cv.s + (size_t)ug * cv.cap,
                  cv.pos + (size_t)ug * cv.cap, cv.w + (size_t)ug * cv.cap,
                  reinterpret_cast<const T*>(a.k_new) + (size_t)lu * D, reinterpret_cast<const T*>(a.v_new) + (size_t)lu * D};
    const int BzG = cv.cap + 1;
    const double* Eu = cv.sp_E + (size_t)lu * G * BzG;
    FinishPre<T, D, NW, G> pre;
    pre.load(u, cv.cap, Br, Eu, BzG);
    const int wg0 = lu * P;
    // the parts' denominators: wave 0, lane p
    double lp[G];
#pragma unroll
    for (int g = 0; g < G; ++g) lp[g] = (wave == 0 && lane < P) ? cv.sp_L[(size_t)(wg0 + lane) * G + g] : 0.0;
    // the first parts' output shares of this thread's first channel (the rest after the barrier)
    constexpr int OPT = (G * D + NT - 1) / NT;   // outputs per thread
    constexpr int PPRE = 16;
    float vpre[PPRE];
#pragma unroll
    for (int p = 0; p < PPRE; ++p) vpre[p] = (p < P && tid < G * D) ? cv.sp_acc[(size_t)(wg0 + p) * G * D + tid] : 0.f;
    const int Bp = cv.Bp[b], Bc = cv.Bc[b];
    const int ntok = Bp + Bc, B = ntok + Br;
    const long long Tseen = cv.n_seen[ug];
    const int nocc = cv.n_occ[ug];
    const bool full = nocc == ntok;
    if (tid == 0) { misc[0] = -1; misc[2] = 0x7fffffff; }
    if (wave == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (lane < P) Lp[lane][g] = lp[g];
            const double t = wave_sum(lp[g]);
            if (lane == 0) Lsum[g] = t;
        }
    }
    __syncthreads();
    double rL[G];
#pragma unroll
    for (int g = 0; g < G; ++g) rL[g] = (G > 1 && g >= Gr) ? 0.0 : 1.0 / Lsum[g];   // part 0 counted the incoming token: the sum is >= 1
#pragma unroll
    for (int x = 0; x < OPT; ++x) {
        const int idx = x * NT + tid;
        if (idx >= Gr * D) break;
        const int g = idx / D;
        double rl = 0.0;
#pragma unroll
        for (int gg = 0; gg < G; ++gg) rl = gg == g ? rL[gg] : rl;
        float o = 0.f;
        int p = 0;
        if (x == 0) {
#pragma unroll
            for (int y = 0; y < PPRE; ++y)
                if (y < P) o = fmaf((float)(Lp[y][g] * rl), vpre[y], o);
            p = P < PPRE ? P : PPRE;
        }
        for (; p + 4 <= P; p += 4) {
            float v[4];
#pragma unroll
            for (int y = 0; y < 4; ++y) v[y] = cv.sp_acc[(size_t)(wg0 + p + y) * G * D + idx];
#pragma unroll
            for (int y = 0; y < 4; ++y) o = fmaf((float)(Lp[p + y][g] * rl), v[y], o);
        }
        for (; p < P; ++p) o = fmaf((float)(Lp[p][g] * rl), cv.sp_acc[(size_t)(wg0 + p) * G * D + idx], o);
        a.out[(size_t)lu * Gr * D + idx] = o;
    }
    decode_finish<T, D, G, NW, G>(a, cv, u, lu, ug, Bp, Br, B, Tseen, nocc, full, Eu, BzG, rL, pre, keyw, dotw, misc);
}

// Second kernel of a step over groups of more than eight query heads, one workgroup per unit: the per-slot sums the
// shares left in a.pool are added up in the order of the heads and become the head mean (sum / G, as the appendix's grouped-query adaptation pools the heads),
// then D3-D6 as for a single head whose probabilities are those means.
template <typename T, int D, int NW>
__global__ __launch_bounds__(NW * 64) void decode_pool_finish_kernel(DecodeArgs a) {
    constexpr int NT = NW * 64;
    const CacheView& cv = a.cv;
    const int lu = blockIdx.x;
    const int ug = a.unit0 + lu;
    const int b = (ug / cv.H) % cv.S;
    const int tid = threadIdx.x;
    const int Br = cv.Br;
    __shared__ unsigned long long keyw[NW];
    __shared__ double dotw[NW];
    __shared__ int misc[4 + NW];
    T* Kt = reinterpret_cast<T*>(cv.Kt) + (size_t)ug * cv.cap_tok * D;
    T* Vt = reinterpret_cast<T*>(cv.Vt) + (size_t)ug * cv.cap_tok * D;
    UnitRefs<T> u{Kt, Vt, cv.Kr + (size_t)ug * Br * D, cv.Vr + (size_t)ug * Br * D, cv.s + (size_t)ug * cv.cap,
                  cv.pos + (size_t)ug * cv.cap, cv.w + (size_t)ug * cv.cap,
                  reinterpret_cast<const T*>(a.k_new) + (size_t)lu * D, reinterpret_cast<const T*>(a.v_new) + (size_t)lu * D};
    FinishPre<T, D, NW> pre;
    pre.load(u, cv.cap, Br);
    const int Bp = cv.Bp[b], Bc = cv.Bc[b];
    const int ntok = Bp + Bc, B = ntok + Br;
    const long long Tseen = cv.n_seen[ug];
    const int nocc = cv.n_occ[ug];
    const bool full = nocc == ntok;
    if (tid == 0) { misc[0] = -1; misc[2] = 0x7fffffff; }
    double* pool = a.pool + (size_t)lu * a.n_shares * (cv.cap + 1);   // the sums end up in the first share's slice
    const double heads = (double)a.q_heads;
    for (int j = tid; j <= B; j += NT) {
        double t = pool[j];
        for (int sh = 1; sh < a.n_shares; ++sh) t += pool[(size_t)sh * (cv.cap + 1) + j];
        pool[j] = t / heads;
    }
    __threadfence_block();
    __syncthreads();
    const double one[1] = {1.0};
    decode_finish<T, D, 1, NW, 0>(a, cv, u, lu, ug, Bp, Br, B, Tseen, nocc, full, pool, cv.cap + 1, one, pre, keyw, dotw, misc);
}

// Host side: pick the instantiation for (D, G) and launch.
constexpr int DECODE_NW = 4;
constexpr size_t DECODE_LDS_MAX = 160 * 1024;   // LDS of one compute unit

// Waves per workgroup.  Four, unless the per-slot values of one workgroup (G * (slots + 1) * 8 bytes of LDS) leave
// room for fewer workgroups per compute unit than the registers would allow waves: then a workgroup of 8, 12 or 16
// waves keeps the compute unit's SIMDs supplied with loads in flight (measured at four query heads and B = 2700,
// where only one workgroup fits: 0.336 ms with 4 waves, 0.285 with 8, 0.281 with 12; a single query head at
// B = 12000: 1.25 ms with 4 waves, 1.08 with 16).  Where two or more workgroups of four waves fit they stay: at
// B = 6000 two of them stream as fast as sixteen waves do, and with three resident, as at four query heads and
// B = 1024, larger workgroups lose to the serial stretches of a unit.
template <typename T, int D, int G, bool SPLIT, int NWK, int AWK = NWK>
inline hipError_t launch_decode_nw(const DecodeArgs& a, hipStream_t stream);

// Lets a kernel use a compute unit's whole LDS as dynamic shared memory.  The attribute is per device; bit `dev` of
// `done` (one flag per kernel) records that it has been set there.  Two host threads that meet here for the first
// time may both set it (harmless: same value), neither reads a torn flag.
inline hipError_t allow_whole_lds(const void* kern, std::atomic<unsigned long long>& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = 1ull << (dev & 63);
    if (!(done.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        done.fetch_or(bit, std::memory_order_release);
    }
    return hipSuccess;
}

// waves a compute unit holds of this kernel by its registers (the launch bound's waves per SIMD, times four)
template <typename T, int D, int G>
constexpr int decode_cu_waves() { return G == 1 ? 16 : ((G == 4 && DecodeShape<T, D, G, DECODE_NW>::MFMA4) ? 12 : 8); }

// LDS slots for the waves' partial outputs: one per wave, or two where that lets a second workgroup of four waves
// into a compute unit (eight query heads: 16 KB against 8 KB of staging; measured at B = 1024, 4096 units:
// 0.72 ms per step with one workgroup of eight waves per compute unit, 0.58 with two of four)
template <typename T, int D, int G, int NWK>
inline int decode_out_slots(int nz) {
    if constexpr (G == 8 && NWK == 4) {
        using Sh = DecodeShape<T, D, G, NWK>;
        if (DECODE_LDS_MAX / Sh::lds_bytes(nz, 2) >= 2 && DECODE_LDS_MAX / Sh::lds_bytes(nz, NWK) < 2) return 2;
    }
    return NWK;
}

template <typename T, int D, int G, int NWK>
inline int decode_resident_waves(int nz) {
    const size_t lds = DecodeShape<T, D, G, NWK>::lds_bytes(nz, decode_out_slots<T, D, G, NWK>(nz));
    if (lds > DECODE_LDS_MAX) return 0;
    const int by_lds = (int)(DECODE_LDS_MAX / lds) * NWK, by_regs = decode_cu_waves<T, D, G>() / NWK * NWK;
    return by_lds < by_regs ? by_lds : by_regs;
}

template <typename T, int D, int G, bool SPLIT>
inline hipError_t launch_decode_dgs(const DecodeArgs& a, hipStream_t stream) {
    if constexpr (!SPLIT) {
        const int nz = a.cv.cap + 1;
        const int w4 = decode_resident_waves<T, D, G, 4>(nz), w8 = decode_resident_waves<T, D, G, 8>(nz);
        constexpr int NWX = G == 1 ? 16 : 12;   // the largest workgroup of this kernel, where it has one
        constexpr bool HAS_X = decode_cu_waves<T, D, G>() >= NWX;
        int wx = 0;
        if constexpr (HAS_X) wx = decode_resident_waves<T, D, G, NWX>(nz);
        if (w4 <= 4 && (w8 > w4 || wx > w4)) {   // two resident workgroups of four waves already stream at the full rate
            if constexpr (HAS_X) {
                if (wx > w8) return launch_decode_nw<T, D, G, SPLIT, NWX>(a, stream);
            }
            return launch_decode_nw<T, D, G, SPLIT, 8>(a, stream);
        }
    }
    return launch_decode_nw<T, D, G, SPLIT, DECODE_NW>(a, stream);
}

template <typename T, int D, int G, bool SPLIT, int NWK, int AWK>
inline hipError_t launch_decode_nw(const DecodeArgs& a, hipStream_t stream) {
    using Sh = DecodeShape<T, D, G, NWK>;
    const int nz = SPLIT ? a.part_rows + a.cv.Br + 1 : a.cv.cap + 1;
    if constexpr (G == 8 && NWK == 4 && !SPLIT && AWK == NWK) {
        if (decode_out_slots<T, D, G, NWK>(nz) == 2) return launch_decode_nw<T, D, G, SPLIT, NWK, 2>(a, stream);
    }
    const size_t lds = Sh::lds_bytes(nz, AWK);
    auto kern = decode_kernel<T, D, G, NWK, SPLIT, AWK>;
    static std::atomic<unsigned long long> attr_done{0ull};
    const hipError_t e = allow_whole_lds(reinterpret_cast<const void*>(kern), attr_done);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(a.n_units * (SPLIT ? a.parts : 1)), dim3(NWK * 64), lds, stream, a);
    if (SPLIT) hipLaunchKernelGGL((decode_combine_kernel<T, D, G, DECODE_NW>), dim3(a.n_units), dim3(DECODE_NW * 64), 0, stream, a);
    return hipGetLastError();
}

template <typename T, int D, int G>
inline hipError_t launch_decode_dg(const DecodeArgs& a, hipStream_t stream) {
    return a.parts > 1 ? launch_decode_dgs<T, D, G, true>(a, stream) : launch_decode_dgs<T, D, G, false>(a, stream);
}

template <typename T, int D, int G>
inline size_t decode_lds_dg(int nz) { return DecodeShape<T, D, G, DECODE_NW>::lds_bytes(nz); }

// rows of one wave tile for a K/V element size (the unit the parts of a split step are cut in)
inline int decode_tile_rows(int D, int esize) { return DecodeShape<float, 64, 1, DECODE_NW>::UT * (64 / (D * esize / 16)); }

// the compiled number of query heads that serves a cache with G of them (1..8)
inline int decode_compiled_heads(int G) { return G <= 2 ? G : (G <= 4 ? 4 : 8); }

template <typename T>
inline hipError_t launch_decode_t(const DecodeArgs& a, hipStream_t stream) {
    const int D = a.cv.D, G = decode_compiled_heads(a.cv.G);
#define ZSM_CASE(DD, GG) if (D == DD && G == GG) return launch_decode_dg<T, DD, GG>(a, stream);
    ZSM_CASE(64, 1) ZSM_CASE(64, 2) ZSM_CASE(64, 4) ZSM_CASE(64, 8)
    ZSM_CASE(128, 1) ZSM_CASE(128, 2) ZSM_CASE(128, 4) ZSM_CASE(128, 8)
#undef ZSM_CASE
    return hipErrorInvalidValue;
}

// A step over groups of more than eight query heads: one workgroup per unit and share of GS heads (the eight-head
// kernel, or the four-head kernel where the per-slot values of eight heads do not fit the LDS), then the finishing
// kernel.  a.q_heads, a.n_shares (= ceil(q_heads / GS)), a.pool, a.n_units, a.unit0 and the tensors are set by the caller.
template <typename T, int D, int GS>
inline hipError_t launch_decode_pooled_share(DecodeArgs a, hipStream_t stream) {
    using Sh = DecodeShape<T, D, GS, DECODE_NW>;
    const size_t lds = Sh::lds_bytes(a.cv.cap + 1);
    auto kern = decode_kernel<T, D, GS, DECODE_NW, false, DECODE_NW, true>;
    static std::atomic<unsigned long long> attr_done{0ull};
    const hipError_t e = allow_whole_lds(reinterpret_cast<const void*>(kern), attr_done);
    if (e != hipSuccess) return e;
    a.parts = 1;
    a.part_rows = 0;
    hipLaunchKernelGGL(kern, dim3((a.n_units + 7) / 8 * 8 * a.n_shares), dim3(DECODE_NW * 64), lds, stream, a);
    hipLaunchKernelGGL((decode_pool_finish_kernel<T, D, DECODE_NW>), dim3(a.n_units), dim3(DECODE_NW * 64), 0, stream, a);
    return hipGetLastError();
}

// waves of the four-wave kernel for GS heads that a compute unit holds at `nz` per-slot values (0: one workgroup does not fit)
template <typename T, int D, int GS>
inline int decode_pool_resident_waves(int nz) {
    const size_t lds = DecodeShape<T, D, GS, DECODE_NW>::lds_bytes(nz);
    if (lds > DECODE_LDS_MAX) return 0;
    const int by_lds = (int)(DECODE_LDS_MAX / lds) * DECODE_NW, by_regs = decode_cu_waves<T, D, GS>();
    return by_lds < by_regs ? by_lds : by_regs;
}

// Heads per share of a pooled step: 8, or 4 where that keeps more waves resident on a compute unit (the per-slot
// values of 8 heads leave room for one workgroup from B of about 1000 on, those of 4 for two or three; measured
// on 512 units of 71 heads, d = 64: 0.43 against 0.49 ms at B = 1024, where both have two workgroups resident, 0.85
// against 0.64 at B = 1500; d = 128, 256 units: 0.42 against 0.33 at B = 1024).  0: neither fits.
template <typename T, int D>
inline int decode_pool_share_heads(int nz) {
    const int w8 = decode_pool_resident_waves<T, D, 8>(nz), w4 = decode_pool_resident_waves<T, D, 4>(nz);
    if (w8 == 0 && w4 == 0) return 0;
    return w4 > w8 ? 4 : 8;
}

template <typename T, int D>
inline hipError_t launch_decode_pooled_d(const DecodeArgs& a, hipStream_t stream) {
    switch (decode_pool_share_heads<T, D>(a.cv.cap + 1)) {
        case 8: return launch_decode_pooled_share<T, D, 8>(a, stream);
        case 4: return launch_decode_pooled_share<T, D, 4>(a, stream);
        default: return hipErrorInvalidValue;
    }
}

template <typename T>
inline int decode_pool_share_heads_t(int D, int nz) {
    return D == 64 ? decode_pool_share_heads<T, 64>(nz) : (D == 128 ? decode_pool_share_heads<T, 128>(nz) : 0);
}

template <typename T>
inline hipError_t launch_decode_pooled_t(const DecodeArgs& a, hipStream_t stream) {
    if (a.cv.D == 64) return launch_decode_pooled_d<T, 64>(a, stream);
    if (a.cv.D == 128) return launch_decode_pooled_d<T, 128>(a, stream);
    return hipErrorInvalidValue;
}

// LDS bytes of a launch that keeps `nz` per-slot values per query head in LDS
template <typename T>
inline size_t decode_lds_t(int D, int Gr, int nz) {
    const int G = decode_compiled_heads(Gr);
#define ZSM_CASE(DD, GG) if (D == DD && G == GG) return decode_lds_dg<T, DD, GG>(nz);
    ZSM_CASE(64, 1) ZSM_CASE(64, 2) ZSM_CASE(64, 4) ZSM_CASE(64, 8)
    ZSM_CASE(128, 1) ZSM_CASE(128, 2) ZSM_CASE(128, 4) ZSM_CASE(128, 8)
#undef ZSM_CASE
    return (size_t)-1;
}

// one translation unit per dtype provides these
hipError_t launch_decode_f32(const DecodeArgs& a, hipStream_t stream);
hipError_t launch_decode_f16(const DecodeArgs& a, hipStream_t stream);
hipError_t launch_decode_bf16(const DecodeArgs& a, hipStream_t stream);
hipError_t launch_decode_pooled_f32(const DecodeArgs& a, hipStream_t stream);
hipError_t launch_decode_pooled_f16(const DecodeArgs& a, hipStream_t stream);
hipError_t launch_decode_pooled_bf16(const DecodeArgs& a, hipStream_t stream);
int decode_pool_share_heads_f32(int D, int nz);
int decode_pool_share_heads_f16(int D, int nz);
int decode_pool_share_heads_bf16(int D, int nz);
size_t decode_lds_f32(int D, int G, int nz);
size_t decode_lds_f16(int D, int G, int nz);
size_t decode_lds_bf16(int D, int G, int nz);

}  // namespace zsm
