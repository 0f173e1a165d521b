// One-shot prefill compression: score every prompt token, keep the latest B_p and the
// top-B_c, fold the rest into the residual slot (Sec. 3.2, Eq. 3, Alg. 1 residual branch;
// appendix "Implementation Details" for the query window).
#pragma once

#include "zsm_common.hpp"

namespace zsm {

struct PrefillArgs {
    CacheView cv;
    int32_t unit0;      // first global unit of the call's first layer
    int32_t n_units;    // layers of this launch group * S * H
    const void* Q;      // [layers][S][H][G][W][D]
    const void* K;      // [layers][S][H][T_max][D]
    const void* V;
    const int32_t* seq_lens;   // [S]
    int32_t W, T_max;
    char* ws;
};

constexpr int PF_MR = 32;      // query rows per pass of the scoring kernels (two 16-row matrix blocks)
constexpr int PF_KQ = 128;     // granule of a workgroup's key range in the scoring kernels (4 waves x 32 keys)
constexpr int PF_SCORE_WGS = 1024;   // scoring launches aim at this many workgroups (4 per compute unit, one round)
constexpr int PF_RC = 1024;    // prompt positions per workgroup in the residual sum

struct PrefillWs {
    size_t Qd, pl, rowm, roww, sc, sacc, ev, keep, kept_pos, sel, rsum, total;
    int Wp, nsums, chunk_keys, nchunks;   // nsums key ranges of chunk_keys keys per unit in the scoring kernels
    int multi;                            // more than one (query head, 32-row block) per unit: scores pass through sacc
    int rz;                               // groups the passes of a unit are dealt to (grid.z of the scoring launches)
    int fold;                             // a workgroup takes key ranges x and nsums-1-x
    int store_e;                          // the first sweep keeps every exp(z - C) (ev), the scores are summed from there
    int ev_units;                         // store_e: units per scoring launch (their exponentials fit PF_EV_MAX)
    int lu0;                              // store_e: first unit of the current scoring launch (set by the launcher)
};

// The exponentials of the first scoring sweep are kept, and the second sweep of K replaced by a
// weighted column sum over them; a call is scored in batches of units whose exponentials (fp64,
// rows x T_max per unit) fit this many bytes.
constexpr size_t PF_EV_MAX = (size_t)1 << 30;

// Units one group of launches may cover (grid dimension y of the per-unit kernels); a call with more is
// worked off in groups of whole layers.
constexpr int PF_MAX_GROUP_UNITS = 32768;

// whole layers per launch group for a call of n_layers layers (0: a single layer has too many units)
inline int prefill_group_layers(const CacheView& cv, int n_layers) {
    const long long lu = (long long)cv.S * cv.H;
    if (lu > PF_MAX_GROUP_UNITS) return 0;
    const long long g = PF_MAX_GROUP_UNITS / lu;
    return (int)(g < n_layers ? g : n_layers);
}

// layout for launches that cover `n_units` units at a time
inline PrefillWs prefill_ws_layout(const CacheView& cv, int n_units, int T_max, int W) {
    PrefillWs w{};
    const size_t units = (size_t)n_units;
    w.Wp = (W + PF_MR - 1) / PF_MR * PF_MR;
    {
        // Work of the scoring launches: (unit, key range, group of 32-row passes).  With one pass
        // per unit the key ranges alone make up about PF_SCORE_WGS workgroups; with many passes
        // (a long window, grouped queries) the passes are dealt round-robin to up to 8 groups, so
        // that a key range stays long enough to pay for re-staging the query block every pass.
        const int npass = cv.G * (w.Wp / PF_MR);
        w.multi = npass > 1;
        w.rz = npass >= 8 ? (npass / 4 < 8 ? npass / 4 : 8) : 1;
        // Rows attend to keys up to their own position only, so with many row blocks the early key
        // ranges carry far more work than the late ones: a workgroup then takes key range x together
        // with range nsums-1-x ("fold"), which evens the work out whatever XCD the workgroup lands on.
        w.fold = w.rz > 1 && 2 * (long long)W >= T_max;   // a short window sits at the end of the prompt: every key range sees all of it
        const size_t ev_unit = sizeof(double) * cv.G * w.Wp * (size_t)T_max;          // exponentials of one unit
        w.store_e = !w.fold && ev_unit <= PF_EV_MAX && units > 0;
        w.ev_units = w.store_e ? (int)(PF_EV_MAX / ev_unit < units ? PF_EV_MAX / ev_unit : units) : 0;
        if (w.store_e && (size_t)w.ev_units < units) {
            // Several batches: a batch of u units is scored by u * (wgs / (u * rz)) * rz workgroups, one round of
            // at most `wgs` resident ones.  Take the batch size (at least half the largest that fits) that wastes the
            // fewest workgroup slots, the ragged last batch counted.
            const int wgs1 = PF_SCORE_WGS / 4 * 3;
            double best = -1.0;
            int best_u = w.ev_units;
            for (int u = w.ev_units; u >= (w.ev_units + 1) / 2; --u) {
                const int per_unit = w.rz * (wgs1 / (u * w.rz) > 0 ? wgs1 / (u * w.rz) : 1);   // workgroups per unit
                const int nb = (int)(units / u), rem = (int)(units % u);
                const double f = ((double)nb * u + rem) * per_unit / ((double)(nb + (rem ? 1 : 0)) * wgs1);
                if (f > best + 1e-9) { best = f; best_u = u; }
            }
            w.ev_units = best_u;
        }
        const size_t su = w.store_e ? (size_t)w.ev_units : units;                     // units per scoring launch
        // one round of workgroups: 4 per compute unit, 3 for the sweep that also stores its exponentials (more registers)
        const int wgs = w.store_e ? PF_SCORE_WGS / 4 * 3 : PF_SCORE_WGS;
        int n = wgs / (int)((su > 0 ? su : 1) * w.rz) * (w.fold ? 2 : 1);
        const int most = (T_max + PF_KQ - 1) / PF_KQ;
        n = n < 1 ? 1 : (n > most ? most : n);
        w.chunk_keys = ((T_max + n - 1) / n + PF_KQ - 1) / PF_KQ * PF_KQ;
        w.nsums = (T_max + w.chunk_keys - 1) / w.chunk_keys;
    }
    w.nchunks = (T_max + PF_RC - 1) / PF_RC;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    size_t o = 0;
    w.Qd = o; o += up(sizeof(double) * units * cv.G * w.Wp * cv.D);
    w.pl = o; o += up(sizeof(double) * units * cv.G * w.Wp * w.nsums);
    w.rowm = o; o += up(sizeof(double) * units * cv.G * w.Wp);
    w.roww = o; o += up(sizeof(double) * units * cv.G * w.Wp);
    w.sc = o; o += up(sizeof(float) * units * T_max);
    w.ev = o; o += up(w.store_e ? sizeof(double) * (size_t)w.ev_units * T_max * cv.G * w.Wp : 0);   // [ev_units][T_max][G * Wp]
    w.sacc = o; o += up(w.multi && !w.store_e ? sizeof(double) * w.rz * units * T_max : 0);   // [rz][units][T_max]
    w.keep = o; o += up(units * (size_t)T_max);
    w.kept_pos = o; o += up(sizeof(int32_t) * units * (cv.cap_tok > 0 ? cv.cap_tok : 1));
    w.sel = o; o += up(sizeof(int32_t) * units * 4);
    w.rsum = o; o += up(sizeof(double) * units * w.nchunks * 2 * cv.D);
    w.total = o;
    return w;
}

inline size_t prefill_workspace_bytes(const CacheView& cv, int n_layers, int T_max, int W) {
    const int gl = prefill_group_layers(cv, n_layers);
    return gl > 0 ? prefill_ws_layout(cv, gl * cv.S * cv.H, T_max, W).total : 0;
}

hipError_t launch_prefill(const PrefillArgs& a, hipStream_t stream);

}  // namespace zsm
