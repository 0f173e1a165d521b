// One-shot prefill compression: score every prompt token, keep the latest B_p and the
// top-B_c, fold the rest into the residual slot (Sec. 3.2, Eq. 3, Alg. 1 residual branch;
// appendix "Implementation Details" for the query window).
#pragma once

#include "zsm_common.hpp"

namespace zsm {

struct PrefillArgs {
    CacheView cv;
    int32_t unit0;      // first global unit of the layer
    int32_t n_units;    // S * H
    const void* Q;      // [S][H][G][W][D]
    const void* K;      // [S][H][T_max][D]
    const void* V;
    const int32_t* seq_lens;   // [S]
    int32_t W, T_max;
    char* ws;
};

constexpr int PF_TK = 256;     // keys per workgroup pass in the scoring kernels (one per thread)
constexpr int PF_KCH = 4;      // key passes per workgroup in the row-sum kernel (PF_TK * PF_KCH keys)
constexpr int PF_MR = 32;      // query rows per pass
constexpr int PF_RC = 512;     // prompt positions per workgroup in the residual sum

struct PrefillWs {
    size_t Qd, pl, rowm, roww, sc, keep, kept_pos, sel, rsum, total;
    int Wp, ntiles, nsums, nchunks;
};

inline PrefillWs prefill_ws_layout(const CacheView& cv, int T_max, int W) {
    PrefillWs w{};
    const size_t units = (size_t)cv.S * cv.H;
    w.Wp = (W + PF_MR - 1) / PF_MR * PF_MR;
    w.ntiles = (T_max + PF_TK - 1) / PF_TK;
    w.nsums = (T_max + PF_TK * PF_KCH - 1) / (PF_TK * PF_KCH);
    w.nchunks = (T_max + PF_RC - 1) / PF_RC;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    size_t o = 0;
    w.Qd = o; o += up(sizeof(double) * units * cv.G * w.Wp * cv.D);
    w.pl = o; o += up(sizeof(double) * units * cv.G * w.Wp * w.nsums);
    w.rowm = o; o += up(sizeof(double) * units * cv.G * w.Wp);
    w.roww = o; o += up(sizeof(double) * units * cv.G * w.Wp);
    w.sc = o; o += up(sizeof(float) * units * T_max);
    w.keep = o; o += up(units * (size_t)T_max);
    w.kept_pos = o; o += up(sizeof(int32_t) * units * (cv.cap_tok > 0 ? cv.cap_tok : 1));
    w.sel = o; o += up(sizeof(int32_t) * units * 4);
    w.rsum = o; o += up(sizeof(double) * units * w.nchunks * 2 * cv.D);
    w.total = o;
    return w;
}

inline size_t prefill_workspace_bytes(const CacheView& cv, int T_max, int W) {
    return prefill_ws_layout(cv, T_max, W).total;
}

hipError_t launch_prefill(const PrefillArgs& a, hipStream_t stream);

}  // namespace zsm
