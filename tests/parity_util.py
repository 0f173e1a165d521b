"""Shared machinery of the GPU-vs-oracle parity tests.

The GPU side is called through the C ABI (paper_2503_10714_amd.binding); the oracle side
is oracle/zsmerge_oracle.py (unit by unit) or oracle/zsmerge_oracle_c.c (every unit of a layer
at once).  Both get the same bytes: inputs are generated once (on the
device the test says) and copied.

Tolerances (the benchmark definition's): slot indices, counts, positions and eviction
choices bit-exact, except that the device may pick another eviction victim (or another
boundary token in the prefill selection) when the oracle's competing scores differ by
less than 1e-6 relative; outputs, merged K/V and scores within max-abs 2e-3 for
fp16/bf16 storage and 1e-5 for fp32.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

from oracle.zsmerge_oracle import UnitCache
from paper_2503_10714_amd import synth

TIE_REL = 1e-6


def tol_for(dtype: str) -> float:
    return 1e-5 if dtype == "f32" else 2e-3


def lam32(x: float) -> float:
    """The decay / alpha value the library actually uses: the fp32 config field widened to fp64."""
    return float(np.float32(x))


def np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


# ---------------------------------------------------------------------------------------
# oracle <-> tensors
# ---------------------------------------------------------------------------------------

def new_oracle_unit(wl: synth.Workload, b_local: int) -> UnitCache:
    bp, bc, br = wl.budgets()
    return UnitCache(wl.head_dim, wl.q_per_kv, bp[b_local], bc[b_local], br,
                     lam=lam32(wl.lam), alpha=lam32(wl.alpha))


def pack_states(units: List[List[UnitCache]], cap: int, Br: int, d: int, kv_dtype: torch.dtype) -> Dict[str, torch.Tensor]:
    """Oracle states of one layer ([S][H] UnitCache) -> the export/import arrays (CPU tensors)."""
    S, H = len(units), len(units[0])
    K = torch.zeros(S, H, cap - Br, d, dtype=torch.float64)
    V = torch.zeros(S, H, cap - Br, d, dtype=torch.float64)
    Kr = torch.zeros(S, H, Br, d, dtype=torch.float64)
    Vr = torch.zeros(S, H, Br, d, dtype=torch.float64)
    s = torch.zeros(S, H, cap, dtype=torch.float64)
    pos = torch.full((S, H, cap), -1, dtype=torch.int32)
    w = torch.zeros(S, H, cap, dtype=torch.int32)
    n_seen = torch.zeros(S, H, dtype=torch.int64)
    for b in range(S):
        for h in range(H):
            u = units[b][h]
            B = u.B
            K[b, h, :B - Br] = torch.from_numpy(u.K[Br:])
            V[b, h, :B - Br] = torch.from_numpy(u.V[Br:])
            Kr[b, h] = torch.from_numpy(u.K[:Br])
            Vr[b, h] = torch.from_numpy(u.V[:Br])
            s[b, h, :B] = torch.from_numpy(u.s)
            pos[b, h, :B] = torch.from_numpy(u.pos.astype(np.int32))
            w[b, h, :B] = torch.from_numpy(u.w.astype(np.int32))
            n_seen[b, h] = u.n_seen
    return dict(K=K.to(torch.float32).to(kv_dtype), V=V.to(torch.float32).to(kv_dtype), Kr=Kr.to(torch.float32),
                Vr=Vr.to(torch.float32), s=s.to(torch.float32), pos=pos, w=w, n_seen=n_seen)


@dataclass
class Mismatch:
    what: str
    detail: str


def compare_state(gpu: Dict[str, torch.Tensor], units: List[List[UnitCache]], Br: int, tol: float,
                  where: str = "", sel: Optional[Sequence[Tuple[int, int]]] = None) -> None:
    """Exported GPU state of one layer vs the oracle units: integers exact, floats within tol.
    `sel` restricts the comparison to some (b, h) pairs (units[b][h] may be None elsewhere)."""
    g = {k: v.cpu() for k, v in gpu.items()}
    S, H = len(units), len(units[0])
    pairs = sel if sel is not None else [(b, h) for b in range(S) for h in range(H)]
    for b, h in pairs:
        u = units[b][h]
        B = u.B
        tag = f"{where} unit(b={b},h={h})"
        assert int(g["n_seen"][b, h]) == u.n_seen, f"{tag}: n_seen {int(g['n_seen'][b, h])} != {u.n_seen}"
        gp = g["pos"][b, h, :B].numpy().astype(np.int64)
        gw = g["w"][b, h, :B].numpy().astype(np.int64)
        assert (gw == u.w).all(), f"{tag}: w differs at slots {np.flatnonzero(gw != u.w)[:8]}"
        occ = u.w > 0
        assert (gp[occ] == u.pos[occ]).all(), f"{tag}: pos differs at slots {np.flatnonzero((gp != u.pos) & occ)[:8]}"
        assert (g["pos"][b, h, B:] == -1).all() and (g["w"][b, h, B:] == 0).all(), f"{tag}: slots past B touched"
        tok = occ[Br:]
        gK = np64(g["K"][b, h, :B - Br]); gV = np64(g["V"][b, h, :B - Br])
        assert (gK[tok] == u.K[Br:][tok]).all(), f"{tag}: token K rows differ"
        assert (gV[tok] == u.V[Br:][tok]).all(), f"{tag}: token V rows differ"
        if Br:
            ro = occ[:Br]
            dk = np.abs(np64(g["Kr"][b, h]) - u.K[:Br])[ro]
            dv = np.abs(np64(g["Vr"][b, h]) - u.V[:Br])[ro]
            if dk.size:
                assert dk.max() <= tol and dv.max() <= tol, f"{tag}: residual K/V off by {dk.max():.3e}/{dv.max():.3e}"
        ds = np.abs(np64(g["s"][b, h, :B]) - u.s)[occ]
        if ds.size:
            assert ds.max() <= tol, f"{tag}: scores off by {ds.max():.3e}"


@dataclass
class StepStats:
    steps: int = 0
    unit_steps: int = 0
    near_ties: int = 0
    max_out_err: float = 0.0
    evictions: int = 0
    merges: int = 0
    s_bit_equal: int = 0
    s_total: int = 0


def check_step(out_gpu: np.ndarray, info_gpu, out_or: np.ndarray, info_or, unit: UnitCache, tol: float,
               stats: StepStats, tag: str) -> bool:
    """One unit, one decode step.  Returns True when the device legitimately took another
    eviction victim (a near tie) and the two sides have to be brought together again."""
    err = float(np.abs(out_gpu - out_or).max())
    stats.max_out_err = max(stats.max_out_err, err)
    assert err <= tol, f"{tag}: attention output off by {err:.3e} (tol {tol})"
    ws, ep, ms = info_gpu
    stats.unit_steps += 1
    if info_or.evicted_pos >= 0:
        stats.evictions += 1
    if info_or.merged_slot >= 0:
        stats.merges += 1
    if ep == info_or.evicted_pos and ws == info_or.write_slot:
        assert ms == info_or.merged_slot, f"{tag}: merged_slot {ms} != {info_or.merged_slot}"
        return False
    # another victim: allowed only inside the near-tie band of the oracle's own scores
    assert info_or.evicted_pos >= 0 and ep >= 0, f"{tag}: write_slot/evicted_pos {ws}/{ep} vs {info_or.write_slot}/{info_or.evicted_pos}"
    cp = info_or.cand_pos.tolist()
    assert ep in cp, f"{tag}: device evicted position {ep}, which is not a candidate"
    s_dev = float(info_or.cand_s[cp.index(ep)])
    s_best = float(info_or.cand_s[cp.index(info_or.evicted_pos)])
    rel = abs(s_dev - s_best) / max(abs(s_best), 1e-300)
    assert rel < TIE_REL, f"{tag}: device evicted pos {ep} (s={s_dev:.9e}) but the lowest score is pos {info_or.evicted_pos} (s={s_best:.9e}), rel gap {rel:.2e}"
    stats.near_ties += 1
    return True


# ---------------------------------------------------------------------------------------
# drivers
# ---------------------------------------------------------------------------------------

def oracle_prefill_layer(wl: synth.Workload, Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, lens: Sequence[int],
                         sel: Optional[Sequence[Tuple[int, int]]] = None) -> List[List[Optional[UnitCache]]]:
    """Oracle prefill of one layer from the tensors the device got (any device)."""
    S, H = K.shape[0], K.shape[1]
    units: List[List[Optional[UnitCache]]] = [[None] * H for _ in range(S)]
    pairs = sel if sel is not None else [(b, h) for b in range(S) for h in range(H)]
    for b, h in pairs:
        u = new_oracle_unit(wl, b)
        tb = lens[b]
        nb = min(Q.shape[3], tb)
        if tb > 0:
            u.prefill_compress(np64(Q[b, h, :, :nb]), np64(K[b, h, :tb]), np64(V[b, h, :tb]))
        units[b][h] = u
    return units


def make_cache(wl: synth.Workload, device="cuda:0"):
    from paper_2503_10714_amd.binding import Cache
    bp, bc, br = wl.budgets()
    return Cache(wl.n_layers, wl.n_seqs, wl.n_kv_heads, wl.q_per_kv, wl.head_dim, bp, bc, br, wl.dtype,
                 lam=wl.lam, alpha=wl.alpha, slot_capacity=wl.slot_capacity, device=device)


def check_every_unit(wl: synth.Workload, cache, steps_done: int, layers: Optional[Sequence[int]] = None) -> None:
    """Invariants of Alg. 1 that hold for EVERY unit at any size, checked on the device (torch ops on the
    exported metadata): tokens seen = prompt + steps; fusion counts sum to the tokens seen (B_r > 0); a slot is
    empty exactly where it has no position; token slots hold one token each, at distinct positions below the
    tokens seen, the latest B_p positions among them; the occupied token slots are min(T, B_p + B_c) many (what
    the kernels' own occupancy counter must say for them to take the right path); slots past B stay empty."""
    from paper_2503_10714_amd import binding as zb
    S, H, cap, Br = cache.S, cache.H, cache.cap, cache.B_r
    dev = cache.device
    bp, bc, _ = wl.budgets()
    lens = torch.tensor(wl.seq_lens(), dtype=torch.int64, device=dev)[:, None]            # [S,1]
    ntok = torch.tensor([p + c for p, c in zip(bp, bc)], dtype=torch.int64, device=dev)[:, None]
    bpt = torch.tensor(bp, dtype=torch.int64, device=dev)[:, None]
    pos = torch.empty(S, H, cap, dtype=torch.int32, device=dev)
    w = torch.empty(S, H, cap, dtype=torch.int32, device=dev)
    n_seen = torch.empty(S, H, dtype=torch.int64, device=dev)
    idx = torch.arange(cap, device=dev)[None, None, :]
    for l in (range(wl.n_layers) if layers is None else layers):
        with torch.cuda.device(dev):
            zb.zsm_cache_export(cache.handle, l, pos=pos, w=w, n_seen=n_seen)
        tag = f"{wl.name} layer {l} after {steps_done} steps"
        T = lens + steps_done
        assert bool((n_seen == T).all()), f"{tag}: tokens seen"
        occ = w > 0
        assert bool((occ == (pos >= 0)).all()), f"{tag}: empty slots and positions disagree"
        assert bool((pos.to(torch.int64) < T[:, :, None]).all()), f"{tag}: a position at or past the tokens seen"
        past = idx >= (ntok[:, :, None] + Br)
        assert bool((~occ | ~past).all()), f"{tag}: a slot past the budget is occupied"
        if Br > 0:
            assert bool((w.sum(-1, dtype=torch.int64) == T).all()), f"{tag}: fusion counts do not sum to the tokens seen"
        tw, tp = w[..., Br:], pos[..., Br:].to(torch.int64)
        assert bool((tw <= 1).all()), f"{tag}: a token slot with a fusion count above 1"
        n_occ = (tw > 0).sum(-1)
        assert bool((n_occ == torch.minimum(T, ntok)).all()), f"{tag}: occupied token slots"
        # distinct positions: empty slots get distinct negative stand-ins, then a sort must be strictly increasing
        key = torch.where(tw > 0, tp, -1 - torch.arange(cap - Br, device=dev)[None, None, :])
        srt = torch.sort(key, dim=-1).values
        assert bool((srt[..., 1:] > srt[..., :-1]).all()), f"{tag}: two token slots hold the same position"
        # the latest min(B_p, T) positions are all present (nothing inside the proximity window is ever evicted)
        n_recent = ((tw > 0) & (tp >= (T - bpt)[:, :, None])).sum(-1)
        assert bool((n_recent == torch.minimum(T, bpt)).all()), f"{tag}: a token of the latest B_p is missing"


def run_decode_parity(wl: synth.Workload, cache, units_by_layer: List[List[List[UnitCache]]], n_steps: int,
                      sel: Optional[Sequence[Tuple[int, int, int]]] = None, gen_device="cpu",
                      state_every: int = 0, first_step: int = 0, after_step=None) -> StepStats:
    """Lock-step decode of GPU cache and oracle units; all layers per launch.

    sel: (layer, b, h) triples to check (default: all).  state_every: also compare the
    whole exported state every that many steps (0 = only at the end).  first_step: number of the
    first decode step (its inputs are a function of the step number)."""
    L, S, H, G, d = wl.n_layers, wl.n_seqs, wl.n_kv_heads, wl.q_per_kv, wl.head_dim
    tol = tol_for(wl.dtype)
    stats = StepStats()
    triples = sel if sel is not None else [(l, b, h) for l in range(L) for b in range(S) for h in range(H)]
    dev = cache.device
    for step in range(first_step, first_step + n_steps):
        qs, ks, vs = [], [], []
        for l in range(L):
            q, k, v = synth.decode_inputs(wl, l, step, device=gen_device)
            qs.append(q); ks.append(k); vs.append(v)
        q = torch.stack(qs).to(dev); k = torch.stack(ks).to(dev); v = torch.stack(vs).to(dev)
        out, (ws, ep, ms) = cache.decode_step(q, k, v)
        out_c, ws_c, ep_c, ms_c = out.cpu().numpy().astype(np.float64), ws.cpu().numpy(), ep.cpu().numpy(), ms.cpu().numpy()
        qc, kc, vc = np64(q), np64(k), np64(v)
        resync_layers = set()
        for (l, b, h) in triples:
            u = units_by_layer[l][b][h]
            o, info = u.decode_step(qc[l, b, h], kc[l, b, h], vc[l, b, h])
            tag = f"{wl.name} step {step} unit(l={l},b={b},h={h})"
            if check_step(out_c[l, b, h], (int(ws_c[l, b, h]), int(ep_c[l, b, h]), int(ms_c[l, b, h])), o, info, u, tol, stats, tag):
                resync_layers.add(l)
        for l in resync_layers:
            assert sel is None, "a near tie in a sampled run cannot be re-synchronised"
            cache.import_layer(l, **pack_states(units_by_layer[l], cache.cap, cache.B_r, d, cache.kv_dtype))
        stats.steps += 1
        if after_step is not None:
            after_step(step + 1)
        if state_every and (step + 1) % state_every == 0 and step + 1 < first_step + n_steps:
            compare_all_state(wl, cache, units_by_layer, tol, f"after step {step}", sel)
    compare_all_state(wl, cache, units_by_layer, tol, "final", sel, stats)
    return stats


def compare_all_state(wl, cache, units_by_layer, tol, where, sel=None, stats: Optional[StepStats] = None):
    for l in range(wl.n_layers):
        pairs = None if sel is None else [(b, h) for (ll, b, h) in sel if ll == l]
        if pairs is not None and not pairs:
            continue
        st = cache.export_layer(l)
        compare_state(st, units_by_layer[l], cache.B_r, tol, f"{wl.name} {where} layer {l}", pairs)
        if stats is not None:
            g = st["s"].cpu().numpy()
            for (b, h) in (pairs if pairs is not None else [(b, h) for b in range(wl.n_seqs) for h in range(wl.n_kv_heads)]):
                u = units_by_layer[l][b][h]
                occ = u.w > 0
                stats.s_total += int(occ.sum())
                stats.s_bit_equal += int((g[b, h, :u.B][occ] == u.s[occ].astype(np.float32)).sum())


# ---------------------------------------------------------------------------------------
# every unit of a layer at once, against the plain-C oracle (oracle/zsmerge_oracle_c.c)
# ---------------------------------------------------------------------------------------

def new_c_oracle_layer(wl: synth.Workload):
    """The C oracle's state for the S x H units of one layer, unit (b, h) at index b * H + h."""
    from oracle import zsmerge_oracle_c as oc
    bp, bc, br = wl.budgets()
    H = wl.n_kv_heads
    return oc.BatchCache(wl.n_seqs * H, wl.head_dim, wl.q_per_kv, np.repeat(bp, H), np.repeat(bc, H), br,
                         lam=lam32(wl.lam), alpha=lam32(wl.alpha), cap=wl.slot_capacity)


def c_oracle_prefill_layer(wl: synth.Workload, Q, K, V, lens: Sequence[int]):
    """C-oracle prefill of every unit of one layer from the tensors the device got.
    Returns (state, prompt scores [S*H, T_max])."""
    S, H, T_max, d = K.shape
    W = Q.shape[3]
    assert min(lens) >= W, "the batched oracle call takes one window length for all units"
    cb = new_c_oracle_layer(wl)
    s = cb.prefill_compress(np64(Q).reshape(S * H, wl.q_per_kv, W, d), np64(K).reshape(S * H, T_max, d),
                            np64(V).reshape(S * H, T_max, d), np.repeat(np.asarray(lens), H))
    return cb, s


def pack_c_state(cb, S: int, H: int, kv_dtype: torch.dtype) -> Dict[str, torch.Tensor]:
    """C-oracle state of one layer -> the import arrays (CPU tensors)."""
    Br, cap, d = cb.B_r, cb.cap, cb.d
    t = lambda a, *shape: torch.from_numpy(np.ascontiguousarray(a)).reshape(S, H, *shape)
    return dict(K=t(cb.K[:, Br:], cap - Br, d).to(torch.float32).to(kv_dtype), V=t(cb.V[:, Br:], cap - Br, d).to(torch.float32).to(kv_dtype),
                Kr=t(cb.K[:, :Br], Br, d).to(torch.float32), Vr=t(cb.V[:, :Br], Br, d).to(torch.float32),
                s=t(cb.s, cap).to(torch.float32), pos=t(cb.pos, cap).to(torch.int32), w=t(cb.w, cap).to(torch.int32),
                n_seen=t(cb.n_seen))


def compare_layer_with_c_oracle(gpu: Dict[str, torch.Tensor], cb, tol: float, where: str,
                                stats: Optional[StepStats] = None, prompt_scores: Optional[np.ndarray] = None) -> List[int]:
    """Exported device state of one layer against the C oracle's, every unit: integers and token rows exact, residual
    rows and scores within tol.  With `prompt_scores` (right after the prefill) a unit may hold other tokens than the
    oracle's where the oracle's own scores of the tokens in question lie within TIE_REL of its selection boundary;
    the indices of such units are returned (the caller brings the two sides together again)."""
    n, cap, Br, d = cb.n, cb.cap, cb.B_r, cb.d
    g = {k: v.cpu() for k, v in gpu.items()}
    gp = g["pos"].reshape(n, cap).numpy().astype(np.int64)
    gw = g["w"].reshape(n, cap).numpy().astype(np.int64)
    gs = np64(g["s"]).reshape(n, cap)
    assert (g["n_seen"].reshape(n).numpy() == cb.n_seen).all(), f"{where}: tokens seen differ"
    occ = cb.w > 0
    same = (gw == cb.w).all(axis=1) & ((gp == cb.pos) | ~occ).all(axis=1)
    flipped = []
    for u in np.flatnonzero(~same):
        assert prompt_scores is not None, f"{where} unit {u}: slots differ at {np.flatnonzero((gw[u] != cb.w[u]) | ((gp[u] != cb.pos[u]) & occ[u]))[:8]}"
        B = Br + int(cb.B_p[u] + cb.B_c[u])
        dev_set = set(gp[u, Br:B][gw[u, Br:B] > 0].tolist())
        or_set = set(cb.pos[u, Br:B][occ[u, Br:B]].tolist())
        T = int(cb.n_seen[u])
        ctx = [t for t in or_set if t < T - int(cb.B_p[u])]
        s_b = min(prompt_scores[u, t] for t in ctx)             # lowest score the oracle kept
        for t in dev_set ^ or_set:
            rel = abs(prompt_scores[u, t] - s_b) / max(abs(s_b), 1e-300)
            assert rel < TIE_REL, f"{where} unit {u}: position {t} (s={prompt_scores[u, t]:.9e}) kept by one side only, boundary score {s_b:.9e}, rel gap {rel:.2e}"
        assert len(dev_set) == len(or_set), f"{where} unit {u}: {len(dev_set)} tokens kept, oracle {len(or_set)}"
        flipped.append(int(u))
    ok = same
    tokocc = occ[:, Br:] & ok[:, None]
    gK = np64(g["K"]).reshape(n, cap - Br, d)
    assert (gK[tokocc] == cb.K[:, Br:][tokocc]).all(), f"{where}: token K rows differ"
    del gK
    gV = np64(g["V"]).reshape(n, cap - Br, d)
    assert (gV[tokocc] == cb.V[:, Br:][tokocc]).all(), f"{where}: token V rows differ"
    del gV
    if Br:
        ro = occ[:, :Br] & ok[:, None]
        dk = np.abs(np64(g["Kr"]).reshape(n, Br, d) - cb.K[:, :Br])[ro]
        dv = np.abs(np64(g["Vr"]).reshape(n, Br, d) - cb.V[:, :Br])[ro]
        if dk.size:
            assert dk.max() <= tol and dv.max() <= tol, f"{where}: residual K/V off by {dk.max():.3e}/{dv.max():.3e}"
    m = occ & ok[:, None]
    ds = np.abs(gs - cb.s)[m]
    if ds.size:
        assert ds.max() <= tol, f"{where}: scores off by {ds.max():.3e}"
    if stats is not None:
        stats.s_total += int(m.sum())
        stats.s_bit_equal += int((gs[m].astype(np.float32) == cb.s[m].astype(np.float32)).sum())
    return flipped


def decode_step_with_c_oracle(wl: synth.Workload, cache, cbs, step: int, stats: StepStats, gen_device="cpu") -> None:
    """One decode step of every unit of every layer on the device (one launch) and in the C oracle; outputs within
    tolerance, decisions equal for every unit (or, inside the near-tie band of the oracle's own scores, brought
    together again by handing the oracle's state of that layer to the device)."""
    L, S, H, G, d = wl.n_layers, wl.n_seqs, wl.n_kv_heads, wl.q_per_kv, wl.head_dim
    n = S * H
    tol = tol_for(wl.dtype)
    dev = cache.device
    qs, ks, vs = [], [], []
    for l in range(L):
        q, k, v = synth.decode_inputs(wl, l, step, device=gen_device)
        qs.append(q); ks.append(k); vs.append(v)
    q = torch.stack(qs).to(dev); k = torch.stack(ks).to(dev); v = torch.stack(vs).to(dev)
    out, (ws, ep, ms) = cache.decode_step(q, k, v)
    out_c = out.cpu().numpy().astype(np.float64).reshape(L, n, G, d)
    ws_c, ep_c, ms_c = (x.cpu().numpy().reshape(L, n) for x in (ws, ep, ms))
    qc, kc, vc = np64(q).reshape(L, n, G, d), np64(k).reshape(L, n, d), np64(v).reshape(L, n, d)
    for l in range(L):
        o, ws_o, ev_o, mg_o, _, cand, cand_s, cand_pos = cbs[l].decode_step(qc[l], kc[l], vc[l], debug=True)
        err = float(np.abs(out_c[l] - o).max())
        stats.max_out_err = max(stats.max_out_err, err)
        assert err <= tol, f"{wl.name} step {step} layer {l}: attention output off by {err:.3e} (tol {tol})"
        stats.unit_steps += n
        stats.evictions += int((ev_o >= 0).sum())
        stats.merges += int((mg_o >= 0).sum())
        same = (ep_c[l] == ev_o) & (ws_c[l] == ws_o)
        assert (ms_c[l][same] == mg_o[same]).all(), f"{wl.name} step {step} layer {l}: merged slots differ"
        for u in np.flatnonzero(~same):
            tag = f"{wl.name} step {step} layer {l} unit {u}"
            ep_d = int(ep_c[l, u])
            assert ev_o[u] >= 0 and ep_d >= 0, f"{tag}: write_slot/evicted_pos {ws_c[l, u]}/{ep_d} vs {ws_o[u]}/{ev_o[u]}"
            cp = cand_pos[u, :cand[u, 0]].tolist()
            assert ep_d in cp, f"{tag}: device evicted position {ep_d}, which is not a candidate"
            s_dev, s_best = float(cand_s[u, cp.index(ep_d)]), float(cand_s[u, cp.index(int(ev_o[u]))])
            rel = abs(s_dev - s_best) / max(abs(s_best), 1e-300)
            assert rel < TIE_REL, f"{tag}: device evicted pos {ep_d} (s={s_dev:.9e}) but the lowest score is pos {ev_o[u]} (s={s_best:.9e}), rel gap {rel:.2e}"
            stats.near_ties += 1
        if not same.all():
            cache.import_layer(l, **pack_c_state(cbs[l], S, H, cache.kv_dtype))
    stats.steps += 1
