"""Numerical-error sweep: eviction versus residual merging at several cache budgets.

Re-runs the experiment of the paper's "Numerical Error Analysis" (the log-scale figure that
compares pure eviction with residual merging) on the seeded synthetic workload: for a cache
budget of 50 / 20 / 10 / 5 % of the prompt, the relative error of the attention output of
the budgeted cache against full attention over the whole history, once with B_r = 0 (pure
eviction, Sec. 3.2) and once with B_r = 1 (residual merging, Eq. 5-6, compensated by Eq. 4).
The paper's inputs are not specified, so its magnitudes cannot be matched; what carries over
is the sign: merging has the lower error.

The budgeted path runs through the C ABI (prefill compression + decode steps).  The full
attention it is compared with is evaluation code (torch, fp64), not part of the product.

The same harness sweeps the compensation weight alpha of Eq. 4 (the paper's hyper-parameter
study varies it between 0, the eviction-like end, and 1, the value it fixes).

    python -m paper_2503_10714_amd.error_sweep [--prompt 4096] [--steps 128] [--heads 32] [--alphas 0,0.5,1]
"""
from __future__ import annotations

import argparse
import json
import math

import torch

from . import synth
from . import binding as zb


def full_attention(q: torch.Tensor, K: torch.Tensor, V: torch.Tensor) -> torch.Tensor:
    """Eq. 1 for every (head, query head): q [H, G, d], K/V [H, n, d] -> [H, G, d] (fp64)."""
    d = q.shape[-1]
    z = torch.einsum("hgd,hnd->hgn", q.double(), K.double()) / math.sqrt(d)
    return torch.einsum("hgn,hnd->hgd", torch.softmax(z, dim=-1), V.double())


def run_policy(wl: synth.Workload, device="cuda:0"):
    """Prefill + decode of one workload (one layer, one sequence); returns the relative error
    ||o_budgeted - o_full|| / ||o_full|| per (step, head, query head) as a tensor."""
    assert wl.n_layers == 1 and wl.n_seqs == 1
    bp, bc, br = wl.budgets()
    cache = zb.Cache(1, 1, wl.n_kv_heads, wl.q_per_kv, wl.head_dim, bp, bc, br, wl.dtype, lam=wl.lam,
                     alpha=wl.alpha, slot_capacity=wl.slot_capacity, device=device)
    Q, K, V, lens = synth.prompt(wl, 0, device=device)
    cache.prefill_compress(0, Q, K, V, lens)
    hist_k, hist_v = [K[0]], [V[0]]
    errs = []
    for step in range(wl.decode_steps):
        q, k, v = synth.decode_inputs(wl, 0, step, device=device)
        out, _ = cache.decode_step(q[None], k[None], v[None], info=False)
        hist_k.append(k[0][:, None]); hist_v.append(v[0][:, None])
        ref = full_attention(q[0], torch.cat(hist_k, 1), torch.cat(hist_v, 1))
        o = out[0, 0].double()
        errs.append(torch.linalg.vector_norm(o - ref, dim=-1) / torch.linalg.vector_norm(ref, dim=-1))
    cache.close()
    return torch.stack(errs)


def sweep(prompt=4096, steps=128, heads=32, ratios=(0.5, 0.2, 0.1, 0.05), dtype="f16", device="cuda:0"):
    rows = []
    for rho in ratios:
        B = int(math.ceil(rho * prompt))
        res = {}
        for name, br in (("evict", 0), ("merge", 1)):
            wl = synth.Workload(f"err-{name}-{rho}", 1, 1, heads, 1, 128, dtype, prompt, B, steps, 32, True, n_residual=br)
            res[name] = float(run_policy(wl, device).mean())
        rows.append({"budget_ratio": rho, "B": B, "rel_err_evict": res["evict"], "rel_err_merge": res["merge"],
                     "reduction": 1.0 - res["merge"] / res["evict"]})
    return rows


def alpha_sweep(prompt=4096, steps=128, heads=32, ratio=0.05, alphas=(0.0, 0.25, 0.5, 0.75, 1.0), dtype="f16",
                device="cuda:0"):
    """Residual merging (B_r = 1) at one budget for several alpha of Eq. 4: mean relative output error."""
    B = int(math.ceil(ratio * prompt))
    rows = []
    for al in alphas:
        wl = synth.Workload(f"err-alpha-{al}", 1, 1, heads, 1, 128, dtype, prompt, B, steps, 32, True, n_residual=1, alpha=al)
        rows.append({"budget_ratio": ratio, "B": B, "alpha": al, "rel_err_merge": float(run_policy(wl, device).mean())})
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--prompt", type=int, default=4096)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--heads", type=int, default=32)
    ap.add_argument("--alphas", type=str, default="", help="comma-separated alpha values: also sweep Eq. 4's alpha at a 5 % budget")
    args = ap.parse_args()
    for r in sweep(args.prompt, args.steps, args.heads):
        print(json.dumps(r))
    if args.alphas:
        for r in alpha_sweep(args.prompt, args.steps, args.heads, alphas=tuple(float(x) for x in args.alphas.split(","))):
            print(json.dumps(r))


if __name__ == "__main__":
    main()
