#!/usr/bin/env python3
"""Benchmark of the ZSMerge budgeted KV-cache step on one MI355X.

Workload (the benchmark definition's headline one): Llama2-7B shape, 32 layers x 32 KV heads
= 1024 units, head_dim 128, fp16, a 54 000-token prompt compressed per head to 5 %
(B = 2700 slots), then decode steps.  A "step" is one fused decode step of all 1024 units
(all layers in one launch).  The prefill compression of the 32 layers runs on the device
before the timed region and is reported beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 2] [--no-cpu-baseline]

Prints one JSON line (rank 0).  Inputs are seeded synthetic data generated on the device
before the timed region; everything the timed region reads is already resident in HBM.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published peak


def algorithmic_bytes_per_unit_step(B_tok: int, B_r: int, d: int, e: int, G: int) -> int:
    """HBM bytes one unit must move in one decode step when every byte moves once.

    token K and V rows once; residual K and V rows (fp32) once; per slot: score read + score
    write + position read (12 B); q, k_new, v_new in; out (fp32) out; the evicted row re-read
    and the incoming row written (K and V each); the merged residual row written back;
    a few header words.
    """
    B = B_tok + B_r
    kv = 2 * B_tok * d * e + 2 * B_r * d * 4
    meta = 12 * B
    io = (G + 2) * d * e + 4 * G * d
    evict = 2 * d * e + 2 * d * e + 2 * d * 4
    return kv + meta + io + evict + 40


def read_traffic_from_profiles(name: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), as recorded
    in profiles/<name>.  Returns None when no such summary has been committed."""
    p = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(p):
        return None
    m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(p).read())
    return float(m.group(1)) if m else None


def device_info():
    """Name, compute units and (from the driver's sysfs files, when readable) performance level and
    memory clock.  Files only: a process that has touched the GPU starts no other program."""
    import glob
    import torch
    p = torch.cuda.get_device_properties(0)
    info = {"name": p.name, "compute_units": p.multi_processor_count, "memory_GiB": round(p.total_memory / 2 ** 30, 1)}
    for dev in sorted(glob.glob("/sys/class/drm/card[0-9]*/device")):
        try:
            level = open(os.path.join(dev, "power_dpm_force_performance_level")).read().strip()
            mclk = open(os.path.join(dev, "pp_dpm_mclk")).read()
        except OSError:
            continue
        info["perf_level"] = level
        m = re.search(r"(\d+)\s*Mhz\s*\*", mclk, re.I)
        if m:
            info["mclk_MHz"] = int(m.group(1))
        break
    return info


def cpu_baseline(wl, n_units: int, n_steps: int, numpy_units: int = 2, numpy_steps: int = 16):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: `n_units` units (layer 0,
    heads 0..) through their own prefill, then `n_steps` timed decode steps in the plain-C oracle (one OpenMP
    thread per unit).  The NumPy oracle is timed beside it on a smaller sample."""
    import numpy as np
    import torch
    from oracle import zsmerge_oracle_c as oc
    from oracle.zsmerge_oracle import UnitCache
    from paper_2503_10714_amd import synth
    sub = wl.sliced(n_layers=1, n_kv_heads=n_units)
    dev = "cuda:0" if torch.cuda.is_available() else "cpu"
    Q, K, V, lens = synth.prompt(sub, 0, device=dev)
    f = lambda t: t.detach().to("cpu").to(torch.float64).numpy()
    bp, bc, br = sub.budgets()
    lam, alpha = float(np.float32(sub.lam)), float(np.float32(sub.alpha))
    T0, G, d = lens[0], sub.q_per_kv, sub.head_dim
    q, k, v = synth.decode_inputs_uniform(sub, [0], list(range(n_steps)), device=dev)
    q, k, v = f(q), f(k), f(v)

    cb = oc.BatchCache(n_units, d, G, bp[0], bc[0], br, lam=lam, alpha=alpha)
    t0 = time.perf_counter()
    cb.prefill_compress(f(Q[0]), f(K[0, :, :T0]), f(V[0, :, :T0]))
    t_prefill = time.perf_counter() - t0
    t0 = time.perf_counter()
    for s in range(n_steps):
        cb.decode_step(q[s, 0, 0], k[s, 0, 0], v[s, 0, 0])
    t_decode = time.perf_counter() - t0

    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    except Exception:
        blas_threads = 1
    units = []
    for h in range(numpy_units):
        u = UnitCache(d, G, bp[0], bc[0], br, lam=lam, alpha=alpha)
        u.prefill_compress(f(Q[0, h]), f(K[0, h, :T0]), f(V[0, h, :T0]))
        units.append(u)
    t0 = time.perf_counter()
    for s in range(numpy_steps):
        for h, u in enumerate(units):
            u.decode_step(q[s, 0, 0, h], k[s, 0, 0, h], v[s, 0, 0, h])
    t_numpy = time.perf_counter() - t0
    return {
        "value": n_units * n_steps / t_decode, "unit": "unit-steps/s", "cores": int(min(oc.threads(), n_units)), "kind": "oracle",
        "host_cores": os.cpu_count(),
        "threads_note": "cores = OpenMP threads of the C oracle that had a unit to work on; host_cores = os.cpu_count()",
        "sample": f"{n_units} units of layer 0 (T={T0}, B={sub.slot_capacity}) x {n_steps} decode steps, plain C fp64 "
                  f"(oracle/zsmerge_oracle_c.c, gcc -O2 -fopenmp); their oracle prefill took {t_prefill / n_units:.2f} s per unit "
                  f"(not in value)",
        "numpy_oracle": {"value": numpy_units * numpy_steps / t_numpy, "unit": "unit-steps/s", "cores": int(blas_threads),
                         "sample": f"{numpy_units} of the same units x {numpy_steps} steps, NumPy fp64 (oracle/zsmerge_oracle.py)"},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=512)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-units", type=int, default=32,
                    help="units of layer 0 the CPU oracle is timed on (32 = one full layer of workload 2; with the default steps about 10 s of CPU work)")
    ap.add_argument("--cpu-steps", type=int, default=8192)
    ap.add_argument("--layers-per-launch", type=int, default=0,
                    help="0 = all layers of the workload in one launch (the headline configuration); N = one launch "
                         "per N layers, as a model that runs its layers one after the other would call it")
    ap.add_argument("--graph", action="store_true",
                    help="capture the launches of one step in a HIP graph (inputs in fixed buffers, refreshed by three small "
                         "copies before every replay) and time replays instead of eager calls: what a serving loop that runs "
                         "its layers one call each would do (use with --layers-per-launch 1)")
    ap.add_argument("--decode-parts", type=int, default=0,
                    help="workgroups per unit in the decode step: 0 = the library's choice per launch, 1 = never split, n = n")
    ap.add_argument("--window", type=int, default=None,
                    help="override the number of prompt queries W the prefill scores from (0 = every prompt query: "
                         "the full-history initialisation)")
    ap.add_argument("--n-residual", type=int, default=None,
                    help="override the workload's number of residual slots B_r (B stays the same, B_c shrinks)")
    ap.add_argument("--settle-seconds", type=float, default=5.0,
                    help="idle time between the set-up and the warm-up steps.  Generating 28 GB of synthetic prompts in fp64 "
                         "and scoring them leaves the chip, for a second or two, in a state in which every kernel (the plain "
                         "streaming read included) runs about 4 %% slower; a decode that has been running for a few seconds "
                         "is not in that state (16 384 steps right after the set-up average what 512 steps do after this "
                         "pause).  0 = start at once")
    ap.add_argument("--budget", type=int, default=None,
                    help="override the workload's budget B (slots per unit at the full prompt length)")
    ap.add_argument("--q-per-kv", type=int, default=None,
                    help="override the workload's number of query heads per KV head G (same KV heads, G times the queries)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="after the run, copy a 1 GiB buffer three times with the library's plain copy kernel, so that "
                         "a counter run holds dispatches of known size to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--prefill-layers-per-call", type=int, default=0,
                    help="layers compressed by one zsm_prefill_compress call; the prompts of that many layers are resident "
                         "at once.  0 = as many as keep them under 64 GiB (a call of many layers has no launch gaps between "
                         "its layers' kernels, and the sequential absorption of several residual slots, one wave per unit, "
                         "needs the units of many layers to fill the chip)")
    ap.add_argument("--skip-prefill", action="store_true",
                    help="fill the cache by import of synthetic rows instead of running the prefill (profiling runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (units are independent and would shard with no "
              "exchange; no multi-GPU path is built). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2503_10714_amd import synth
    from paper_2503_10714_amd import binding as zb

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    zb.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = synth.workload(args.workload)
    if args.n_residual is not None:
        wl = wl.sliced(n_residual=args.n_residual)
    if args.window is not None:
        wl = wl.sliced(window=args.window)
    if args.q_per_kv is not None:
        wl = wl.sliced(q_per_kv=args.q_per_kv)
    if args.budget is not None:
        wl = wl.sliced(budget=args.budget)
    if wl.ragged is not None and not args.skip_prefill:
        print("bench.py: a ragged workload is a parity-test case; its decode step can be timed with --skip-prefill "
              "(slots filled by import, inputs of all sequences drawn at the same positions)", file=sys.stderr)
        sys.exit(2)
    L, S, H, G, d = wl.n_layers, wl.n_seqs, wl.n_kv_heads, wl.q_per_kv, wl.head_dim
    bp, bc, br = wl.budgets()
    cache = zb.Cache(L, S, H, G, d, bp, bc, br, wl.dtype, lam=wl.lam, alpha=wl.alpha, slot_capacity=wl.slot_capacity, device=dev)
    e = 4 if wl.dtype == "f32" else 2

    # ---- prefill compression of every layer (device-generated prompts) -------------------
    prefill_ms = None
    t_setup = time.perf_counter()
    if not args.skip_prefill:
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        tot = 0.0
        # untimed warm-up: one head of one layer through the same kernels (their code is loaded on first use)
        w1 = wl.sliced(n_layers=1, n_kv_heads=1)
        c1 = zb.Cache(1, S, 1, G, d, bp, bc, br, wl.dtype, lam=wl.lam, alpha=wl.alpha, slot_capacity=wl.slot_capacity, device=dev)
        q1, k1, v1, lens1 = synth.prompt(w1, 0, device=dev)
        c1.prefill_compress(0, q1, k1, v1, lens1)
        torch.cuda.synchronize()
        c1.close()
        del q1, k1, v1, c1
        # default: as many layers per call as keep the resident prompts (K and V) under 64 GiB
        per_layer = 2 * S * H * max(wl.seq_lens()) * d * e
        plc = args.prefill_layers_per_call if args.prefill_layers_per_call > 0 else max(1, min(L, (64 << 30) // per_layer))
        for l0 in range(0, L, plc):
            l1 = min(L, l0 + plc)
            Q = K = V = None
            for l in range(l0, l1):
                q1, k1, v1, lens = synth.prompt(wl, l, device=dev)
                if Q is None:
                    Q = torch.empty((l1 - l0,) + tuple(q1.shape), dtype=q1.dtype, device=dev)
                    K = torch.empty((l1 - l0,) + tuple(k1.shape), dtype=k1.dtype, device=dev)
                    V = torch.empty_like(K)
                Q[l - l0].copy_(q1); K[l - l0].copy_(k1); V[l - l0].copy_(v1)
                del q1, k1, v1
            lens_t = torch.tensor(lens, dtype=torch.int32, device=dev)
            cache.reserve_workspace(l1 - l0, K.shape[-2], Q.shape[-2])      # the allocation is not the library's work
            torch.cuda.synchronize()
            ev0.record()
            cache.prefill_compress(l0, Q, K, V, lens_t, layer_end=l1)
            ev1.record()
            torch.cuda.synchronize()
            tot += ev0.elapsed_time(ev1)
            del Q, K, V
        prefill_ms = tot
        cache.release_workspace()
    else:
        # every slot filled with synthetic rows: the decode kernel's traffic does not depend on how
        # (a sequence with a smaller budget fills its own B_p + B_c token slots; the rest stay empty)
        n = wl.slot_capacity - br
        ntok_b = torch.tensor([p + c for p, c in zip(bp, bc)], dtype=torch.int32, device=dev)
        occ = torch.arange(n, dtype=torch.int32, device=dev)[None, :] < ntok_b[:, None]          # [S, n]
        lens_b = torch.tensor(wl.seq_lens(), dtype=torch.int64, device=dev)
        for l in range(L):
            K, V = synth.kv_rows(wl, l, torch.arange(n), device=dev)
            pos = torch.full((S, H, wl.slot_capacity), -1, dtype=torch.int32, device=dev)
            pos_tok = (lens_b[:, None] - ntok_b[:, None] + torch.arange(n, device=dev)[None, :]).to(torch.int32)   # latest tokens
            pos[..., br:] = torch.where(occ, pos_tok, torch.full_like(pos_tok, -1))[:, None, :]
            w = torch.zeros(S, H, wl.slot_capacity, dtype=torch.int32, device=dev)
            w[..., br:] = occ[:, None, :].to(torch.int32)
            s = torch.rand(S, H, wl.slot_capacity, device=dev) * 0.01
            cache.import_layer(l, K=K, V=V, s=s, pos=pos, w=w, n_seen=lens_b[:, None].expand(S, H).contiguous())
            del K, V
    torch.cuda.empty_cache()

    # ---- decode inputs for all steps, resident before the timed region -------------------
    n_total = args.warmup + args.steps
    q_all, k_all, v_all = synth.decode_inputs_uniform(wl.sliced(ragged=None), list(range(L)), list(range(n_total)), device=dev)
    out = torch.empty(L, S, H, G, d, dtype=torch.float32, device=dev)
    info = tuple(torch.empty(L, S, H, dtype=torch.int32, device=dev) for _ in range(3))
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t_setup
    if args.settle_seconds > 0:
        time.sleep(args.settle_seconds)

    lpl = args.layers_per_launch if args.layers_per_launch > 0 else L
    cache.set_decode_parts(args.decode_parts)
    parts = cache.decode_parts(0, lpl)

    def step(i):
        for l0 in range(0, L, lpl):
            l1 = min(L, l0 + lpl)
            zb.zsm_decode_step(cache.handle, l0, l1, q_all[i, l0:l1], k_all[i, l0:l1], v_all[i, l0:l1], out[l0:l1],
                               info[0][l0:l1], info[1][l0:l1], info[2][l0:l1])

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    if args.graph:
        q_cur, k_cur, v_cur = q_all[0].clone(), k_all[0].clone(), v_all[0].clone()

        def launches():
            for l0 in range(0, L, lpl):
                l1 = min(L, l0 + lpl)
                zb.zsm_decode_step(cache.handle, l0, l1, q_cur[l0:l1], k_cur[l0:l1], v_cur[l0:l1], out[l0:l1],
                                   info[0][l0:l1], info[1][l0:l1], info[2][l0:l1])

        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):      # records the launches; nothing runs and the cache is not touched
            launches()

        def step(i):
            q_cur.copy_(q_all[i]); k_cur.copy_(k_all[i]); v_cur.copy_(v_all[i])
            graph.replay()

        for i in range(min(5, args.warmup)):
            step(i)
        torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(args.steps):
        step(args.warmup + i)
        evs[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gpu_ms = evs[0].elapsed_time(evs[-1])
    per = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps))
    ms_per_step = wall * 1e3 / args.steps
    kernel_ms = gpu_ms / args.steps / ((L + lpl - 1) // lpl)   # average launch duration over the timed region (HIP events)
    units = wl.n_units
    value = units * args.steps / wall

    bytes_step = sum(algorithmic_bytes_per_unit_step(p + c, br, d, e, G) for p, c in zip(bp, bc)) * L * H   # all units
    bytes_launch = bytes_step / ((L + lpl - 1) // lpl)
    achieved = bytes_launch / (kernel_ms * 1e-3) / 1e9
    traffic = read_traffic_from_profiles(f"decode_step_cfg{args.workload}_pmc.md")

    # achievable read rate on this machine: plain streaming read of the cache buffer
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    nb = (cache.buf.numel() // 16) * 16
    for _ in range(3):
        zb.zsm_stream_read(cache.buf[:nb], sink)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(10):
        zb.zsm_stream_read(cache.buf[:nb], sink)
    b.record()
    torch.cuda.synchronize()
    read_ceiling = nb * 10 / (a.elapsed_time(b) * 1e-3) / 1e9

    res = {
        "metric": "decode unit-steps/s (layer x head x batch units per second, fused ZSMerge decode step)",
        "value": value, "unit": "unit-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"cfg{args.workload} {wl.name}: {L} layers x {S} seq x {H} KV heads = {units} units, G={G}, d={d}, "
                               f"{wl.dtype} KV, prompt {wl.prompt_len} tokens -> B={wl.slot_capacity} slots "
                               + (f"(B_p={bp[0]}, B_c={bc[0]}, B_r={br}), " if wl.ragged is None else
                                  f"at most (prompts of {min(wl.seq_lens())}..{max(wl.seq_lens())} tokens, B = {min(p + c for p, c in zip(bp, bc)) + br}.."
                                  f"{max(p + c for p, c in zip(bp, bc)) + br} per sequence, B_r={br}), ")
                               + ("all layers in one launch" if lpl >= L else f"{lpl} layer(s) per launch")
                               + (f", {parts} workgroups per unit" if parts > 1 else ", one workgroup per unit")
                               + (", replayed from a HIP graph" if args.graph else ""),
                   "units": units, "slots_per_unit": wl.slot_capacity},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic,
                     "traffic_source": (f"profiles/decode_step_cfg{args.workload}_pmc.md: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                        "command, scaled by a copy kernel of known size; read from that file, not measured in this run"
                                        if traffic is not None else None),
                     "kernel": "zsm::decode_kernel", "kernel_ms": kernel_ms,
                     "algorithmic_bytes_per_launch": bytes_launch},
        "step_ms_p10_p50_p90": [per[len(per) // 10], per[len(per) // 2], per[(9 * len(per)) // 10]],
        "tokens_per_s_cache_step_only": value / (L * H) if S == 1 else None,
        "hbm_read_ceiling_GBs": read_ceiling,
        "prefill_compress_ms_all_layers": prefill_ms,
        "prefill_layers_per_call": (None if args.skip_prefill else plc), "settle_seconds": args.settle_seconds,
        "prefill_window": (wl.window if wl.window > 0 else wl.prompt_len),
        "setup_s": setup_s,
        "device": device_info(),
    }
    if args.pmc_calibration:
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            zb.zsm_stream_copy(dst, src)
        torch.cuda.synchronize()
        res["pmc_calibration"] = {"kernel": "stream_copy_kernel", "bytes_read": 1 << 30, "bytes_written": 1 << 30, "launches": 3}
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl, args.cpu_units, args.cpu_steps)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
