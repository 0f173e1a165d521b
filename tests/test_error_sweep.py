"""Eviction versus residual merging: relative error of the attention output against full
attention (the paper's numerical error analysis), on the device path and in the oracle."""
import math

import numpy as np
import pytest
import torch

from oracle.zsmerge_oracle import UnitCache, full_attention_row
from paper_2503_10714_amd import synth
from tests import parity_util as pu


def oracle_errors(wl):
    """Per (step, head) relative error of the oracle's budgeted output against Eq. 1 over the
    whole history, for a one-layer, one-sequence workload with G = 1."""
    Q, K, V, lens = synth.prompt(wl, 0)
    units = pu.oracle_prefill_layer(wl, Q, K, V, lens)
    Kh = [pu.np64(K[0, h]) for h in range(wl.n_kv_heads)]
    Vh = [pu.np64(V[0, h]) for h in range(wl.n_kv_heads)]
    errs = np.zeros((wl.decode_steps, wl.n_kv_heads))
    for step in range(wl.decode_steps):
        q, k, v = synth.decode_inputs(wl, 0, step)
        q, k, v = pu.np64(q), pu.np64(k), pu.np64(v)
        for h in range(wl.n_kv_heads):
            o, _ = units[0][h].decode_step(q[0, h], k[0, h], v[0, h])
            Kh[h] = np.vstack([Kh[h], k[0, h]]); Vh[h] = np.vstack([Vh[h], v[0, h]])
            ref, _ = full_attention_row(q[0, h, 0], Kh[h], Vh[h], 1 / math.sqrt(wl.head_dim))
            errs[step, h] = np.linalg.norm(o[0] - ref) / np.linalg.norm(ref)
    return errs


def policy(name, br, prompt, B, steps, heads):
    return synth.Workload(f"err-{name}", 1, 1, heads, 1, 128, "f16", prompt, B, steps, 32, True, n_residual=br)


def test_oracle_merging_beats_eviction_on_skewed_data():
    """Soft check of the figure's sign: at a tight budget the residual slot lowers the mean error."""
    ev = oracle_errors(policy("evict", 0, 600, 30, 40, 3)).mean()
    mg = oracle_errors(policy("merge", 1, 600, 30, 40, 3)).mean()
    assert mg < ev, (mg, ev)


@pytest.mark.gpu
def test_device_error_sweep_matches_oracle_and_trend():
    from paper_2503_10714_amd import error_sweep as es
    for name, br in (("evict", 0), ("merge", 1)):
        wl = policy(name, br, 512, 26, 32, 4)
        dev = es.run_policy(wl)[:, :, 0].cpu().numpy()
        ora = oracle_errors(wl)
        assert np.abs(dev - ora).max() < 1e-4, (name, np.abs(dev - ora).max())
    rows = es.sweep(prompt=2048, steps=64, heads=8, ratios=(0.2, 0.05))
    print(rows, flush=True)
    for r in rows:
        assert r["rel_err_merge"] < r["rel_err_evict"], r


@pytest.mark.gpu
def test_device_alpha_sweep_matches_oracle():
    """Eq. 4's alpha on the device path against the oracle, at the two ends and in the middle."""
    from paper_2503_10714_amd import error_sweep as es
    for al in (0.0, 0.5, 1.0):
        wl = synth.Workload(f"err-alpha-{al}", 1, 1, 3, 1, 128, "f16", 400, 20, 24, 32, True, n_residual=1, alpha=al)
        dev = es.run_policy(wl)[:, :, 0].cpu().numpy()
        ora = oracle_errors(wl)
        assert np.abs(dev - ora).max() < 1e-4, (al, np.abs(dev - ora).max())
