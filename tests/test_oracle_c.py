"""The plain-C oracle against the NumPy oracle on random workloads (CPU only).

The pins of tests/test_oracle_pins.py already run against both; this file adds what only the
batched C interface has (many units at once, one budget per unit, ragged prompt lengths, the
slot stride) and long random walks where the two must take the same decisions step by step.
Decisions are compared exactly, stored fp32 values bit for bit except where a value sits within
an fp64 rounding of an fp32 rounding boundary (allowed: one unit in the last place, counted).
"""
import numpy as np
import pytest

from oracle import zsmerge_oracle as opy
from oracle import zsmerge_oracle_c as oc


def f32(x):
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


def make_inputs(seed, n, G, d, T_max, n_steps):
    rng = np.random.default_rng(seed)
    u = rng.standard_normal(d); u /= np.linalg.norm(u)
    K = rng.standard_normal((n, T_max, d)); V = rng.standard_normal((n, T_max, d))
    K[rng.random((n, T_max)) < 0.1] += 2.5 * d ** 0.25 * u
    Q = rng.standard_normal((n, G, T_max, d)) + d ** 0.25 * u
    dq = rng.standard_normal((n_steps, n, G, d)) + d ** 0.25 * u
    dk = rng.standard_normal((n_steps, n, d)); dv = rng.standard_normal((n_steps, n, d))
    return tuple(f32(x) for x in (Q, K, V, dq, dk, dv))


def ulp_close(a, b):
    """equal, or one fp32 unit in the last place apart"""
    a32, b32 = np.asarray(a).astype(np.float32), np.asarray(b).astype(np.float32)
    return np.abs(a32.view(np.int32).astype(np.int64) - b32.view(np.int32).astype(np.int64)) <= 1


@pytest.mark.parametrize("G,B_r,W", [(1, 1, 4), (2, 3, 6), (4, 0, 5), (1, 2, 24), (7, 1, 6), (12, 2, 5)])
def test_batch_matches_the_numpy_oracle_step_by_step(G, B_r, W):
    n, d, T_max, n_steps = 5, 16, 40, 30
    Q, K, V, dq, dk, dv = make_inputs(100 + G + B_r, n, G, d, T_max, n_steps)
    rng = np.random.default_rng(7)
    B_p = rng.integers(1, 6, n); B_c = rng.integers(0, 7, n)
    T = rng.integers(W, T_max + 1, n)
    T[0] = W                                    # a prompt as short as the window
    B_p[1], B_c[1] = 30, 20                     # a budget larger than its prompt: nothing is dropped
    cap = int((B_p + B_c).max()) + B_r + 3      # slot stride larger than any unit needs
    cb = oc.BatchCache(n, d, G, B_p, B_c, B_r, lam=0.9, alpha=1.0, cap=cap)
    Qw = np.stack([Q[u, :, T[u] - W:T[u]] for u in range(n)])
    s_c = cb.prefill_compress(Qw, K, V, T)
    units = []
    for u in range(n):
        pu = opy.UnitCache(d, G, int(B_p[u]), int(B_c[u]), B_r, lam=0.9, alpha=1.0)
        s_p = pu.prefill_compress(Qw[u], K[u, :T[u]], V[u, :T[u]])
        assert ulp_close(s_c[u, :T[u]], s_p).all()
        units.append(pu)

    def same_state(where):
        off = 0
        for u, pu in enumerate(units):
            B = pu.B
            assert (cb.pos[u, :B] == pu.pos).all() and (cb.w[u, :B] == pu.w).all(), (where, u)
            assert (cb.pos[u, B:] == -1).all() and (cb.w[u, B:] == 0).all()
            assert cb.n_seen[u] == pu.n_seen
            for a, b in ((cb.s[u, :B], pu.s), (cb.K[u, :B], pu.K), (cb.V[u, :B], pu.V)):
                ok = ulp_close(a, b)
                assert ok.all(), (where, u)
                off += int((np.asarray(a) != np.asarray(b)).sum())
        return off

    same_state("prefill")
    for t in range(n_steps):
        out, ws, ev, mg = cb.decode_step(dq[t], dk[t], dv[t])
        for u, pu in enumerate(units):
            o, info = pu.decode_step(dq[t, u], dk[t, u], dv[t, u])
            assert (ws[u], ev[u], mg[u]) == (info.write_slot, info.evicted_pos, info.merged_slot), (t, u)
            np.testing.assert_allclose(out[u], o, rtol=0, atol=1e-12)
        same_state(f"step {t}")


def test_state_handed_over_slot_by_slot_continues_alike():
    """A state handed over slot by slot, token slots in another order (as the parity tests do after a
    device step), goes on exactly like the cache it was taken from: the state is the per-slot arrays alone."""
    n, G, d, T_max, n_steps = 3, 2, 8, 30, 12
    Q, K, V, dq, dk, dv = make_inputs(5, n, G, d, T_max, n_steps)
    a = oc.BatchCache(n, d, G, [3, 4, 2], [4, 2, 5], 2, lam=0.95)
    a.prefill_compress(Q[:, :, -5:], K, V)
    for t in range(4):
        a.decode_step(dq[t], dk[t], dv[t])
    b = oc.BatchCache(n, d, G, [3, 4, 2], [4, 2, 5], 2, lam=0.95)
    rng = np.random.default_rng(3)
    for u in range(n):                      # token slots handed over in another order
        B = 2 + int(a.B_p[u] + a.B_c[u])
        perm = np.concatenate([np.arange(2), 2 + rng.permutation(B - 2)])
        for name in ("K", "V", "pos", "w", "s"):
            getattr(b, name)[u, :B] = getattr(a, name)[u, :B][perm]
    b.n_seen[:] = a.n_seen
    for t in range(4, n_steps):
        oa, _, ea, ma = a.decode_step(dq[t], dk[t], dv[t])
        ob, _, eb, mb = b.decode_step(dq[t], dk[t], dv[t])
        assert (ea == eb).all() and (ma == mb).all()
        np.testing.assert_allclose(oa, ob, rtol=0, atol=1e-12)


def test_reports_what_it_cannot_do():
    with pytest.raises(ValueError):
        oc.BatchCache(2, 8, 1, [2, 0], [1, 1], 1)          # B_p = 0
    c = oc.BatchCache(1, 8, 1, 2, 2, 1)
    x = np.zeros((1, 6, 8))
    c.prefill_compress(np.zeros((1, 1, 2, 8)), x, x)
    with pytest.raises(RuntimeError):
        c.prefill_compress(np.zeros((1, 1, 2, 8)), x, x)   # the cache is not empty any more
    assert oc.threads() >= 1
