"""Pins for the CPU oracle: each test fixes it to something other than itself.

Closed forms, library routines (scipy softmax), special cases that reduce to textbook
attention, a separately written eviction policy, arithmetic means tracked by the test,
brute-force enumeration, the theorem's inequality, and the structure of the paper's
illustrated cache walk (tests/golden/fig2_structure.txt).
"""
import itertools
import math
import os

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import sys

from oracle import zsmerge_oracle as oracle_py
from oracle import zsmerge_oracle_c as oracle_c
from oracle.zsmerge_oracle import UnitCache, prompt_scores, full_attention_row

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(params=["python", "c"], autouse=True)
def oracle_under_test(request, monkeypatch):
    """Every pin runs twice: against the NumPy oracle and against the plain-C one (same
    interface).  The tests name the three entry points as module globals; this swaps them."""
    impl = oracle_py if request.param == "python" else oracle_c
    me = sys.modules[__name__]
    for name in ("UnitCache", "prompt_scores", "full_attention_row"):
        monkeypatch.setattr(me, name, getattr(impl, name))
    return request.param


def rnd(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32).astype(np.float64)


def skewed(seed, T, d, G=1):
    """Random Q/K/V with a few strongly attended keys (float32-representable)."""
    rng = np.random.default_rng(seed)
    u = rng.standard_normal(d); u /= np.linalg.norm(u)
    K = rng.standard_normal((T, d)); V = rng.standard_normal((T, d)); Q = rng.standard_normal((G, T, d))
    hot = rng.random(T) < 0.1
    hot[:2] = True
    K[hot] += 3.0 * d ** 0.25 * u
    Q += d ** 0.25 * u
    f = lambda x: x.astype(np.float32).astype(np.float64)
    return f(Q), f(K), f(V)


# ---------------------------------------------------------------------------------------
# Eq. 1 / Eq. 4 with nothing merged: textbook attention
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("G", [1, 4])
def test_large_budget_is_full_causal_attention_online(G):
    """B - B_r >= T: every step's output is softmax(q K^T / sqrt d) V over all tokens so far."""
    T, d = 40, 16
    Q, K, V = skewed(1, T, d, G)
    c = UnitCache(d, G, B_p=8, B_c=40, B_r=2)
    outs = c.online_prefill(Q, K, V)
    for t in range(T):
        for g in range(G):
            p = sp_softmax((K[:t + 1] @ Q[g, t]) / math.sqrt(d))
            np.testing.assert_allclose(outs[t, g], p @ V[:t + 1], rtol=0, atol=1e-13)
    assert c.w[:2].sum() == 0 and (c.w[2:2 + T] == 1).all()


def test_large_budget_one_shot_then_decode_is_full_attention():
    T, d, n_dec = 30, 8, 10
    Q, K, V = skewed(2, T + n_dec, d)
    c = UnitCache(d, 1, B_p=5, B_c=40, B_r=1)
    c.prefill_compress(Q[:, T - 6:T], K[:T], V[:T])
    assert c.n_seen == T and c.w[0] == 0
    for t in range(T, T + n_dec):
        o, info = c.decode_step(Q[:, t], K[t], V[t])
        p = sp_softmax((K[:t + 1] @ Q[0, t]) / math.sqrt(d))
        np.testing.assert_allclose(o[0], p @ V[:t + 1], atol=1e-13)
        assert info.evicted_pos == -1 and info.merged_slot == -1


def test_custom_scale_is_used():
    d = 8
    Q, K, V = skewed(3, 6, d)
    c = UnitCache(d, 1, 3, 10, 0, scale=0.37)
    outs = c.online_prefill(Q, K, V)
    p = sp_softmax((K @ Q[0, 5]) * 0.37)
    np.testing.assert_allclose(outs[5, 0], p @ V, atol=1e-13)


# ---------------------------------------------------------------------------------------
# Eq. 4 closed form: q = 0 makes the probabilities w^alpha / sum w^alpha
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("alpha", [0.0, 0.5, 1.0])
def test_zero_query_gives_count_weighted_mean(alpha):
    d = 4
    c = UnitCache(d, 1, B_p=2, B_c=2, B_r=2, alpha=alpha)
    V = rnd(4, 6, d)
    K = rnd(5, 6, d)
    # two residual slots holding 5 and 3 merged tokens, three single tokens, one empty slot
    c.import_state(K, V, pos=np.array([0, 1, 7, 8, 9, -1]), w=np.array([5, 3, 1, 1, 1, 0]),
                   s=np.zeros(6), n_seen=12)
    v_new = rnd(6, d)
    o, _ = c.decode_step(np.zeros((1, d)), rnd(7, d), v_new)
    wt = np.array([5.0 ** alpha, 3.0 ** alpha, 1, 1, 1, 1])          # last = incoming token
    expect = (wt[:5] @ V[:5] + v_new) / wt.sum()
    np.testing.assert_allclose(o[0], expect, atol=1e-14)
    np.testing.assert_allclose(c.last_a[0], wt / wt.sum(), atol=1e-15)


def test_alpha_zero_treats_residual_as_a_single_token():
    """alpha = 0: the merged slot's logit carries no count term (eviction-like limit)."""
    d = 8
    K, V = rnd(8, 5, d), rnd(9, 5, d)
    q, kn, vn = rnd(10, 1, d), rnd(11, d), rnd(12, d)
    c = UnitCache(d, 1, 2, 2, 1, alpha=0.0)
    c.import_state(K, V, np.array([3, 10, 11, 12, 13]), np.array([9, 1, 1, 1, 1]), np.zeros(5), 14)
    o, _ = c.decode_step(q, kn, vn)
    Kall, Vall = np.vstack([K, kn]), np.vstack([V, vn])
    p = sp_softmax((Kall @ q[0]) / math.sqrt(d))
    np.testing.assert_allclose(o[0], p @ Vall, atol=1e-14)


def test_alpha_one_adds_log_count():
    d = 8
    K, V = rnd(8, 5, d), rnd(9, 5, d)
    q, kn, vn = rnd(10, 1, d), rnd(11, d), rnd(12, d)
    c = UnitCache(d, 1, 2, 2, 1, alpha=1.0)
    c.import_state(K, V, np.array([3, 10, 11, 12, 13]), np.array([9, 1, 1, 1, 1]), np.zeros(5), 14)
    o, _ = c.decode_step(q, kn, vn)
    Kall, Vall = np.vstack([K, kn]), np.vstack([V, vn])
    num = np.exp((Kall @ q[0]) / math.sqrt(d)) * np.array([9, 1, 1, 1, 1, 1.0])   # w * exp(.)
    np.testing.assert_allclose(o[0], (num / num.sum()) @ Vall, atol=1e-14)


def test_empty_residual_slot_is_masked_for_every_alpha():
    d = 4
    for alpha in (0.0, 1.0):
        c = UnitCache(d, 1, 2, 1, 1, alpha=alpha)
        K, V = rnd(13, 4, d), rnd(14, 4, d)
        K[0] = 100.0                                  # would dominate if it took part
        c.import_state(K, V, np.array([-1, 0, 1, 2]), np.array([0, 1, 1, 1]), np.zeros(4), 3)
        q, kn, vn = rnd(15, 1, d), rnd(16, d), rnd(17, d)
        o, _ = c.decode_step(q, kn, vn)
        Kall, Vall = np.vstack([K[1:], kn]), np.vstack([V[1:], vn])
        np.testing.assert_allclose(o[0], sp_softmax(Kall @ q[0] / 2.0) @ Vall, atol=1e-14)


# ---------------------------------------------------------------------------------------
# Eq. 3: score sums
# ---------------------------------------------------------------------------------------

def causal_attention_matrix(Q, K, d):
    T = K.shape[0]
    Z = (Q @ K.T) / math.sqrt(d)
    Z[np.triu_indices(T, 1)] = -np.inf
    return sp_softmax(Z, axis=1)


def test_prompt_scores_full_history_lambda_one_are_column_sums():
    T, d = 24, 8
    Q, K, V = skewed(20, T, d)
    s = prompt_scores(Q, K, lam=1.0, scale=1 / math.sqrt(d))
    A = causal_attention_matrix(Q[0], K, d)
    np.testing.assert_allclose(s, A.sum(axis=0), rtol=2e-7)
    assert abs(s.sum() - T) < 1e-5


def test_prompt_scores_decay_weights_and_total():
    T, d, lam = 24, 8, 0.9
    Q, K, V = skewed(21, T, d)
    s = prompt_scores(Q, K, lam=lam, scale=1 / math.sqrt(d))
    A = causal_attention_matrix(Q[0], K, d)
    wts = lam ** (T - 1 - np.arange(T))
    np.testing.assert_allclose(s, wts @ A, rtol=2e-7)
    assert abs(s.sum() - (1 - lam ** T) / (1 - lam)) < 1e-5


def test_prompt_scores_window_uses_only_last_rows_and_pools_groups():
    T, d, W, G, lam = 30, 8, 5, 3, 0.98
    Q, K, V = skewed(22, T, d, G)
    s = prompt_scores(Q[:, T - W:], K, lam=lam, scale=1 / math.sqrt(d))
    expect = np.zeros(T)
    for g in range(G):
        A = causal_attention_matrix(Q[g], K, d)
        expect += (lam ** (T - 1 - np.arange(T - W, T))) @ A[T - W:] / G
    np.testing.assert_allclose(s, expect, rtol=2e-7, atol=1e-12)
    assert abs(s.sum() - (1 - lam ** W) / (1 - lam)) < 1e-5


def test_decode_score_increments_sum_to_one():
    """Probabilities sum to one, so sum_j (s_j' - lam s_j) + s_incoming = 1 at every step."""
    T, d, lam = 60, 8, 0.98
    Q, K, V = skewed(23, T, d, 2)
    c = UnitCache(d, 2, 4, 6, 1, lam=lam)
    for t in range(T):
        before, occ = c.s.copy(), c.w > 0
        o, info = c.decode_step(Q[:, t], K[t], V[t])
        after = c.s.copy()
        if info.evicted_pos >= 0:
            # the evicted slot now holds the incoming token; its updated score is in the candidate list
            after[info.write_slot] = info.cand_s[list(info.cand_slots).index(info.write_slot)]
        inc = (after - lam * before)[occ].sum()
        assert abs(inc + c.s[info.write_slot] - 1.0) < 5e-6, t


def test_uniform_attention_score_recursion_closed_form():
    """q = 0 and no eviction: token t's score after n tokens is sum_{m=t}^{n-1} lam^(n-1-m)/(m+1)."""
    d, n, lam = 4, 12, 0.8
    c = UnitCache(d, 1, 3, 20, 1, lam=lam)
    K, V = rnd(24, n, d), rnd(25, n, d)
    c.online_prefill(np.zeros((1, n, d)), K, V)
    for t in range(n):
        expect = sum(lam ** (n - 1 - m) / (m + 1) for m in range(t, n))
        j = int(np.flatnonzero(c.pos == t)[0])
        assert abs(c.s[j] - expect) < 1e-6


# ---------------------------------------------------------------------------------------
# Alg. 1 with B_r = 0: a separately written eviction policy
# ---------------------------------------------------------------------------------------

def eviction_only_reference(Q, K, V, B_p, B_c, lam):
    """'Latest B_p tokens plus the best-scored others': list of records, no slots, no merging."""
    d = K.shape[1]
    cache, outs, victims = [], [], []
    for T in range(K.shape[0]):
        keys = np.array([r["k"] for r in cache] + [K[T]])
        vals = np.array([r["v"] for r in cache] + [V[T]])
        p = sp_softmax((keys @ Q[0, T]) / math.sqrt(d))
        outs.append(p @ vals)
        for r, pj in zip(cache, p[:-1]):
            r["s"] = float(np.float32(lam * r["s"] + pj))
        cache.append(dict(t=T, k=K[T], v=V[T], s=float(np.float32(p[-1]))))
        if len(cache) > B_p + B_c:
            old = sorted(cache, key=lambda r: r["t"])[:-B_p]
            victim = min(old, key=lambda r: (r["s"], r["t"]))
            cache.remove(victim)
            victims.append(victim["t"])
        else:
            victims.append(-1)
    return np.array(outs), victims, sorted(r["t"] for r in cache)


@pytest.mark.parametrize("B_p,B_c", [(3, 4), (1, 6), (6, 0), (5, 5)])
def test_no_residual_budget_is_plain_eviction(B_p, B_c):
    T, d = 80, 8
    Q, K, V = skewed(30 + B_p, T, d)
    c = UnitCache(d, 1, B_p, B_c, 0)
    outs, ev = [], []
    for t in range(T):
        o, info = c.decode_step(Q[:, t], K[t], V[t])
        outs.append(o[0]); ev.append(info.evicted_pos)
        assert info.merged_slot == -1
    r_outs, r_ev, r_left = eviction_only_reference(Q, K, V, B_p, B_c, 0.98)
    assert ev == r_ev
    np.testing.assert_allclose(np.array(outs), r_outs, atol=1e-13)
    assert sorted(c.pos[c.w > 0].tolist()) == r_left
    assert c.w.sum() == B_p + B_c                       # evicted tokens are simply dropped


# ---------------------------------------------------------------------------------------
# Eq. 5 / Eq. 6: residual absorption
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("mode", ["online", "one_shot"])
def test_single_residual_slot_is_the_mean_of_everything_evicted(mode):
    T0, n_dec, d = 50, 40, 8
    Q, K, V = skewed(40, T0 + n_dec, d)
    c = UnitCache(d, 1, 4, 5, 1)
    gone = []
    if mode == "online":
        start = 0
    else:
        c.prefill_compress(Q[:, T0 - 8:T0], K[:T0], V[:T0])
        kept = set(c.pos[1:].tolist())
        gone = [t for t in range(T0) if t not in kept]
        start = T0
        assert len(gone) == T0 - 9
    for t in range(start, T0 + n_dec):
        o, info = c.decode_step(Q[:, t], K[t], V[t])
        if info.evicted_pos >= 0:
            gone.append(info.evicted_pos)
            assert info.merged_slot == 0
        assert c.w.sum() == t + 1                      # merged-slot weights sum to tokens seen
        if gone:
            assert c.w[0] == len(gone)
            np.testing.assert_allclose(c.K[0], K[gone].mean(axis=0), atol=2e-6)
            np.testing.assert_allclose(c.V[0], V[gone].mean(axis=0), atol=2e-6)
    assert len(set(gone)) == len(gone) == T0 + n_dec - 9


def test_residual_slot_choice_follows_largest_dot_product():
    """Two residual slots along e0 and e1: an evicted key is absorbed by the better aligned one."""
    d = 4
    c = UnitCache(d, 1, B_p=1, B_c=1, B_r=2)
    e = np.eye(d)
    K = np.array([2 * e[0], 3 * e[1], 5 * e[1] + 1 * e[0], 9 * e[2]])
    V = np.array([[1.0, 0, 0, 0], [0, 2.0, 0, 0], [4.0, 4.0, 4.0, 4.0], [7.0, 7, 7, 7]])
    c.import_state(K, V, pos=np.array([0, 1, 2, 3]), w=np.array([1, 3, 1, 1]), s=np.array([0, 0, 0.0, 5.0]), n_seen=4)
    o, info = c.decode_step(np.zeros((1, d)), e[3], e[3])
    assert info.evicted_pos == 2 and info.merged_slot == 1         # dots: slot0 -> 2, slot1 -> 15
    np.testing.assert_allclose(c.K[1], (3 * 3 * e[1] + 5 * e[1] + e[0]) / 4)
    np.testing.assert_allclose(c.V[1], (3 * V[1] + V[2]) / 4)
    assert c.w[1] == 4 and c.w[0] == 1
    np.testing.assert_allclose(c.K[0], K[0])                        # the other slot is untouched


def test_residual_dot_product_is_raw_not_cosine():
    d = 2
    c = UnitCache(d, 1, 1, 1, 2)
    # slot 0: short but perfectly aligned; slot 1: long, less aligned -> raw dot prefers slot 1
    K = np.array([[0.1, 0.0], [5.0, 5.0], [1.0, 0.0], [0.0, 9.0]])
    V = np.zeros((4, d))
    c.import_state(K, V, np.array([0, 1, 2, 3]), np.array([1, 1, 1, 1]), np.array([0, 0, 0.0, 1.0]), 4)
    _, info = c.decode_step(np.zeros((1, d)), np.ones(d), np.ones(d))
    assert info.merged_slot == 1


def test_residual_tie_goes_to_lowest_index_and_slots_open_in_order():
    d = 2
    c = UnitCache(d, 1, 1, 1, 3)
    rng_k = [np.array([1.0, 0.0])] * 8
    infos = []
    for t in range(8):
        _, info = c.decode_step(np.zeros((1, d)), rng_k[t], np.array([float(t), 0.0]))
        infos.append(info.merged_slot)
    # tokens 0..1 fill the two token slots; evictions start at t=2: slots 0,1,2 open in order, then ties -> 0
    assert infos == [-1, -1, 0, 1, 2, 0, 0, 0]


# ---------------------------------------------------------------------------------------
# eviction choice
# ---------------------------------------------------------------------------------------

def test_eviction_takes_lowest_score_outside_the_latest_Bp_and_breaks_ties_by_position():
    d = 2
    c = UnitCache(d, 1, B_p=2, B_c=3, B_r=1)
    K = rnd(50, 6, d); V = rnd(51, 6, d)
    # token slots 1..5 hold positions 10..14 shuffled; scores: two equal minima among the candidates
    pos = np.array([3, 13, 10, 14, 11, 12])
    s = np.array([9.0, 0.0, 0.5, 0.0, 0.5, 0.7])      # 13 and 14 score 0 but 14 is inside the window
    c.import_state(K, V, pos, np.array([4, 1, 1, 1, 1, 1]), s, n_seen=15)
    _, info = c.decode_step(np.zeros((1, d)), rnd(52, d), rnd(53, d))
    # incoming token has position 15: the window is {14, 15}; candidates 10, 11, 12, 13.
    # uniform attention adds the same amount to every score, so the order is that of s
    assert sorted(info.cand_pos.tolist()) == [10, 11, 12, 13]
    assert info.evicted_pos == 13 and info.write_slot == 1
    c.import_state(K, V, pos, np.array([4, 1, 1, 1, 1, 1]), np.array([9.0, 3.0, 0.5, 0.0, 0.5, 0.7]), n_seen=15)
    _, info = c.decode_step(np.zeros((1, d)), rnd(52, d), rnd(53, d))
    assert info.evicted_pos == 10 and info.write_slot == 2           # 10 and 11 tie -> earlier position


def test_slot_order_does_not_matter():
    """Permuting the physical order of the token slots changes slot numbers only."""
    T0, d = 40, 8
    Q, K, V = skewed(60, T0 + 20, d)
    a = UnitCache(d, 1, 4, 6, 1)
    a.prefill_compress(Q[:, T0 - 4:T0], K[:T0], V[:T0])
    st = a.export_state()
    perm = np.concatenate([[0], 1 + np.random.default_rng(0).permutation(10)])
    b = UnitCache(d, 1, 4, 6, 1)
    b.import_state(st["K"][perm], st["V"][perm], st["pos"][perm], st["w"][perm], st["s"][perm], st["n_seen"])
    for t in range(T0, T0 + 20):
        oa, ia = a.decode_step(Q[:, t], K[t], V[t])
        ob, ib = b.decode_step(Q[:, t], K[t], V[t])
        np.testing.assert_allclose(oa, ob, atol=1e-14)
        assert ia.evicted_pos == ib.evicted_pos
    assert sorted(a.pos.tolist()) == sorted(b.pos.tolist())


# ---------------------------------------------------------------------------------------
# prefill selection
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(6))
def test_selection_brute_force(seed):
    """T <= 12: among all size-B_c subsets of the old positions, the kept one has the largest
    score total, and no dropped position outranks a kept one under (score, -position)."""
    T, d, B_p, B_c = 12, 4, 3, 4
    Q, K, V = skewed(70 + seed, T, d)
    if seed % 2:                                   # force exact score ties
        K[1:7] = K[1]
    c = UnitCache(d, 1, B_p, B_c, 1)
    s = c.prefill_compress(Q[:, T - 5:], K, V)
    kept = sorted(c.pos[1:].tolist())
    assert kept[-B_p:] == [9, 10, 11]
    ctx = kept[:B_c]
    head = list(range(T - B_p))
    best = max(itertools.combinations(head, B_c), key=lambda S: (sum(s[list(S)]), [-t for t in S]))
    assert abs(sum(s[ctx]) - sum(s[list(best)])) < 1e-12
    for t in head:
        if t not in ctx:
            for k in ctx:
                assert (s[k], -k) > (s[t], -t)
    # layout: residual first, then context by position, then proximity by position
    assert c.pos[1:].tolist() == ctx + [9, 10, 11]
    assert (c.s[1:] == s[c.pos[1:]]).all()
    assert c.w[0] == T - B_p - B_c and c.w.sum() == T


def test_selection_ties_keep_earlier_positions():
    T, d = 10, 4
    K = np.tile(rnd(80, 1, d), (T, 1))             # identical keys -> identical scores within a row
    V = rnd(81, T, d)
    Q = rnd(82, 1, 1, d)                           # a single query row (the last position)
    c = UnitCache(d, 1, 2, 3, 1)
    s = c.prefill_compress(Q, K, V)
    assert np.ptp(s) == 0
    assert c.pos[1:].tolist() == [0, 1, 2, 8, 9]


def test_short_prompt_keeps_everything():
    d = 4
    Q, K, V = skewed(83, 6, d)
    c = UnitCache(d, 1, 4, 5, 2)
    c.prefill_compress(Q[:, 3:], K, V)
    assert c.pos.tolist() == [-1, -1, 0, 1, 2, 3, 4, 5, -1, -1, -1]
    assert list(c.Kp) == [4, 5, 6, 7] and c.Kc == [2, 3]


# ---------------------------------------------------------------------------------------
# Thm. 1
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("alpha,B_r", [(1.0, 1), (1.0, 3), (0.5, 2)])
def test_theorem_unmerged_tokens_never_lose_attention(alpha, B_r):
    T, d = 120, 8
    Q, K, V = skewed(90, T, d)
    c = UnitCache(d, 1, 5, 6, B_r, alpha=alpha)
    for t in range(T):
        pos_before, w_before = c.pos.copy(), c.w.copy()
        c.decode_step(Q[:, t], K[t], V[t])
        _, a_full = full_attention_row(Q[0, t], K[:t + 1], V[:t + 1], 1 / math.sqrt(d))
        occ = c.last_occ
        for idx, j in enumerate(occ):
            if j >= B_r:                                       # an unmerged token
                assert c.last_a[0, idx] >= a_full[pos_before[j]] - 1e-12
        assert c.last_a[0, -1] >= a_full[t] - 1e-12          # the incoming token


# ---------------------------------------------------------------------------------------
# the paper's illustrated walk (structure only: the figure itself is an image)
# ---------------------------------------------------------------------------------------

def test_figure_walk_structure():
    cfg = {}
    with open(os.path.join(GOLDEN, "fig2_structure.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                cfg[k.strip()] = int(v)
    d = 8
    T1 = cfg["T_end"]
    Q, K, V = skewed(99, T1, d)
    c = UnitCache(d, 1, cfg["B_p"], cfg["B_c"], cfg["B_r"])
    for t in range(T1):
        c.decode_step(Q[:, t], K[t], V[t])
        n = t + 1
        if n >= cfg["T_start"]:
            tok = c.pos[cfg["B_r"]:]
            assert len(c.Kp) == cfg["B_p"] and len(c.Kc) == cfg["B_c"] and len(c.Kr) == cfg["B_r"]
            assert sorted(c.pos[list(c.Kp)].tolist()) == list(range(n - cfg["B_p"], n))   # latest 3
            assert c.w[:cfg["B_r"]].sum() == n - cfg["B_p"] - cfg["B_c"]
            assert (c.w[cfg["B_r"]:] == 1).all() and len(set(tok.tolist())) == tok.size


# ---------------------------------------------------------------------------------------
# grouped queries in the decode update (appendix, GQA adaptation, with Eq. 3)
# ---------------------------------------------------------------------------------------

def test_decode_score_update_pools_the_group_by_its_unweighted_mean():
    """G = 2, two very different query heads, nothing evicted: every stored score becomes
    lam * s + (p_head0 + p_head1) / 2 with p_g the scipy softmax row of head g, and the
    incoming token starts at the mean of its own two probabilities."""
    d, lam = 4, 0.9
    K, V = rnd(100, 5, d), rnd(101, 5, d)
    q = np.array([[3.0, 0.0, -1.0, 0.5], [-2.0, 1.0, 0.0, 4.0]])        # head 0, head 1
    kn, vn = rnd(102, d), rnd(103, d)
    s0 = np.array([0.25, 0.5, 1.0, 2.0, 0.125, 0.0, 0.0, 0.0])
    c = UnitCache(d, 2, B_p=3, B_c=5, B_r=0, lam=lam)
    Kst, Vst = np.zeros((8, d)), np.zeros((8, d))
    Kst[:5], Vst[:5] = K, V
    c.import_state(Kst, Vst, pos=np.array([0, 1, 2, 3, 4, -1, -1, -1]),
                   w=np.array([1, 1, 1, 1, 1, 0, 0, 0]), s=s0, n_seen=5)
    out, info = c.decode_step(q, kn, vn)
    assert info.evicted_pos == -1 and info.write_slot == 5
    Kall, Vall = np.vstack([K, kn]), np.vstack([V, vn])
    p0 = sp_softmax(Kall @ q[0] / math.sqrt(d))
    p1 = sp_softmax(Kall @ q[1] / math.sqrt(d))
    assert np.abs(p0 - p1).max() > 0.2                                   # the heads really differ
    expect = lam * s0[:5] + 0.5 * (p0[:5] + p1[:5])
    np.testing.assert_allclose(c.s[:5], expect, rtol=1e-6)
    assert abs(c.s[5] - 0.5 * (p0[5] + p1[5])) < 1e-7
    # head 0 alone, head 1 alone, or an uneven weighting would all be off by far more than that
    assert np.abs(lam * s0[:5] + p0[:5] - c.s[:5]).max() > 1e-2
    np.testing.assert_allclose(out[0], p0 @ Vall, atol=1e-13)            # one softmax per head
    np.testing.assert_allclose(out[1], p1 @ Vall, atol=1e-13)


def test_decode_eviction_choice_uses_the_pooled_score():
    """G = 2: head 0 alone would make position 0 the weakest token, the mean over both heads
    makes it position 1 (Alg. 1 context overflow on the pooled Eq. 3 scores)."""
    d = 2
    K = np.array([[0.0, 8.0], [1.0, 1.0], [4.0, 4.0], [4.0, 4.0]])
    V = np.eye(4)[:, :d] * 0 + np.arange(4)[:, None]
    q = np.array([[4.0, 0.0], [0.0, 4.0]])        # head 0 ignores position 0, head 1 loves it
    c = UnitCache(d, 2, B_p=2, B_c=2, B_r=0, lam=1.0, scale=1.0)
    c.import_state(K, V, pos=np.arange(4), w=np.ones(4, dtype=int), s=np.zeros(4), n_seen=4)
    _, info = c.decode_step(q, np.array([4.0, 4.0]), np.zeros(d))
    Kall = np.vstack([K, [4.0, 4.0]])
    p = 0.5 * (sp_softmax(Kall @ q[0]) + sp_softmax(Kall @ q[1]))
    assert sp_softmax(Kall @ q[0])[0] < sp_softmax(Kall @ q[0])[1]      # head 0's view
    assert p[1] < p[0]                                                    # the pooled view
    assert sorted(info.cand_pos.tolist()) == [0, 1, 2]
    assert info.evicted_pos == 1


# ---------------------------------------------------------------------------------------
# one-shot prefill with two residual slots: absorption order (Alg. 1 residual branch,
# Eq. 5, Eq. 6; the tokens not kept are taken in position order)
# ---------------------------------------------------------------------------------------

def _two_slot_prompt():
    """Eight tokens, d = 2, B_p = 1, B_c = 1, B_r = 2.  The single query (last position) points
    along (1, 1), so position 2 with key (5, 5) has by far the largest score and is the context
    token; position 7 is the proximity token.  Dropped, in position order: 0, 1, 3, 4, 5, 6."""
    K = np.array([[1.0, 0.0],      # 0  opens residual slot 0
                  [2.0, 0.5],      # 1  opens residual slot 1
                  [5.0, 5.0],      # 2  kept (context)
                  [0.0, 2.0],      # 3  dots 0 vs 1            -> slot 1: K = (1, 1.25), w = 2
                  [3.0, 0.0],      # 4  dots 3 vs 3, a tie     -> slot 0: K = (2, 0), w = 2
                  [0.0, 1.0],      # 5  dots 0 vs 1.25         -> slot 1: K = (2/3, 7/6), w = 3
                  [1.0, 1.0],      # 6  dots 2 vs 11/6         -> slot 0 (it would go to slot 1, 1 vs 11/6,
                                   #    had token 4 not moved slot 0 first): K = (5/3, 1/3), w = 3
                  [0.5, 0.5]])     # 7  kept (proximity)
    V = np.array([[1.0, 10.0], [2.0, 20.0], [3.0, 30.0], [4.0, 40.0],
                  [5.0, 50.0], [6.0, 60.0], [7.0, 70.0], [8.0, 80.0]])
    Q = np.array([[[1.0, 1.0]]])
    return Q, K, V


def test_one_shot_prefill_two_residual_slots_hand_computed():
    Q, K, V = _two_slot_prompt()
    c = UnitCache(2, 1, B_p=1, B_c=1, B_r=2, scale=1.0)
    s = c.prefill_compress(Q, K, V)
    assert c.pos[2:].tolist() == [2, 7]
    # values worked out by hand from Eq. 5 (largest raw dot product, ties to the lower slot)
    # and Eq. 6 (incremental mean): slot 0 absorbed tokens 0, 4, 6 and slot 1 tokens 1, 3, 5
    np.testing.assert_allclose(c.K[0], [5.0 / 3, 1.0 / 3], rtol=3e-7)
    np.testing.assert_allclose(c.K[1], [2.0 / 3, 3.5 / 3], rtol=3e-7)
    np.testing.assert_allclose(c.V[0], [13.0 / 3, 130.0 / 3], rtol=3e-7)
    np.testing.assert_allclose(c.V[1], [4.0, 40.0], rtol=3e-7)
    assert c.w.tolist() == [3, 3, 1, 1] and c.w.sum() == 8
    # a residual slot keeps the position and the score of the token that opened it
    assert c.pos[:2].tolist() == [0, 1]
    assert c.s[0] == s[0] and c.s[1] == s[1] and s[1] > s[0] > 0
    assert c.n_seen == 8 and c.Kr == [0, 1]


def test_one_shot_prefill_absorbs_in_position_order_not_another():
    """The same prompt walked by an explicit Eq. 5 / Eq. 6 loop written here: position order
    reproduces the oracle, the reverse order gives a different residual set."""
    Q, K, V = _two_slot_prompt()
    c = UnitCache(2, 1, 1, 1, 2, scale=1.0)
    c.prefill_compress(Q, K, V)

    def walk(order):
        Kr, Vr, w = [], [], []
        for t in order:
            if len(Kr) < 2:
                Kr.append(K[t].copy()); Vr.append(V[t].copy()); w.append(1)
                continue
            dots = [float(kr @ K[t]) for kr in Kr]
            r = 0 if dots[0] >= dots[1] else 1
            Kr[r] = (w[r] * Kr[r] + K[t]) / (w[r] + 1)
            Vr[r] = (w[r] * Vr[r] + V[t]) / (w[r] + 1)
            w[r] += 1
        return np.array(Kr), np.array(Vr), w

    dropped = [0, 1, 3, 4, 5, 6]
    Kf, Vf, wf = walk(dropped)
    np.testing.assert_allclose(c.K[:2], Kf, rtol=3e-7)
    np.testing.assert_allclose(c.V[:2], Vf, rtol=3e-7)
    assert c.w[:2].tolist() == wf
    Kb, Vb, wb = walk(dropped[::-1])
    assert np.abs(Kb - Kf).max() > 0.1 and np.abs(Vb - Vf).max() > 0.1


def test_eviction_that_opens_a_residual_slot_hands_over_position_and_score():
    """Decode: the first eviction fills the unused residual slot with the evicted token's
    key, value, count 1, position, and its score as updated in this very step (Eq. 3)."""
    d, lam = 2, 0.5
    K = np.array([[9.0, 9.0], [1.0, 2.0], [3.0, 4.0], [5.0, 6.0]])
    V = np.array([[9.0, 9.0], [0.5, 0.25], [7.0, 8.0], [1.0, 1.0]])
    c = UnitCache(d, 1, B_p=1, B_c=2, B_r=1, lam=lam)
    c.import_state(K, V, pos=np.array([-1, 4, 5, 6]), w=np.array([0, 1, 1, 1]),
                   s=np.array([0.0, 0.25, 2.0, 3.0]), n_seen=7)
    _, info = c.decode_step(np.zeros((1, d)), np.array([0.0, 1.0]), np.array([1.0, 0.0]))
    # q = 0: four entries (three tokens + the incoming one) get probability 1/4 each
    assert info.evicted_pos == 4 and info.merged_slot == 0 and info.write_slot == 1
    assert c.pos[0] == 4 and c.w[0] == 1
    assert c.s[0] == np.float32(lam * 0.25 + 0.25)
    np.testing.assert_array_equal(c.K[0], K[1]); np.testing.assert_array_equal(c.V[0], V[1])
    # a later merge leaves that position and score alone (the score only decays and accrues)
    _, info = c.decode_step(np.zeros((1, d)), np.array([1.0, 1.0]), np.array([2.0, 2.0]))
    assert info.merged_slot == 0 and c.w[0] == 2 and c.pos[0] == 4
    # entries: residual (w = 2 -> weight 2), three tokens, incoming: probabilities 2/5? no - the
    # count seen by the softmax is the one before this step's merge (w = 1): 1/5 each
    assert c.s[0] == np.float32(lam * float(np.float32(lam * 0.25 + 0.25)) + 0.2)


# ---------------------------------------------------------------------------------------
# the full-attention checker itself (Eq. 1)
# ---------------------------------------------------------------------------------------

def test_full_attention_row_is_textbook_softmax_attention():
    T, d = 17, 8
    Q, K, V = skewed(110, T, d)
    K[3] *= 40.0                                      # large logits: the shift by the maximum matters
    for scale in (1 / math.sqrt(d), 0.21):
        o, a = full_attention_row(Q[0, 5], K, V, scale)
        p = sp_softmax(K @ Q[0, 5] * scale)
        np.testing.assert_allclose(a, p, rtol=1e-13, atol=1e-300)
        np.testing.assert_allclose(o, p @ V, atol=1e-12)
        assert abs(a.sum() - 1) < 1e-14
    # an asymmetric case worked by hand: logits (0, ln 3) -> probabilities (1/4, 3/4)
    o, a = full_attention_row(np.array([1.0, 0.0]), np.array([[0.0, 5.0], [math.log(3.0), -2.0]]),
                              np.array([[4.0, 0.0], [0.0, 8.0]]), 1.0)
    np.testing.assert_allclose(a, [0.25, 0.75], rtol=1e-14)
    np.testing.assert_allclose(o, [1.0, 6.0], rtol=1e-14)
