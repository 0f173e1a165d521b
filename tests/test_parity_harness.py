"""The parity harness's own rule for near ties, checked on the CPU with hand-made step records: another eviction
victim is accepted only when the oracle's two competing scores differ by less than 1e-6 relative."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle.zsmerge_oracle import StepInfo
from tests import parity_util as pu


def _info(scores, positions, slots, victim_idx):
    return StepInfo(write_slot=slots[victim_idx], evicted_pos=positions[victim_idx], merged_slot=0,
                    cand_slots=np.array(slots), cand_s=np.array(scores, dtype=np.float64), cand_pos=np.array(positions))


def test_same_victim_is_no_tie():
    st = pu.StepStats()
    info = _info([0.5, 0.25, 0.75], [10, 11, 12], [4, 5, 6], 1)
    out = np.zeros((1, 4))
    assert pu.check_step(out, (5, 11, 0), out, info, None, 1e-5, st, "t") is False
    assert st.near_ties == 0 and st.evictions == 1 and st.merges == 1
    with pytest.raises(AssertionError):                      # same victim, another residual slot: never allowed
        pu.check_step(out, (5, 11, 1), out, info, None, 1e-5, st, "t")


def test_other_victim_inside_the_band_is_a_permitted_flip():
    st = pu.StepStats()
    lo = 0.25
    info = _info([0.5, lo, lo * (1 + 5e-7)], [10, 11, 12], [4, 5, 6], 1)
    out = np.zeros((1, 4))
    assert pu.check_step(out, (6, 12, 0), out, info, None, 1e-5, st, "t") is True
    assert st.near_ties == 1


def test_other_victim_outside_the_band_fails():
    st = pu.StepStats()
    info = _info([0.5, 0.25, 0.25 * (1 + 1e-5)], [10, 11, 12], [4, 5, 6], 1)
    out = np.zeros((1, 4))
    with pytest.raises(AssertionError):
        pu.check_step(out, (6, 12, 0), out, info, None, 1e-5, st, "t")
    with pytest.raises(AssertionError):                      # a victim that was no candidate at all
        pu.check_step(out, (9, 99, 0), out, info, None, 1e-5, st, "t")
    with pytest.raises(AssertionError):                      # the device evicted although the oracle only filled a free slot
        free = StepInfo(7, -1, -1, np.zeros(0, dtype=np.int64), np.zeros(0), np.zeros(0, dtype=np.int64))
        pu.check_step(out, (6, 12, 0), out, free, None, 1e-5, st, "t")


def test_output_error_beyond_the_tolerance_fails():
    st = pu.StepStats()
    info = _info([0.5, 0.25], [10, 11], [4, 5], 1)
    with pytest.raises(AssertionError):
        pu.check_step(np.full((1, 4), 3e-5), (5, 11, 0), np.zeros((1, 4)), info, None, 1e-5, st, "t")


# ---- the every-unit comparison against the C oracle: what it accepts and what it rejects ----------------

def _layer(seed=0):
    """A C-oracle layer of 4 units (2 sequences x 2 heads) after a small prefill, its state in the form the device
    exports (the tests below edit that copy), and the prompt scores."""
    from oracle import zsmerge_oracle_c as oc
    rng = np.random.default_rng(seed)
    n, G, d, T, W = 4, 2, 8, 24, 5
    f = lambda x: x.astype(np.float32).astype(np.float64)
    Q, K, V = f(rng.standard_normal((n, G, W, d))), f(rng.standard_normal((n, T, d))), f(rng.standard_normal((n, T, d)))
    cb = oc.BatchCache(n, d, G, 3, 4, 2, lam=0.9, cap=10)
    s = cb.prefill_compress(Q, K, V)
    exported = {k: v.clone() for k, v in pu.pack_c_state(cb, 2, 2, torch.float32).items()}
    return cb, s, exported


def test_every_unit_comparison_accepts_the_oracles_own_state():
    cb, s, g = _layer()
    st = pu.StepStats()
    assert pu.compare_layer_with_c_oracle(g, cb, 1e-5, "t", st, prompt_scores=s) == []
    assert st.s_total == int((cb.w > 0).sum()) and st.s_bit_equal == st.s_total


@pytest.mark.parametrize("what", ["score", "residual", "token_row", "count", "n_seen"])
def test_every_unit_comparison_rejects_a_wrong_value(what):
    cb, s, g = _layer()
    if what == "score":
        g["s"][1, 0, 3] += 1e-3
    elif what == "residual":
        g["Kr"][0, 1, 0, 2] += 1e-3
    elif what == "token_row":
        g["V"][1, 1, 4, 0] += 1e-6        # token rows are copies: any difference counts
    elif what == "count":
        g["w"][0, 0, 0] += 1
    else:
        g["n_seen"][1, 1] += 1
    with pytest.raises(AssertionError):
        pu.compare_layer_with_c_oracle(g, cb, 1e-5, "t")


def test_every_unit_comparison_and_the_selection_boundary():
    """Another token kept at the boundary is a permitted flip only when the oracle's scores of the two tokens lie
    within the tie band; the flipped unit is reported and left out of the value comparisons."""
    cb, s, g = _layer()
    u, Br = 2, cb.B_r
    B = Br + int(cb.B_p[u] + cb.B_c[u])
    T = int(cb.n_seen[u])
    ctx_slots = [j for j in range(Br, B) if cb.pos[u, j] < T - cb.B_p[u]]
    j_low = min(ctx_slots, key=lambda j: s[u, cb.pos[u, j]])              # the kept token of lowest score
    kept = set(cb.pos[u, Br:B].tolist())
    t_out = max((t for t in range(T - int(cb.B_p[u])) if t not in kept), key=lambda t: s[u, t])   # best token not kept
    g["pos"][u // 2, u % 2, j_low] = t_out                                # the "device" kept that one instead
    with pytest.raises(AssertionError):                                   # scores well apart: not a tie
        pu.compare_layer_with_c_oracle(g, cb, 1e-5, "t", prompt_scores=s)
    s2 = s.copy()
    s2[u, t_out] = s[u, cb.pos[u, j_low]] * (1 - 5e-7)                    # now the oracle itself sees a near tie
    assert pu.compare_layer_with_c_oracle(g, cb, 1e-5, "t", prompt_scores=s2) == [u]
    with pytest.raises(AssertionError):                                   # after the prefill stage no flips are taken
        pu.compare_layer_with_c_oracle(g, cb, 1e-5, "t")
