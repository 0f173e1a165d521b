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
