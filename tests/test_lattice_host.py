"""Host-side lattice bookkeeping (paper_2311_04996_amd.lattice): n-best paths on a hand-made lattice."""
import numpy as np
import pytest

from paper_2311_04996_amd.binding import LINK_DTYPE
from paper_2311_04996_amd.lattice import Lattice


def _lattice():
    # frame 0: token 0 (state 5, the start) and token 1 (state 2, reached over an epsilon link)
    # frame 1: tokens 2 (state 7) and 3 (state 8)
    off = np.array([0, 2, 4], np.int64)
    state = np.array([5, 2, 7, 8], np.int32)
    cost = np.array([0.0, 0.5, 1.0, 1.25], np.float32)
    rows = [(0, 1, 0, 11, 0.5, 0.0, 0.5, 0),      # epsilon link 5 -> 2, word 11
            (0, 2, 1, 0, 0.25, 0.75, 1.0, 1),     # 5 -> 7
            (1, 2, 2, 12, 0.5, 1.0, 2.0, 1),      # 2 -> 7, dearer than token 2's stored cost
            (1, 3, 1, 13, 0.25, 0.5, 1.25, 1),    # 2 -> 8
            (3, 2, 0, 0, 0.5, 0.0, 1.75, 1)]      # epsilon link 8 -> 7 inside frame 1
    return Lattice(off, state, cost, np.array(rows, dtype=LINK_DTYPE))


def test_nbest_lists_all_paths_in_cost_order():
    lat = _lattice()
    got = lat.nbest(10, start_state=5)
    assert [(c, links, words) for c, links, words in got] == [
        (1.0, [1], []), (1.25, [0, 3], [11, 13]), (1.75, [0, 3, 4], [11, 13]), (2.0, [0, 2], [11, 12])]
    assert lat.nbest(2, 5) == got[:2]


def test_nbest_with_final_costs_skips_non_final_tokens():
    lat = _lattice()
    final = np.full(9, np.inf, np.float32)
    final[8] = 0.5
    got = lat.nbest(10, 5, final)
    assert got == [(1.75, [0, 3], [11, 13])]
    final[:] = np.inf                            # nobody final: all end tokens count, at no cost
    assert [c for c, _, _ in lat.nbest(10, 5, final)] == [1.0, 1.25, 1.75, 2.0]


def test_start_token_must_be_unique():
    lat = _lattice()
    with pytest.raises(ValueError):
        lat.start_token(9)
