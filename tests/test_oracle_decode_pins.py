"""Decode-level pins for the CPU oracle: the prune step, the initial closure and every
tie-break, checked on whole decodes of graphs whose answer is known in closed form.

All costs are dyadic (multiples of 1/16, log-likelihoods 0), so every sum is exact in fp32 and
the expected token sets follow from the rule itself (Section "Offline inference": beam = largest
score gap to the best hypothesis, max-active = largest number of hypotheses; readings R3, R4,
R5, R8 and the initial-set reading in oracle/wfst_oracle.c).  tests/test_oracle_mutations.py
plants single mistakes in a copy of the oracle and checks that this file then fails.
"""
import numpy as np

from oracle import Oracle
from workloads.graphs import _from_arc_list

INF = float("inf")
IMAX = 2**31 - 1


def star(weights, extra=()):
    """Start state 0 with one blank-labelled arc of weight weights[j] to state j + 1."""
    arcs = [(0, j + 1, 1, 0, float(w)) for j, w in enumerate(weights)] + list(extra)
    S = len(weights) + 1
    return _from_arc_list(S, 0, 1, arcs, np.zeros(S, np.float32))


def kept_states(g, beam, max_active):
    r = Oracle(g).decode(np.zeros((1, 1), np.float32), beam=beam, max_active=max_active, want_frames=True)
    st, co = r.frames[1]
    return sorted(st.tolist()), dict(zip(st.tolist(), co.tolist())), r


# ---------------------------------------------------------------- R4/R5 inside a decode
def test_star_keeps_exactly_the_lowest_bins():
    """257 tokens at best + j/16 (beam 16: bin j, gap == beam in bin 255) and one outside the
    beam.  max_active 100: the running count first exceeds 100 in bin 100, so bins 0..99 stay."""
    w = [j / 16.0 for j in range(256)] + [16.0, 16.0625]
    g = star(w)
    st, co, r = kept_states(g, 16.0, 100)
    assert st == list(range(1, 101))
    assert all(co[s] == (s - 1) / 16.0 for s in st)
    assert r.counters[5] == 1 and r.counters[6] == 0 and r.counters[3] == 100 and r.counters[7] == 258


def test_star_gap_equal_to_beam_is_kept_and_beyond_is_not():
    w = [j / 16.0 for j in range(256)] + [16.0, 16.0625]
    st, _, r = kept_states(star(w), 16.0, IMAX)
    assert st == list(range(1, 258))                       # state 257 has gap == beam, state 258 is outside
    assert r.counters[5] == 0


def test_star_everything_stays_when_in_beam_equals_max_active():
    w = [j / 16.0 for j in range(256)] + [16.0, 16.0625]
    st, _, r = kept_states(star(w), 16.0, 257)             # exactly 257 tokens are in the beam
    assert st == list(range(1, 258))
    assert r.counters[5] == 0                              # max-active did not prune
    st, _, r = kept_states(star(w), 16.0, 256)             # one fewer: the last bin (2 tokens) goes
    assert st == list(range(1, 256))
    assert r.counters[5] == 1


def test_star_running_count_must_exceed_not_reach():
    """Two tokens per bin, max_active 100: after bin 49 the count is exactly 100 (not exceeded),
    bin 50 takes it to 102, so bins 0..49 = 100 tokens survive."""
    w = [(j // 2) / 16.0 for j in range(300)]
    st, _, _ = kept_states(star(w), 16.0, 100)
    assert st == list(range(1, 101))
    st, _, _ = kept_states(star(w), 16.0, 99)              # exceeded inside bin 49: bins 0..48
    assert st == list(range(1, 99))


def test_star_bin0_overflow_keeps_all_of_bin0():
    w = [0.0] * 40 + [1.0 / 32.0] * 10 + [1.0, 2.0]       # 50 tokens in bin 0 (width 1/16), 2 above
    st, _, r = kept_states(star(w), 16.0, 7)
    assert st == list(range(1, 51))
    assert r.counters[5] == 1 and r.counters[6] == 1


def test_cutoff_is_frozen_for_the_closure():
    """Epsilon arcs out of kept tokens are held to the same (best, k_keep): with bins 0..99 kept,
    an epsilon arc landing in bin 99 makes a token, one landing in bin 100 does not, and a
    negative one below the best is kept (bin 0)."""
    w = [j / 16.0 for j in range(256)]
    n = len(w)
    extra = [(1, n + 1, 0, 0, 99 / 16.0), (1, n + 2, 0, 0, 100 / 16.0), (2, n + 3, 0, 0, -1.0)]
    arcs = [(0, j + 1, 1, 0, float(x)) for j, x in enumerate(w)] + extra
    g = _from_arc_list(n + 4, 0, 1, arcs, np.zeros(n + 4, np.float32))
    st, co, _ = kept_states(g, 16.0, 100)
    assert st == list(range(1, 101)) + [n + 1, n + 3]
    assert co[n + 1] == 99 / 16.0 and co[n + 3] == 1 / 16.0 - 1.0


# ---------------------------------------------------------------- the initial set
def test_initial_closure_has_no_bin_limit_but_a_beam():
    """A_0 = start token closed over epsilon arcs with best = 0: costs in the upper bins stay
    (no max-active before the first frame), costs beyond the beam do not."""
    arcs = [(0, 1, 0, 0, 9.0), (0, 2, 0, 0, 12.0), (0, 3, 0, 0, 15.9375), (0, 4, 0, 0, 16.0),
            (0, 5, 0, 0, 16.5), (1, 6, 0, 0, 6.5), (0, 0, 1, 0, 0.0)]
    g = _from_arc_list(7, 0, 1, arcs, np.zeros(7, np.float32))
    r = Oracle(g).decode(np.zeros((1, 1), np.float32), length=0, beam=16.0, max_active=2, want_frames=True)
    st, co = r.frames[0]
    got = dict(zip(st.tolist(), co.tolist()))
    assert got == {0: 0.0, 1: 9.0, 2: 12.0, 3: 15.9375, 4: 16.0, 6: 15.5}


# ---------------------------------------------------------------- R3: exact ties in recombination
def _two_step(first_low):
    """start -> {1, 2} (equal cost), then 1 -> 3 and 2 -> 3 with equal weights: an exact tie in
    state 3 between the arc of state 1 (lower global id) and the arc of state 2.  first_low says
    whether the token of state 1 is expanded first (token order = creation order)."""
    a1, a2 = (0, 1, 1, 11, 1.0), (0, 2, 1, 22, 1.0)
    arcs = ([a1, a2] if first_low else [a2, a1]) + [(1, 3, 1, 33, 0.5), (2, 3, 1, 44, 0.5)]
    return _from_arc_list(4, 0, 1, arcs, [INF, INF, INF, 0.0])


def test_emitting_tie_goes_to_the_lower_arc_id():
    for first_low in (True, False):
        g = _two_step(first_low)
        o = Oracle(g)
        r = o.decode(np.zeros((2, 1), np.float32), beam=50.0, max_active=IMAX, want_path=True)
        assert r.cost == 1.5
        # global emitting ids follow (state, order): the arc of state 1 is id 2, of state 2 id 3
        assert r.path_arcs.tolist()[-1] == 2
        assert r.words.tolist() == [11, 33]


def test_epsilon_tie_goes_to_the_lower_arc_id():
    for first_low in (True, False):
        a1, a2 = (0, 1, 1, 11, 1.0), (0, 2, 1, 22, 1.0)
        arcs = ([a1, a2] if first_low else [a2, a1]) + [(1, 3, 0, 33, 0.5), (2, 3, 0, 44, 0.5),
                                                        (1, 1, 1, 0, 9.0), (2, 2, 1, 0, 9.0)]
        g = _from_arc_list(4, 0, 1, arcs, [INF, INF, INF, 0.0])
        o = Oracle(g)
        r = o.decode(np.zeros((1, 1), np.float32), beam=50.0, max_active=IMAX, want_path=True)
        assert r.cost == 1.5
        x_ids = [a for a in r.path_arcs.tolist() if a >= o.num_emitting]
        assert x_ids == [o.num_emitting]                    # the first epsilon arc in (state, order)
        assert r.words.tolist() == [11, 33]


def test_lower_cost_beats_lower_arc_id():
    arcs = [(0, 1, 1, 11, 1.0), (0, 2, 1, 22, 1.0), (1, 3, 1, 33, 0.75), (2, 3, 1, 44, 0.5)]
    g = _from_arc_list(4, 0, 1, arcs, [INF, INF, INF, 0.0])
    r = Oracle(g).decode(np.zeros((2, 1), np.float32), beam=50.0, max_active=IMAX)
    assert r.cost == 1.5 and r.words.tolist() == [22, 44]


# ---------------------------------------------------------------- R8: ties in the final choice
def test_final_tie_goes_to_the_lower_state():
    for first_low in (True, False):
        a1, a2 = (0, 1, 1, 11, 1.0), (0, 2, 1, 22, 1.0)
        arcs = [a1, a2] if first_low else [a2, a1]
        for fin in ([INF, 0.5, 0.5], [INF, INF, INF]):     # with final costs, and without any final state
            g = _from_arc_list(3, 0, 1, arcs, fin)
            r = Oracle(g).decode(np.zeros((1, 1), np.float32), beam=50.0, max_active=IMAX)
            assert r.words.tolist() == [11]
            assert r.reached_final == (fin[1] != INF)
            assert r.cost == (1.5 if fin[1] != INF else 1.0)


def test_final_cost_decides_before_the_state_id():
    arcs = [(0, 1, 1, 11, 1.0), (0, 2, 1, 22, 1.0)]
    g = _from_arc_list(3, 0, 1, arcs, [INF, 0.5, 0.25])
    r = Oracle(g).decode(np.zeros((1, 1), np.float32), beam=50.0, max_active=IMAX)
    assert r.words.tolist() == [22] and r.cost == 1.25
