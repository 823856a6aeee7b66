"""Pins for the oracle's word boosting (paper, Section "Word boosting"): the utterance is decoded
as if the graph were TLG o B for a single-state acceptor B given as a table word id -> score."""
import os

import numpy as np
import pytest

from oracle import Oracle
from workloads import micro_graph, make_config
from workloads.graphs import Graph, _from_arc_list

from checkers import all_paths_best

INF = float("inf")
IMAX = 2**31 - 1


def composed_eagerly(g, ids, scores):
    """TLG o B materialised: B has one state, so composition only adds B's score to every arc
    whose output label is in the table."""
    b = np.zeros(int(g.olabel.max()) + 1 if g.num_arcs else 1, dtype=np.float32)
    for i, s in zip(ids, scores):
        if 0 < i < len(b):
            b[i] = s
    return Graph(g.num_states, g.start_state, g.num_classes, g.row_offsets, g.next_state, g.ilabel,
                 g.olabel, (g.weight + b[g.olabel]).astype(np.float32), g.final_cost, g.meta)


@pytest.mark.parametrize("seed", range(30))
def test_lazy_boosting_equals_eager_composition(seed):
    """Exhaustive enumeration over the eagerly composed micro graph vs the oracle's on-the-fly
    boosting, unpruned.  Dyadic weights and boosts: the two orders of addition agree exactly.
    Micro graphs carry output labels on epsilon arcs too, so both arc kinds are covered."""
    rng = np.random.default_rng(2000 + seed)
    S, V, T = int(rng.integers(3, 8)), int(rng.integers(2, 4)), int(rng.integers(1, 6))
    g = micro_graph(700 + seed, num_states=S, num_classes=V, max_deg=3, dyadic=True, neg_eps=False)
    ll = -(rng.integers(0, 40, size=(T, V)).astype(np.float32) / 8.0)
    ids = np.array([1, 3, 5], np.int32)
    scores = -(rng.integers(1, 9, size=3).astype(np.float32) / 4.0)
    best, wordsets, fin = all_paths_best(composed_eagerly(g, ids, scores), ll)
    r = Oracle(g).decode(ll, beam=INF, max_active=IMAX, boost=(ids, scores))
    if not np.isfinite(best):
        assert r.dead
        return
    assert r.cost == best and r.reached_final == fin
    assert tuple(r.words.tolist()) in wordsets


def test_two_word_table_like_the_paper_figure():
    """Figure "Example word boosting WFSA": "fish" boosted by 6, "fox" by 2 (negative scores,
    since the decoder minimises).  Three competing one-arc words; costs worked out by hand."""
    FISH, FOX, DOG = 1, 2, 3
    here = os.path.dirname(os.path.abspath(__file__))
    amounts = dict(ln.split() for ln in open(os.path.join(here, "golden", "word_boosting_wfsa.txt")) if ln[0] != "#")
    fish, fox = -float(amounts["fish"]), -float(amounts["fox"])       # boosted = negative score
    assert (fish, fox) == (-6.0, -2.0)
    arcs = [(0, 1, 2, FISH, 7.0), (0, 1, 3, FOX, 3.5), (0, 1, 4, DOG, 1.0), (1, 1, 1, 0, 0.0)]
    g = _from_arc_list(2, 0, 4, arcs, [INF, 0.0])
    ll = np.array([[-9.0, -1.0, -1.0, -1.0], [-0.5, -9.0, -9.0, -9.0]], np.float32)
    o = Oracle(g)
    plain = o.decode(ll, beam=50.0)
    assert plain.words.tolist() == [DOG] and plain.cost == 1.0 + 1.0 + 0.5
    boosted = o.decode(ll, beam=50.0, boost=([FISH, FOX], [fish, fox]))
    #   fish: 7.0 + 1.0 - 6.0 + 0.5 = 2.5 ; fox: 3.5 + 1.0 - 2.0 + 0.5 = 3.0 ; dog: 2.5 (tie with fish!)
    assert boosted.cost == 2.5
    only_fox = o.decode(ll, beam=50.0, boost=([FOX], [fox - 1.0]))
    assert only_fox.words.tolist() == [FOX] and only_fox.cost == 3.5 + 1.0 - 3.0 + 0.5


def test_absent_words_and_empty_table_change_nothing(c1):
    o, ll = Oracle(c1.graph), c1.loglikes[0]
    a = o.decode(ll, beam=c1.beam, max_active=c1.max_active, want_digests=True)
    b = o.decode(ll, beam=c1.beam, max_active=c1.max_active, want_digests=True, boost=([], []))
    c = o.decode(ll, beam=c1.beam, max_active=c1.max_active, want_digests=True, boost=([100000, 7777], [-5.0, -5.0]))
    for r in (b, c):
        assert r.cost == a.cost and r.words.tolist() == a.words.tolist()
        assert (r.digest_sum == a.digest_sum).all()


def test_larger_boost_means_more_of_the_word(c1):
    """Section "Word boosting", first limitation: a large enough boost makes the transcript
    degenerate towards the boosted word.  Without pruning this is a theorem: the optimum of
    cost(path) - m * count(path) is non-increasing in m and the count on the optimal path is
    non-decreasing; for a boost far beyond the beam width the word dominates the output."""
    o, ll = Oracle(c1.graph), c1.loglikes[0]
    word = 17
    costs, counts, lens = [], [], []
    for m in (0.0, 5.0, 10.0, 30.0, 100.0):
        r = o.decode(ll, beam=INF, max_active=IMAX, boost=([word], [-m]))
        costs.append(r.cost); counts.append(int((r.words == word).sum())); lens.append(len(r.words))
    assert counts[0] == 0
    assert all(c1_ >= c2_ - 1e-3 for c1_, c2_ in zip(costs, costs[1:]))
    assert all(n1 <= n2 for n1, n2 in zip(counts, counts[1:]))
    assert counts[-1] >= 3 and counts[-1] / lens[-1] > 0.5


def test_boosted_traceback_cost_includes_the_scores(c1):
    from checkers import resum_path
    o, ll = Oracle(c1.graph), c1.loglikes[0]
    ids = np.arange(1, 60, dtype=np.int32)
    sc = np.full(len(ids), -2.0, np.float32)
    r = o.decode(ll, beam=c1.beam, max_active=c1.max_active, boost=(ids, sc), want_path=True)
    orig = [o.original_arc(a) for a in r.path_arcs]
    c32, c64, end, frames, words = resum_path(c1.graph, ll, orig)
    nboost = sum(1 for wd in words if wd < 60)
    assert words == r.words.tolist() and nboost > 0
    assert c64 - 2.0 * nboost + float(c1.graph.final_cost[end]) == pytest.approx(r.cost, rel=1e-5)
