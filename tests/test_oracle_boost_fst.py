"""Pins for the oracle's boosting acceptor with several states (reading R12 in
oracle/wfst_oracle.c; paper, Section "Word boosting": decode as if the graph were TLG o B, and the
figure "Example word boosting WFSA" with its failure arc).

What holds the oracle here, none of it the oracle itself:
  * a target of one label per word is the paper's one-state B: equal to the table path bit for bit;
  * exhaustive enumeration of all paths of micro graphs, each path scored by running the acceptor
    over its output labels in plain Python (the rule restated below from the reading);
  * the product TLG o B materialised state by state in plain Python and decoded WITHOUT boosting:
    identical token sets under pruning;
  * hand-computed sequences (match, mismatch -> root, retry at the root, restart after a target).
"""
import numpy as np
import pytest

from oracle import Oracle
from workloads import BoostFst, boost_trie, micro_graph, random_targets
from workloads.graphs import Graph, _from_arc_list

from checkers import all_paths

INF = float("inf")
IMAX = 2**31 - 1


# ---------------------------------------------------------------- the rule, restated for the checks
def step(fst, b, o):
    """(new B state, score or None) for a token in B state b taking output label o != 0."""
    def arc(state):
        hit = np.nonzero((fst.arc_from == state) & (fst.arc_label == o))[0]
        return int(hit[0]) if len(hit) else None
    i = arc(b)
    if i is None and b != 0:
        i = arc(0)                       # failure arc to the root, the label is tried once more there
    if i is None:
        return 0, None
    return int(fst.arc_to[i]), float(fst.arc_score[i])


def score_of_labels(fst, labels):
    b, total = 0, 0.0
    for o in labels:
        b, sc = step(fst, b, o)
        total += sc or 0.0
    return total


def product_graph(g, fst):
    """TLG o B with product state s * nB + b (so the final tie 'lower graph state, then lower B
    state' is 'lower product state').  Every arc keeps its labels; its weight gains B's score."""
    nB = fst.num_states
    arcs = []
    for s in range(g.num_states):
        for b in range(nB):
            for a in g.arcs_of(s):
                o = int(g.olabel[a])
                nb, sc = (b, None) if o == 0 else step(fst, b, o)
                arcs.append((s * nB + b, int(g.next_state[a]) * nB + nb, int(g.ilabel[a]), o,
                             float(g.weight[a]) + (sc or 0.0)))
    final = np.repeat(g.final_cost, nB)
    return _from_arc_list(g.num_states * nB, g.start_state * nB, g.num_classes, arcs, final)


def dyadic_fst(rng, n_targets, vocab, max_len=3):
    fst = boost_trie(random_targets(rng, n_targets, vocab, 1, max_len), -1.0)
    fst.arc_score[:] = -(rng.integers(1, 9, size=fst.num_arcs).astype(np.float32) / 4.0)
    return fst


# ---------------------------------------------------------------- hand-computed sequences
def _chain(labels, weights=None):
    """One path: state i --(class 1, olabel labels[i])--> i + 1, weight 1 each."""
    n = len(labels)
    arcs = [(i, i + 1, 1, int(o), 1.0 if weights is None else weights[i]) for i, o in enumerate(labels)]
    fin = [INF] * n + [0.0]
    return _from_arc_list(n + 1, 0, 1, arcs, fin), np.zeros((n, 1), np.float32)


A, B_, C_, D = 1, 2, 3, 4


@pytest.mark.parametrize("labels,want", [
    ([A, B_], -3.0),            # target [A, B]: -1 for A, -2 for B
    ([A, C_, B_], -1.0),        # A matches; C fails -> root, no arc on C there; B at the root: none
    ([A, D], -1.0 - 4.0),       # A matches; D has no arc after A -> root, retried there: target [D] = -4
    ([A, A, B_], -1.0 - 1.0 - 2.0),   # second A fails after A -> root, retried: A again, then B
    ([A, B_, B_], -3.0),        # after the complete target the next label starts at the root: no arc on B
    ([A, B_, A, B_], -6.0),     # two complete targets in a row
    ([B_, 0, A, 0, B_], -3.0),  # arcs without output label leave B where it is
    ([C_, C_], 0.0),
])
def test_hand_computed_sequences(labels, want):
    fst = BoostFst(2, np.array([0, 1, 0], np.int32), np.array([A, B_, D], np.int32), np.array([1, 0, 0], np.int32),
                   np.array([-1.0, -2.0, -4.0], np.float32))
    g, ll = _chain(labels)
    r = Oracle(g).decode(ll, beam=INF, max_active=IMAX, boost_fst=fst)
    assert r.cost == len(labels) + want
    assert r.words.tolist() == [o for o in labels if o]
    assert score_of_labels(fst, [o for o in labels if o]) == want        # the restated rule agrees with the hand


def test_tokens_in_different_b_states_do_not_recombine():
    """Two paths into graph state 3, one having matched A (B state 1), one not: both tokens live,
    and the dearer one wins in the end because only it can complete the target."""
    fst = BoostFst(2, np.array([0, 1], np.int32), np.array([A, B_], np.int32), np.array([1, 0], np.int32),
                   np.array([-0.5, -8.0], np.float32))
    arcs = [(0, 1, 1, A, 3.0), (0, 2, 1, C_, 1.0), (1, 3, 1, 0, 1.0), (2, 3, 1, 0, 1.0), (3, 4, 1, B_, 1.0)]
    g = _from_arc_list(5, 0, 1, arcs, [INF, INF, INF, INF, 0.0])
    ll = np.zeros((3, 1), np.float32)
    r = Oracle(g).decode(ll, beam=INF, max_active=IMAX, boost_fst=fst, want_frames=True)
    assert sorted(zip(r.frames[2][0].tolist(), r.frames_b[2].tolist(), r.frames[2][1].tolist())) == \
        [(3, 0, 2.0), (3, 1, 3.5)]
    assert r.words.tolist() == [A, B_] and r.cost == 3.0 - 0.5 + 1.0 + 1.0 - 8.0
    plain = Oracle(g).decode(ll, beam=INF, max_active=IMAX)
    assert plain.words.tolist() == [C_, B_] and plain.cost == 3.0


def test_final_tie_lower_graph_state_then_lower_b_state():
    fst = BoostFst(2, np.array([0, 1], np.int32), np.array([A, B_], np.int32), np.array([1, 0], np.int32),
                   np.array([-1.0, -1.0], np.float32))
    # both arcs reach state 1 at cost 1: one over A (weight 2 - 1) into B state 1, one over C into the root
    for order in ((A, 2.0, C_, 1.0), (C_, 1.0, A, 2.0)):
        arcs = [(0, 1, 1, order[0], order[1]), (0, 1, 1, order[2], order[3])]
        g = _from_arc_list(2, 0, 1, arcs, [INF, 0.0])
        r = Oracle(g).decode(np.zeros((1, 1), np.float32), beam=INF, max_active=IMAX, boost_fst=fst, want_frames=True)
        assert sorted(r.frames_b[1].tolist()) == [0, 1] and r.cost == 1.0
        assert r.words.tolist() == [C_]                     # the token in the root of B


def test_same_arc_taken_in_two_b_states_lower_source_b_state_wins():
    """Tokens (state 3, root) and (state 3, B state 1) at equal cost both take the arc 3 -> 4 whose
    label C matches nowhere, so both land in (4, root) with the same cost and the same arc id:
    the hypothesis that came out of the lower B state is kept.  Emitting and epsilon variant, and
    both orders of creation of the two tokens."""
    fst = BoostFst(2, np.array([0, 1], np.int32), np.array([A, B_], np.int32), np.array([1, 0], np.int32),
                   np.array([-1.0, -8.0], np.float32))
    for eps in (False, True):
        for first_a in (True, False):
            via_a, via_d = (0, 1, 1, A, 2.0), (0, 2, 1, D, 1.0)          # A: 2 - 1 = 1, into B state 1; D: 1, root
            arcs = ([via_a, via_d] if first_a else [via_d, via_a]) + \
                [(1, 3, 1, 0, 1.0), (2, 3, 1, 0, 1.0), (3, 4, 0 if eps else 1, C_, 1.0)]
            if eps:
                arcs.append((4, 4, 1, 0, 0.0))
            g = _from_arc_list(5, 0, 1, arcs, [INF, INF, INF, INF, 0.0])
            r = Oracle(g).decode(np.zeros((3, 1), np.float32), beam=INF, max_active=IMAX, boost_fst=fst)
            assert r.cost == 3.0 and r.words.tolist() == [D, C_]


# ---------------------------------------------------------------- one label per target = the table
def test_single_label_targets_equal_the_table_path(c1, c2):
    """Targets of one label: B is the paper's one-state acceptor, a self-loop per word.  Token sets,
    words and cost are those of the table path, bit for bit, under pruning."""
    for w, n_utt, frames in ((c1, 1, 100), (c2, 2, 60)):
        o = Oracle(w.graph)
        rng = np.random.default_rng(5)
        nw = int(w.graph.olabel.max())
        ids = rng.choice(nw, size=min(100, nw), replace=False).astype(np.int32) + 1
        sc = -(rng.integers(1, 17, size=len(ids)).astype(np.float32) / 4.0)
        fst = BoostFst(1, np.zeros(len(ids), np.int32), ids, np.zeros(len(ids), np.int32), sc)
        assert boost_trie([[i] for i in ids], -2.0).num_states == 1
        for b in range(n_utt):
            ll = w.loglikes[b, :frames]
            t = o.decode(ll, beam=w.beam, max_active=w.max_active, boost=(ids, sc), want_digests=True)
            f = o.decode(ll, beam=w.beam, max_active=w.max_active, boost_fst=fst, want_digests=True)
            assert f.cost == t.cost and f.words.tolist() == t.words.tolist() and f.flags == t.flags
            assert (f.digest_sum == t.digest_sum).all() and (f.digest_count == t.digest_count).all()
            assert f.counters.tolist() == t.counters.tolist()
            plain = o.decode(ll, beam=w.beam, max_active=w.max_active, want_digests=True)
            assert (plain.digest_sum != f.digest_sum).any()   # the boosts were felt


def test_two_word_acceptor_of_the_paper_figure():
    """Figure "Example word boosting WFSA": one state, a self-loop per boosted word, and the failure
    arc for every other word.  Same numbers as the table test: fish -6, fox -2."""
    FISH, FOX, DOG = 1, 2, 3
    arcs = [(0, 1, 2, FISH, 7.0), (0, 1, 3, FOX, 3.5), (0, 1, 4, DOG, 1.0), (1, 1, 1, 0, 0.0)]
    g = _from_arc_list(2, 0, 4, arcs, [INF, 0.0])
    ll = np.array([[-9.0, -1.0, -1.0, -1.0], [-0.5, -9.0, -9.0, -9.0]], np.float32)
    fst = BoostFst(1, np.zeros(2, np.int32), np.array([FISH, FOX], np.int32), np.zeros(2, np.int32),
                   np.array([-6.0, -3.0], np.float32))
    r = Oracle(g).decode(ll, beam=50.0, boost_fst=fst)
    assert r.words.tolist() == [FOX] and r.cost == 3.5 + 1.0 - 3.0 + 0.5


# ---------------------------------------------------------------- exhaustive enumeration
@pytest.mark.parametrize("seed", range(40))
def test_bruteforce_all_paths_with_acceptor(seed):
    """Unpruned decode == minimum over ALL paths of (path cost + B's score of its output labels).
    Micro graphs: 5 words, output labels on emitting and epsilon arcs, exact ties, dyadic values."""
    rng = np.random.default_rng(3000 + seed)
    S, V, T = int(rng.integers(3, 8)), int(rng.integers(2, 4)), int(rng.integers(1, 6))
    g = micro_graph(900 + seed, num_states=S, num_classes=V, max_deg=3, dyadic=True, neg_eps=seed % 2 == 0)
    ll = -(rng.integers(0, 40, size=(T, V)).astype(np.float32) / 8.0)
    fst = dyadic_fst(rng, int(rng.integers(1, 5)), np.arange(1, 6))
    fin = g.final_cost.astype(np.float64)
    ends = []
    for arcs, (cost, end) in all_paths(g, ll).items():
        labels = [int(g.olabel[a]) for a in arcs if g.olabel[a] != 0]
        ends.append((cost + score_of_labels(fst, labels), end, tuple(labels)))
    r = Oracle(g).decode(ll, beam=INF, max_active=IMAX, boost_fst=fst)
    if not ends:
        assert r.dead
        return
    finals = [(c + fin[e], wd) for c, e, wd in ends if np.isfinite(fin[e])]
    pool = finals if finals else [(c, wd) for c, _, wd in ends]
    best = min(c for c, _ in pool)
    assert r.cost == best and r.reached_final == bool(finals)
    assert tuple(r.words.tolist()) in {wd for c, wd in pool if c == best}


# ---------------------------------------------------------------- the product, materialised
@pytest.mark.parametrize("seed", range(30))
def test_lazy_composition_equals_the_materialised_product(seed):
    """Decode (graph, B) on the fly vs decode the explicit product graph with no boosting, WITH
    pruning: the same token sets (graph state, B state, cost) after every frame and the same cost.
    (Arc numbering differs between the two graphs, so exact ties may pick other words.)"""
    rng = np.random.default_rng(4000 + seed)
    S, V, T = int(rng.integers(4, 30)), 3, int(rng.integers(2, 9))
    g = micro_graph(1100 + seed, num_states=S, num_classes=V, max_deg=4, p_eps=0.35, dyadic=True, neg_eps=False)
    ll = -(rng.integers(0, 40, size=(T, V)).astype(np.float32) / 8.0)
    fst = dyadic_fst(rng, int(rng.integers(2, 7)), np.arange(1, 6))
    nB = fst.num_states
    P = product_graph(g, fst)
    for beam, ma in ((INF, IMAX), (4.0, 8), (2.0, 3)):
        lazy = Oracle(g).decode(ll, beam=beam, max_active=ma, boost_fst=fst, want_frames=True)
        eager = Oracle(P).decode(ll, beam=beam, max_active=ma, want_frames=True)
        assert lazy.cost == eager.cost and lazy.flags == eager.flags
        for t in range(T + 1):
            a = sorted(zip(lazy.frames[t][0].tolist(), lazy.frames_b[t].tolist(), lazy.frames[t][1].tolist()))
            b = sorted((p // nB, p % nB, c) for p, c in zip(eager.frames[t][0].tolist(), eager.frames[t][1].tolist()))
            assert a == b, f"frame {t}"
        assert lazy.counters[[0, 1, 3, 4, 5, 6, 7]].tolist() == eager.counters[[0, 1, 3, 4, 5, 6, 7]].tolist()


def test_acceptor_is_validated():
    g, ll = _chain([A, B_])
    o = Oracle(g)
    bad = [BoostFst(2, np.array([0, 0], np.int32), np.array([A, A], np.int32), np.array([1, 0], np.int32),
                    np.array([-1.0, -1.0], np.float32)),                       # not deterministic
           BoostFst(1, np.array([0], np.int32), np.array([A], np.int32), np.array([1], np.int32),
                    np.array([-1.0], np.float32)),                             # destination out of range
           BoostFst(1, np.array([0], np.int32), np.array([0], np.int32), np.array([0], np.int32),
                    np.array([-1.0], np.float32))]                             # label 0
    for fst in bad:
        with pytest.raises(RuntimeError):
            o.decode(ll, beam=INF, max_active=IMAX, boost_fst=fst)
