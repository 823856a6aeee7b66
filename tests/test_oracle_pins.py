"""Pins for the CPU oracle: it is checked against things other than itself.

Each test names the part of the oracle (readings R1..R8 in oracle/wfst_oracle.c) it pins.
"""
import numpy as np
import pytest

from oracle import Oracle, oracle_cutoff, oracle_keep
from workloads import (ctc_loglikes, ctc_topology_graph, micro_graph, make_config,
                       permute_arcs_within_states, tlg_shaped_graph)
from workloads.graphs import Graph, _from_arc_list

from checkers import all_paths_best, greedy_ctc, resum_path, trellis_viterbi

INF = float("inf")
IMAX = 2**31 - 1


def dyadic_loglikes(seed, T, V):
    """Log-likelihood-like values that are multiples of 1/8 (sums stay exact in fp32)."""
    rng = np.random.default_rng(seed)
    return -(rng.integers(0, 40, size=(T, V)).astype(np.float32) / 8.0)


# ---------------------------------------------------------------- R2 cost formula, by hand
def test_cost_formula_hand_computed():
    """Figure 'Pseudo-code of Expand Arcs': cost + acoustic_cost[ilabel] + graph cost.
    A 3-state chain, one arc per frame, costs worked out by hand."""
    arcs = [(0, 1, 2, 7, 0.5), (1, 2, 1, 0, 1.25), (2, 2, 3, 9, 0.125)]
    g = _from_arc_list(3, 0, 3, arcs, [INF, INF, 0.75])
    ll = np.array([[-1.0, -2.0, -3.0], [-0.5, -9.0, -9.0], [-9.0, -9.0, -0.25]], dtype=np.float32)
    r = Oracle(g).decode(ll, beam=100.0, max_active=IMAX, want_path=True)
    #   frame0: 0.5 + 2.0 ; frame1: +1.25 + 0.5 ; frame2: +0.125 + 0.25 ; final 0.75
    assert r.cost == pytest.approx(0.5 + 2.0 + 1.25 + 0.5 + 0.125 + 0.25 + 0.75, abs=0)
    assert r.words.tolist() == [7, 9] and r.reached_final
    assert r.path_arcs.tolist() == [0, 1, 2]


def test_label_convention_blank_is_ilabel_one():
    """R1: ilabel k reads column k-1.  Swapping two columns must swap the outcome."""
    arcs = [(0, 1, 1, 11, 0.0), (0, 2, 2, 22, 0.0)]
    g = _from_arc_list(3, 0, 2, arcs, [INF, 0.0, 0.0])
    o = Oracle(g)
    assert o.decode(np.array([[-0.1, -5.0]], np.float32), beam=50.0).words.tolist() == [11]
    assert o.decode(np.array([[-5.0, -0.1]], np.float32), beam=50.0).words.tolist() == [22]


# ---------------------------------------------------------------- exhaustive enumeration
@pytest.mark.parametrize("seed", range(40))
def test_bruteforce_all_paths_unpruned(seed):
    """R2+R3+R6+R8 with pruning off == exact least-cost path over ALL paths."""
    rng = np.random.default_rng(1000 + seed)
    S, V, T = int(rng.integers(3, 8)), int(rng.integers(2, 4)), int(rng.integers(1, 6))
    g = micro_graph(seed, num_states=S, num_classes=V, max_deg=3, dyadic=True)
    ll = dyadic_loglikes(seed, T, V)
    best, wordsets, fin = all_paths_best(g, ll)
    r = Oracle(g).decode(ll, beam=INF, max_active=IMAX, want_path=True)
    if not np.isfinite(best):
        assert r.dead
        return
    assert r.cost == best                       # dyadic inputs: exact in fp32 and fp64
    assert r.reached_final == fin
    assert tuple(r.words.tolist()) in wordsets  # ties: any optimal path's words


@pytest.mark.parametrize("seed", range(10))
def test_bruteforce_random_weights(seed):
    g = micro_graph(500 + seed, num_states=6, num_classes=3, max_deg=3, dyadic=False)
    ll = ctc_loglikes(seed, [5], 5, 3, sigma=1.0, p_blank=0.5, blank_boost=2.0, token_boost=1.0)[0]
    best, wordsets, fin = all_paths_best(g, ll)
    r = Oracle(g).decode(ll, beam=INF, max_active=IMAX)
    assert r.cost == pytest.approx(best, rel=1e-5)
    assert r.reached_final == fin
    if len(wordsets) == 1:
        assert tuple(r.words.tolist()) in wordsets


# ---------------------------------------------------------------- fp64 trellis Viterbi on C1
def test_trellis_viterbi_c1(c1):
    g, ll = c1.graph, c1.loglikes[0]
    _, best, fin = trellis_viterbi(g, ll)
    o = Oracle(g)
    r = o.decode(ll, beam=INF, max_active=IMAX, want_path=True)
    assert r.reached_final == fin
    assert r.cost == pytest.approx(best, rel=1e-5)
    # the returned path is a real path of the graph whose fp64 cost is the optimum
    orig = [o.original_arc(a) for a in r.path_arcs]
    c32, c64, end, frames, words = resum_path(g, ll, orig)
    assert frames == ll.shape[0]
    assert c64 + float(g.final_cost[end]) == pytest.approx(best, rel=1e-5)
    assert words == r.words.tolist()


def test_unpruned_never_worse_than_pruned(c1):
    """Only inequality that is a theorem: the unpruned optimum bounds every beam."""
    o, ll = Oracle(c1.graph), c1.loglikes[0]
    opt = o.decode(ll, beam=INF, max_active=IMAX).cost
    for beam in (4.0, 8.0, 12.0, 17.0, 25.0):
        for ma in (50, 1000, IMAX):
            assert o.decode(ll, beam=beam, max_active=ma).cost >= opt - 1e-3


# ---------------------------------------------------------------- greedy CTC on the T graph
@pytest.mark.parametrize("beam", [0.0, 3.0, 17.0])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_greedy_ctc_on_normal_topology(beam, seed):
    """Figure of the 'normal' T transducer: blank is never output and a repeated token needs
    a blank in between.  T accepts every label sequence with weight 0, so for any beam the
    best path is the per-frame argmax, collapsed.  beam = 0 keeps only the best token."""
    V, T = 12, 80
    g = ctc_topology_graph(V)
    ll = ctc_loglikes(seed, [T], T, V, sigma=1.5, p_blank=0.5, blank_boost=3.0, token_boost=3.0)[0]
    top2 = np.sort(ll, axis=1)[:, -2:]
    assert (top2[:, 1] - top2[:, 0] > 1e-6).all()      # no tied maxima
    words, cost = greedy_ctc(ll)
    r = Oracle(g).decode(ll, beam=beam, max_active=IMAX)
    assert r.words.tolist() == words.tolist()
    assert r.cost == cost
    assert r.reached_final


# ---------------------------------------------------------------- R4/R5 histogram rule
def test_cutoff_beam_only_when_under_max_active():
    rng = np.random.default_rng(7)
    c = (100.0 + rng.random(500) * 30.0).astype(np.float32)
    best, k_keep, n_in, hist = oracle_cutoff(c, 17.0, 10_000)
    assert best == c.min() and k_keep == 256
    inbeam = (c - c.min()) <= np.float32(17.0)
    assert n_in == inbeam.sum() == hist.sum()
    assert [oracle_keep(float(x), best, 17.0, k_keep) for x in c] == inbeam.tolist()


def test_cutoff_exact_bin_edges():
    """beam = 16 -> bin width 1/16 exactly; cost best + j/16 sits in bin j; gap == beam clamps
    to bin 255."""
    best0 = 32.0
    c = np.array([best0 + j / 16.0 for j in range(256)] + [best0 + 16.0, best0 + 16.0625], np.float32)
    best, k_keep, n_in, hist = oracle_cutoff(c, 16.0, 10_000)
    assert best == best0 and n_in == 257 and k_keep == 256
    assert hist[:255].tolist() == [1] * 255 and hist[255] == 2
    # max_active = 100: running count first exceeds 100 at bin 100 -> bins 0..99 kept
    best, k_keep, n_in, _ = oracle_cutoff(c, 16.0, 100)
    assert k_keep == 100
    kept = [oracle_keep(float(x), best, 16.0, k_keep) for x in c]
    assert sum(kept) == 100 and kept[:100] == [True] * 100
    # max_active = 256 of 257 in beam: exceeded only in the last bin
    assert oracle_cutoff(c, 16.0, 256)[1] == 255


def test_cutoff_bin0_overflow_keeps_bin0():
    c = np.full(50, 3.5, np.float32)
    best, k_keep, n_in, hist = oracle_cutoff(c, 10.0, 7)
    assert k_keep == 1 and hist[0] == 50
    assert all(oracle_keep(3.5, best, 10.0, k_keep) for _ in range(3))
    assert not oracle_keep(3.5 + 10.0 / 256 * 1.5, best, 10.0, k_keep)


def test_cutoff_never_exceeds_max_active_unless_bin0():
    rng = np.random.default_rng(11)
    for _ in range(50):
        n = int(rng.integers(10, 3000))
        c = (rng.random(n) * rng.uniform(1, 40)).astype(np.float32)
        beam, ma = float(rng.uniform(2, 20)), int(rng.integers(1, 500))
        best, k_keep, n_in, hist = oracle_cutoff(c, beam, ma)
        kept = sum(oracle_keep(float(x), best, beam, k_keep) for x in c)
        if hist[0] <= ma:
            assert kept <= ma
        assert kept >= 1


def test_keep_is_monotone_in_cost():
    rng = np.random.default_rng(5)
    c = np.sort((rng.random(4000) * 25).astype(np.float32))
    for k_keep in (1, 17, 200, 256):
        flags = [oracle_keep(float(x), float(c[0]), 17.0, k_keep) for x in c]
        assert flags == sorted(flags, reverse=True)


# ---------------------------------------------------------------- R6 epsilon closure
def _eps_dag(seed, S=400, deg=3):
    rng = np.random.default_rng(seed)
    arcs = []
    for s in range(1, S):
        for _ in range(int(rng.integers(0, deg + 1))):
            arcs.append((s, int(rng.integers(0, s)), 0, 0, float(rng.uniform(0.0, 2.0))))
    arcs.append((0, 0, 1, 0, 0.0))
    return _from_arc_list(S, 0, 1, arcs, np.zeros(S, np.float32))


@pytest.mark.parametrize("seed", range(5))
def test_closure_equals_dijkstra(seed):
    """Non-negative epsilon weights: the closure is multi-source shortest paths, cut at the
    beam.  scipy's Dijkstra is the library routine it must reduce to."""
    from scipy.sparse import csr_matrix
    from scipy.sparse.csgraph import dijkstra
    g = _eps_dag(seed)
    S = g.num_states
    rng = np.random.default_rng(seed + 99)
    seeds = rng.choice(S, size=20, replace=False).astype(np.int32)
    c0 = rng.uniform(5.0, 7.0, size=20).astype(np.float32)   # every seed inside the beam
    x = np.nonzero(g.ilabel == 0)[0]
    src = g.src_of_arcs()[x]
    # super-source S with an edge to every seed; parallel edges: keep the lighter one
    rows = np.concatenate([src, np.full(20, S)])
    cols = np.concatenate([g.next_state[x], seeds])
    vals = np.concatenate([g.weight[x].astype(np.float64) + 1e-12, c0.astype(np.float64)])
    dense = {}
    for r_, c_, v_ in zip(rows, cols, vals):
        dense[(int(r_), int(c_))] = min(v_, dense.get((int(r_), int(c_)), np.inf))
    rr, cc = zip(*dense.keys())
    m = csr_matrix((list(dense.values()), (rr, cc)), shape=(S + 1, S + 1))
    dist = dijkstra(m, indices=S)[:S]
    best, beam = float(c0.min()), 2.5
    want = {s: dist[s] for s in range(S) if dist[s] - best <= beam}
    for order in (0, 1, 2):
        st, co, _, _ = Oracle(g).eps_closure(seeds, c0, best, beam, 256, order, seed)
        got = dict(zip(st.tolist(), co.tolist()))
        near_edge = {s for s in range(S) if abs(dist[s] - best - beam) < 1e-4}
        assert set(got) - near_edge == set(want) - near_edge
        for s, c in got.items():
            assert c == pytest.approx(dist[s], rel=1e-5)


@pytest.mark.parametrize("seed", range(6))
def test_worklist_order_does_not_matter(seed):
    """The closure is a least fixpoint: FIFO, LIFO and random worklists give identical
    token sets, including negative epsilon weights and exact ties."""
    g = micro_graph(300 + seed, num_states=30, num_classes=3, max_deg=5, p_eps=0.5, dyadic=True)
    ll = dyadic_loglikes(seed, 12, 3)
    o = Oracle(g)
    ref = o.decode(ll, beam=6.0, max_active=12, want_digests=True, want_frames=True, worklist_order=0)
    for order in (1, 2):
        r = o.decode(ll, beam=6.0, max_active=12, want_digests=True, want_frames=True,
                     worklist_order=order, order_seed=seed)
        assert r.cost == ref.cost and r.words.tolist() == ref.words.tolist()
        assert (r.digest_sum == ref.digest_sum).all() and (r.digest_count == ref.digest_count).all()
        for (s1, c1_), (s2, c2_) in zip(r.frames, ref.frames):
            assert sorted(zip(s1.tolist(), c1_.tolist())) == sorted(zip(s2.tolist(), c2_.tolist()))


# ---------------------------------------------------------------- traceback invariant
def test_traceback_cost_is_sum_of_its_arcs(c1, c2):
    for w, nb in ((c1, 1), (c2, 2)):
        o = Oracle(w.graph)
        for b in range(nb):
            ll = w.loglikes[b, :w.lengths[b]]
            r = o.decode(ll, beam=w.beam, max_active=w.max_active, want_path=True)
            orig = [o.original_arc(a) for a in r.path_arcs]
            c32, c64, end, frames, words = resum_path(w.graph, ll, orig)
            fc = np.float32(w.graph.final_cost[end]) if r.reached_final else np.float32(0)
            assert frames == len(ll)
            assert float(np.float32(np.float32(c32) + fc)) == r.cost          # bit-exact
            assert c64 + float(fc) == pytest.approx(r.cost, rel=1e-4)
            assert words == r.words.tolist()


# ---------------------------------------------------------------- invariances
def test_arc_order_within_state_changes_only_tie_breaks(c1):
    ll = c1.loglikes[0]
    a = Oracle(c1.graph).decode(ll, beam=c1.beam, max_active=c1.max_active, want_frames=True)
    g2 = permute_arcs_within_states(c1.graph, 77)
    b = Oracle(g2).decode(ll, beam=c1.beam, max_active=c1.max_active, want_frames=True)
    assert a.cost == b.cost
    for (s1, k1), (s2, k2) in zip(a.frames, b.frames):
        assert sorted(zip(s1.tolist(), k1.tolist())) == sorted(zip(s2.tolist(), k2.tolist()))


def test_digest_is_a_function_of_the_token_set(c1):
    r = Oracle(c1.graph).decode(c1.loglikes[0], beam=c1.beam, max_active=c1.max_active,
                                want_digests=True, want_frames=True)
    assert [len(s) for s, _ in r.frames] == r.digest_count.tolist()
    # distinct sets -> distinct digests (with overwhelming probability)
    assert len(set(r.digest_sum.tolist())) == len(r.digest_sum)
    # one token per state
    for s, _ in r.frames:
        assert len(set(s.tolist())) == len(s)


def test_max_active_bounds_the_pruned_set(c2):
    """Counters: recombined destinations vs stored tokens; max-active binds on this workload."""
    o = Oracle(c2.graph)
    r = o.decode(c2.loglikes[0, :60], beam=c2.beam, max_active=c2.max_active, want_digests=True)
    assert r.counters[5] > 0                      # frames where the histogram pruned
    assert r.counters[7] > r.counters[4]          # recombined destinations exceed stored tokens
    assert r.counters[3] <= r.counters[4]         # the closure only adds tokens
    assert r.digest_count.sum() == r.counters[4]


def test_words_truncation_flag(c1):
    o = Oracle(c1.graph)
    full = o.decode(c1.loglikes[0], beam=c1.beam, max_active=c1.max_active)
    assert len(full.words) > 2 and not full.truncated
    cut = o.decode(c1.loglikes[0], beam=c1.beam, max_active=c1.max_active, max_words=2)
    assert cut.truncated and cut.words.tolist() == full.words[:2].tolist()


def test_dead_utterance_when_nothing_can_be_emitted():
    g = _from_arc_list(2, 0, 2, [(0, 1, 1, 5, 0.0)], [INF, 0.0])   # state 1 has no arcs
    r = Oracle(g).decode(np.zeros((3, 2), np.float32), beam=10.0)
    assert r.dead and len(r.words) == 0 and r.cost == INF


def test_non_final_fallback():
    g = _from_arc_list(2, 0, 1, [(0, 1, 1, 5, 1.0), (1, 1, 1, 0, 0.0)], [INF, INF])
    r = Oracle(g).decode(np.full((2, 1), -0.5, np.float32), beam=10.0)
    assert not r.reached_final and r.cost == 2.0 and r.words.tolist() == [5]


def test_minus_inf_loglike_drops_the_candidate():
    g = _from_arc_list(3, 0, 2, [(0, 1, 1, 1, 0.0), (0, 2, 2, 2, 0.0), (1, 1, 1, 0, 0.0), (2, 2, 1, 0, 0.0)],
                       np.zeros(3, np.float32))
    ll = np.array([[-np.inf, -3.0], [-0.1, -0.2]], np.float32)
    r = Oracle(g).decode(ll, beam=INF, max_active=IMAX, want_digests=True)
    assert r.words.tolist() == [2] and r.digest_count.tolist() == [1, 1, 1]


# ---------------------------------------------------------------- graph validation
def test_rejects_epsilon_cycle_and_bad_labels():
    ok = [(0, 1, 0, 0, 1.0), (1, 0, 1, 0, 1.0)]
    Oracle(_from_arc_list(2, 0, 1, ok, [0.0, 0.0]))
    with pytest.raises(ValueError):
        Oracle(_from_arc_list(2, 0, 1, [(0, 1, 0, 0, 1.0), (1, 0, 0, 0, -1.0)], [0.0, 0.0]))
    with pytest.raises(ValueError):
        Oracle(_from_arc_list(2, 0, 1, [(0, 1, 2, 0, 1.0)], [0.0, 0.0]))       # label > V
    with pytest.raises(ValueError):
        Oracle(_from_arc_list(2, 0, 1, [(0, 1, 1, 0, float("nan"))], [0.0, 0.0]))


def test_generators_are_deterministic_and_well_formed():
    g1 = tlg_shaped_graph(9, 5000, 20000, num_classes=33, p_eps=0.2)
    g2 = tlg_shaped_graph(9, 5000, 20000, num_classes=33, p_eps=0.2)
    assert (g1.next_state == g2.next_state).all() and (g1.weight == g2.weight).all()
    assert abs(g1.num_arcs - 20000) < 200
    assert abs((g1.ilabel == 0).mean() - 0.2) < 0.03
    Oracle(g1)                                     # accepted: epsilon sub-graph is a DAG
    w = make_config("c1_tiny")
    assert w.loglikes.shape == (1, 100, 29)
    assert np.allclose(np.exp(w.loglikes[0].astype(np.float64)).sum(axis=1), 1.0, atol=1e-5)
