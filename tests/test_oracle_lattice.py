"""Pins for the oracle's lattice links (reading R10 in oracle/wfst_oracle.c).

The paper does not define its lattice, so these pin the definition this build takes against
what it implies: on unpruned micro graphs the lattice must hold exactly the paths of the graph
(exhaustive enumeration), the lattice-beam rule must agree with an independent dense fp64
trellis, and under any pruning the decoder's own best path must run through links of
difference 0.
"""
import numpy as np
import pytest

from oracle import Oracle
from workloads import micro_graph
from workloads.graphs import Graph

from checkers import all_paths, trellis_alphas

INF = float("inf")
IMAX = 2**31 - 1


def dyadic_loglikes(seed, T, V):
    rng = np.random.default_rng(seed)
    return -(rng.integers(0, 40, size=(T, V)).astype(np.float32) / 8.0)


def start_at_last_state(g):
    """The same arcs with the highest state as start state: micro graphs send epsilon arcs to
    lower-numbered states only, so this start state can have epsilon arcs (A_0 gets links)."""
    return Graph(g.num_states, g.num_states - 1, g.num_classes, g.row_offsets, g.next_state, g.ilabel,
                 g.olabel, g.weight, g.final_cost, dict(g.meta or {}))


def lattice_paths(o, L, g, T):
    """All paths through the lattice from the start token to any token of A_T, as tuples of
    arc indices into g's arrays."""
    nxt = {}
    for s, d, a in zip(L.src_global().tolist(), L.dst_global().tolist(), L.arc.tolist()):
        nxt.setdefault(s, []).append((d, o.original_arc(a)))
    start = [i for i in range(int(L.set_off[0]), int(L.set_off[1])) if L.states[i] == g.start_state]
    assert len(start) == 1
    last = (int(L.set_off[T]), int(L.set_off[T + 1]))
    out = set()

    def rec(tok, arcs):
        if last[0] <= tok < last[1]:
            out.add(arcs)
        for d, a in nxt.get(tok, ()):
            rec(d, arcs + (a,))

    rec(start[0], ())
    return out


@pytest.mark.parametrize("seed", range(30))
def test_unpruned_lattice_holds_exactly_the_paths_of_the_graph(seed):
    rng = np.random.default_rng(7000 + seed)
    S, V, T = int(rng.integers(3, 8)), int(rng.integers(2, 4)), int(rng.integers(1, 5))
    g = micro_graph(300 + seed, num_states=S, num_classes=V, max_deg=3, dyadic=True, p_eps=0.3 + 0.2 * (seed % 2))
    if seed % 2:
        g = start_at_last_state(g)
    ll = dyadic_loglikes(seed, T, V)
    o = Oracle(g)
    L = o.lattice(ll, beam=INF, max_active=IMAX, lattice_beam=INF)
    want = set(all_paths(g, ll).keys())
    got = lattice_paths(o, L, g, T)
    assert got == want
    # every link starts and ends where its arc does, in the right frame
    src_state, dst_state = L.states[L.src_global()], L.states[L.dst_global()]
    srcs = g.src_of_arcs()
    for k in range(len(L.arc)):
        a = o.original_arc(int(L.arc[k]))
        assert srcs[a] == src_state[k] and g.next_state[a] == dst_state[k]
        emit = g.ilabel[a] != 0
        f_src = np.searchsorted(L.set_off, L.src_global()[k], side="right") - 1
        assert f_src == L.frame[k] - int(emit)


@pytest.mark.parametrize("seed", range(20))
@pytest.mark.parametrize("lattice_beam", [0.0, 0.5, 1.5, 4.0])
def test_lattice_beam_rule_against_dense_trellis(seed, lattice_beam):
    """Unpruned, dyadic costs (exact in fp32 and fp64): the stored token costs are the trellis
    minima, so a link exists iff alpha(src) + arc cost - alpha(dst) <= lattice_beam."""
    rng = np.random.default_rng(8000 + seed)
    S, V, T = int(rng.integers(4, 20)), 3, int(rng.integers(1, 7))
    g = micro_graph(600 + seed, num_states=S, num_classes=V, max_deg=4, dyadic=True, p_eps=0.3)
    if seed % 2:
        g = start_at_last_state(g)
    ll = dyadic_loglikes(50 + seed, T, V)
    o = Oracle(g)
    L = o.lattice(ll, beam=INF, max_active=IMAX, lattice_beam=lattice_beam)
    al = trellis_alphas(g, ll)
    srcs = g.src_of_arcs()
    want = set()
    for t in range(T + 1):
        for a in range(len(g.ilabel)):
            il, s, d, w = int(g.ilabel[a]), int(srcs[a]), int(g.next_state[a]), float(g.weight[a])
            if il == 0:
                c = al[t][s] + w
            elif t > 0:
                c = al[t - 1][s] + w - float(ll[t - 1, il - 1])
            else:
                continue
            if np.isfinite(c) and np.isfinite(al[t][d]) and c - al[t][d] <= lattice_beam:
                want.add((t, a))
    got = {(int(f), o.original_arc(int(a))) for f, a in zip(L.frame, L.arc)}
    assert got == want
    assert len(got) == len(L.arc)               # no link listed twice
    # link costs are the cost through the arc
    for k in range(len(L.arc)):
        a = o.original_arc(int(L.arc[k])); t = int(L.frame[k]); il = int(g.ilabel[a])
        c = al[t][srcs[a]] + float(g.weight[a]) if il == 0 else al[t - 1][srcs[a]] + float(g.weight[a]) - float(ll[t - 1, il - 1])
        assert float(L.cost[k]) == c


@pytest.mark.parametrize("seed", range(10))
def test_best_path_runs_through_links_of_difference_zero(seed, c1):
    """Under real pruning: the decoder's best path is a chain of links whose cost equals the
    destination token's stored cost, whatever the lattice beam (0 included)."""
    rng = np.random.default_rng(9000 + seed)
    if seed == 0:
        g, ll, beam, ma = c1.graph, c1.loglikes[0], c1.beam, c1.max_active
    else:
        V, T = 3, int(rng.integers(2, 9))
        g = micro_graph(900 + seed, num_states=int(rng.integers(5, 40)), num_classes=V, max_deg=5, p_eps=0.4)
        ll = dyadic_loglikes(seed, T, V)
        beam, ma = 3.0, 6
    o = Oracle(g)
    L = o.lattice(ll, beam=beam, max_active=ma, lattice_beam=0.0)
    r = L.result
    if r.dead:
        return
    links = {}
    for k, (s, d, a) in enumerate(zip(L.src_global().tolist(), L.dst_global().tolist(), L.arc.tolist())):
        links[(s, a)] = (d, k)
    tok = [i for i in range(int(L.set_off[0]), int(L.set_off[1])) if L.states[i] == g.start_state][0]
    for a in r.path_arcs.tolist():
        assert (tok, a) in links, "a best-path arc is missing from the lattice"
        d, k = links[(tok, a)]
        assert L.cost[k] == L.costs[d]
        tok = d
    assert tok >= L.set_off[len(ll)]            # ended in the last set
    # and no link is cheaper than the token it enters (the closure is a fixpoint)
    assert (L.cost >= L.costs[L.dst_global()]).all()


def test_links_grow_with_the_lattice_beam(c1):
    o = Oracle(c1.graph)
    prev = None
    for lb in (0.0, 1.0, 4.0, INF):
        L = o.lattice(c1.loglikes[0], beam=c1.beam, max_active=c1.max_active, lattice_beam=lb)
        cur = set(zip(L.frame.tolist(), L.src.tolist(), L.arc.tolist()))
        assert len(cur) == len(L.arc)
        if prev is not None:
            assert prev <= cur
        prev = cur
    assert len(prev) > len(L.states)            # a real lattice: more links than tokens


@pytest.mark.parametrize("seed", range(15))
def test_boosted_lattice_equals_the_lattice_of_the_composed_graph(seed):
    """Word boosting on the fly (scores added on arcs whose output label is in the table) against
    the same graph with the scores added to the arc weights beforehand: same token sets, same
    links, same costs.  Dyadic values, so both orders of addition are exact."""
    rng = np.random.default_rng(9500 + seed)
    V, T = 3, int(rng.integers(1, 8))
    g = micro_graph(800 + seed, num_states=int(rng.integers(4, 30)), num_classes=V, max_deg=4, dyadic=True,
                    p_eps=0.35, neg_eps=False)
    ll = dyadic_loglikes(200 + seed, T, V)
    ids = np.array([1, 3, 5], np.int32)
    scores = -(rng.integers(1, 9, size=3).astype(np.float32) / 4.0)
    b = np.zeros(int(g.olabel.max()) + 1, np.float32)
    b[ids[ids < len(b)]] = scores[ids < len(b)]
    g2 = Graph(g.num_states, g.start_state, V, g.row_offsets, g.next_state, g.ilabel, g.olabel,
               (g.weight + b[g.olabel]).astype(np.float32), g.final_cost, {})
    for beam, ma, lb in ((INF, IMAX, INF), (3.0, 6, 1.0)):
        o1, o2 = Oracle(g), Oracle(g2)
        L1 = o1.lattice(ll, beam=beam, max_active=ma, lattice_beam=lb, boost=(ids, scores))
        L2 = o2.lattice(ll, beam=beam, max_active=ma, lattice_beam=lb)
        assert L1.set_off.tolist() == L2.set_off.tolist()
        key = lambda L, o: sorted((int(f), o.original_arc(int(a)), float(c)) for f, a, c in zip(L.frame, L.arc, L.cost))
        assert key(L1, o1) == key(L2, o2)
        assert L1.result.words.tolist() == L2.result.words.tolist() and L1.result.cost == L2.result.cost
