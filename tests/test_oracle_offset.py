"""Pins for the oracle's cost offsets (reading R11 in oracle/wfst_oracle.c): the option must not
change anything where fp32 is exact, and must do what it is for where fp32 is not."""
import numpy as np
import pytest

from oracle import Oracle
from workloads import ctc_topology_graph, micro_graph

from checkers import greedy_ctc, trellis_viterbi

INF = float("inf")
IMAX = 2**31 - 1


@pytest.mark.parametrize("seed", range(25))
def test_offsets_change_nothing_on_exactly_representable_costs(seed):
    """Dyadic weights and log-likelihoods: every sum and difference is exact in fp32, so rebasing
    the costs is exact too.  Words, flags, reported cost and the states of every token set are
    identical, and the stored costs of a set differ from the plain ones by one constant."""
    rng = np.random.default_rng(3000 + seed)
    V, T = 3, int(rng.integers(1, 10))
    g = micro_graph(1500 + seed, num_states=int(rng.integers(4, 40)), num_classes=V, max_deg=5, p_eps=0.4)
    ll = -(rng.integers(0, 40, size=(T, V)).astype(np.float32) / 8.0)
    o = Oracle(g)
    for beam, ma in ((INF, IMAX), (3.0, 6), (1.0, 3)):
        a = o.decode(ll, beam=beam, max_active=ma, want_frames=True)
        b = o.decode(ll, beam=beam, max_active=ma, want_frames=True, cost_offset=True)
        assert a.words.tolist() == b.words.tolist() and a.flags == b.flags
        assert a.cost == b.cost or (np.isinf(a.cost) and np.isinf(b.cost))
        assert a.counters.tolist() == b.counters.tolist()
        for (sa, ca), (sb, cb) in zip(a.frames, b.frames):
            ia, ib = np.argsort(sa), np.argsort(sb)
            assert sa[ia].tolist() == sb[ib].tolist()
            if len(sa):
                d = ca[ia].astype(np.float64) - cb[ib].astype(np.float64)
                assert (d == d[0]).all()


def test_offsets_keep_a_long_stream_precise():
    """40,000 frames at about 25 cost units per frame on the normal CTC topology, unpruned: the
    plain fp32 cost drifts away from the fp64 trellis by whole units, the rebased one stays within
    the rounding of the final sum, and only the rebased decode still finds the greedy CTC path
    (which is the exact best path on this topology): at a cost of 1e6 one fp32 ulp is 0.06,
    more than many of the per-frame differences between the classes."""
    V, T = 6, 40000
    rng = np.random.default_rng(77)
    ll = (-25.0 - rng.random((T, V)) * 3.0).astype(np.float32)
    g = ctc_topology_graph(V)
    _, ref, _ = trellis_viterbi(g, ll)
    o = Oracle(g)
    plain = o.decode(ll, beam=INF, max_active=IMAX, max_words=T)
    off = o.decode(ll, beam=INF, max_active=IMAX, max_words=T, cost_offset=True)
    err_plain, err_off = abs(plain.cost - ref), abs(off.cost - ref)
    assert ref > 9e5
    assert err_off <= 0.0625 + 1e-3 * 40            # one ulp of the fp32 result at 1e6, and the per-frame rounding of small costs
    assert err_plain > 10 * max(err_off, 0.0625)
    want, _ = greedy_ctc(ll)
    assert off.words.tolist() == want.tolist()
    assert plain.words.tolist() != want.tolist()


@pytest.mark.parametrize("seed", range(15))
def test_lattice_with_offsets_has_the_same_links_and_differences(seed):
    """Dyadic inputs: with cost offsets the lattice has the same links, and every link's cost
    exceeds its destination token's stored cost by exactly as much as without offsets."""
    rng = np.random.default_rng(3500 + seed)
    V, T = 3, int(rng.integers(1, 9))
    g = micro_graph(1700 + seed, num_states=int(rng.integers(4, 40)), num_classes=V, max_deg=5, p_eps=0.4)
    ll = -(rng.integers(0, 40, size=(T, V)).astype(np.float32) / 8.0)
    o = Oracle(g)
    for beam, ma, lb in ((INF, IMAX, INF), (3.0, 6, 1.5), (3.0, 6, 0.0)):
        a = o.lattice(ll, beam=beam, max_active=ma, lattice_beam=lb)
        b = o.lattice(ll, beam=beam, max_active=ma, lattice_beam=lb, cost_offset=True)
        def rows(L):
            diff = L.cost.astype(np.float64) - L.costs[L.dst_global()].astype(np.float64)
            return sorted(zip(L.frame.tolist(), L.states[L.src_global()].tolist(), L.arc.tolist(), diff.tolist()))
        assert rows(a) == rows(b)
