"""GPU parity: the HIP decoder against the CPU oracle, element by element, through the C ABI.

Bar: token sets of every frame identical (size and digest; full dumps on the small
cases), word sequences bit-exact, path cost equal (bit-exact is expected; 1e-4 relative is
the stated tolerance), flags equal.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

INF = float("inf")
IMAX = 2**31 - 1


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def oracle_batch(graph, loglikes, lengths, beam, max_active, max_words=256, threads=16, boosts=None,
                 boost_fsts=None, **kw):
    from oracle import Oracle
    o = Oracle(graph)

    def one(b):
        return o.decode(loglikes[b], length=int(lengths[b]), beam=beam, max_active=max_active,
                        max_words=max_words, want_digests=True, boost=None if boosts is None else boosts[b],
                        boost_fst=None if boost_fsts is None else boost_fsts[b], **kw)
    with ThreadPoolExecutor(threads) as ex:
        return list(ex.map(one, range(len(lengths))))


def check_batch(torch, graph, loglikes, lengths, beam, max_active, max_words=256, refs=None,
                max_active_hint=None, check_counters=True, boosts=None, device_loglikes=None, cost_offset=False,
                boost_fsts=None, launch_workgroups=0, **deckw):
    from paper_2311_04996_amd import Decoder
    B, T, V = loglikes.shape
    dec = Decoder(graph, max_channels=max(B, 1), max_frames=max(T, 1), max_words=max_words,
                  max_active_hint=max_active_hint or min(max_active, 20000), record_digests=True,
                  cost_offset=cost_offset, **deckw)
    dec.set_launch_workgroups(launch_workgroups)
    ll = torch.from_numpy(np.ascontiguousarray(loglikes)).cuda() if device_loglikes is None else device_loglikes
    words, nwords, cost, flags = dec.decode_batch(ll, lengths, beam, max_active, boosts=boosts, boost_fsts=boost_fsts)
    torch.cuda.synchronize()
    words, nwords, cost, flags = words.cpu().numpy(), nwords.cpu().numpy(), cost.cpu().numpy(), flags.cpu().numpy()
    if refs is None:
        refs = oracle_batch(graph, loglikes, lengths, beam, max_active, max_words, boosts=boosts,
                            cost_offset=cost_offset, boost_fsts=boost_fsts)
    near_ties = 0
    for b, r in enumerate(refs):
        cnt, dig = dec.debug_frame_digests(b)
        assert len(cnt) == lengths[b] + 1, f"utt {b}: frames {len(cnt) - 1} != {lengths[b]}"
        bad = np.nonzero((cnt != r.digest_count) | (dig != r.digest_sum))[0]
        assert len(bad) == 0, f"utt {b}: token set differs first at frame {bad[0]}: |A|={cnt[bad[0]]} vs {r.digest_count[bad[0]]}"
        assert int(flags[b]) == r.flags, f"utt {b}: flags {flags[b]} vs {r.flags}"
        assert words[b, :nwords[b]].tolist() == r.words.tolist(), f"utt {b}: words differ"
        if np.isfinite(r.cost):
            assert cost[b] == pytest.approx(r.cost, rel=1e-4)
            near_ties += int(cost[b] != np.float32(r.cost))
        else:
            assert cost[b] == r.cost
    assert near_ties == 0, f"{near_ties} utterances with a cost that is not bit-equal"
    if check_counters:
        want = np.sum([r.counters for r in refs], axis=0)
        got = dec.get_counters()
        assert got[:7].tolist() == want[:7].tolist(), (got, want)
        assert got[7] == int(np.sum(lengths))
    dec.close()
    return refs


# ------------------------------------------------------------------------------- config 1
def test_c1_tiny_matches_oracle(torch_cuda, c1):
    check_batch(torch_cuda, c1.graph, c1.loglikes, c1.lengths, c1.beam, c1.max_active)


def test_c1_token_sets_of_every_frame(torch_cuda, c1):
    """Streaming one frame at a time and dumping the live token set after each frame."""
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder
    torch = torch_cuda
    ref = Oracle(c1.graph).decode(c1.loglikes[0], beam=c1.beam, max_active=c1.max_active, want_frames=True)
    dec = Decoder(c1.graph, max_channels=1, max_frames=100, max_active_hint=c1.max_active)
    ll = torch.from_numpy(c1.loglikes).cuda()
    dec.init_channel(0, c1.beam, c1.max_active)
    for t in range(101):
        st, co = dec.debug_get_tokens(0)
        got = sorted(zip(st.tolist(), co.view(np.uint32).tolist()))
        want = sorted(zip(ref.frames[t][0].tolist(), ref.frames[t][1].view(np.uint32).tolist()))
        assert got == want, f"frame {t}"
        if t < 100:
            dec.advance_chunk([0], ll[:, t:t + 1, :].contiguous(), [1])
    dec.close()


@pytest.mark.parametrize("beam,max_active", [(INF, IMAX), (4.0, 1000), (10.0, 37), (25.0, 3), (0.0, 10)])
def test_c1_pruning_settings(torch_cuda, c1, beam, max_active):
    check_batch(torch_cuda, c1.graph, c1.loglikes, c1.lengths, beam, max_active, max_active_hint=2000)


# ------------------------------------------------------------------------------- micro graphs
def test_micro_graphs_with_ties_and_negative_epsilon(torch_cuda):
    """Exact cost ties (dyadic weights) are broken by arc id on both sides, so even the
    backpointers, hence the words, must agree."""
    from workloads import micro_graph
    for seed in range(25):
        rng = np.random.default_rng(seed)
        V, T, B = 3, 9, 4
        g = micro_graph(seed, num_states=int(rng.integers(4, 40)), num_classes=V, max_deg=5, p_eps=0.4)
        ll = -(rng.integers(0, 40, size=(B, T, V)).astype(np.float32) / 8.0)
        lengths = rng.integers(0, T + 1, size=B).astype(np.int32)
        for beam, ma in ((INF, IMAX), (3.0, 6), (1.0, 2)):
            check_batch(torch_cuda, g, ll, lengths, beam, ma, max_active_hint=1000)


def test_greedy_ctc_on_normal_topology(torch_cuda):
    from checkers import greedy_ctc
    from workloads import ctc_loglikes, ctc_topology_graph
    V, T = 12, 80
    g = ctc_topology_graph(V)
    lengths = np.array([T, T, T], np.int32)
    ll = ctc_loglikes(0, lengths, T, V, sigma=1.5, p_blank=0.5, blank_boost=3.0, token_boost=3.0)
    for beam in (0.0, 3.0, 17.0):
        refs = check_batch(torch_cuda, g, ll, lengths, beam, IMAX, max_active_hint=1000)
        for b, r in enumerate(refs):
            words, cost = greedy_ctc(ll[b])
            assert r.words.tolist() == words.tolist() and r.cost == cost


# ------------------------------------------------------------------------------- edge cases
def _chain():
    from workloads.graphs import _from_arc_list
    arcs = [(0, 1, 2, 7, 0.5), (1, 2, 1, 0, 1.25), (2, 2, 3, 9, 0.125)]
    return _from_arc_list(3, 0, 3, arcs, [INF, INF, 0.75])


def test_empty_batch_and_zero_length(torch_cuda):
    from paper_2311_04996_amd import Decoder
    torch = torch_cuda
    g = _chain()
    dec = Decoder(g, max_channels=2, max_frames=4, max_words=4, max_active_hint=100)
    ll = torch.zeros((0, 3, 3), dtype=torch.float32, device="cuda")
    out = dec.decode_batch(ll, np.zeros(0, np.int32), 5.0, 10)
    assert out[1].numel() == 0
    dec.close()
    ll = np.array([[[-1, -2, -3], [-.5, -9, -9], [-9, -9, -.25]]] * 2, np.float32)
    check_batch(torch, g, ll, np.array([0, 3], np.int32), 100.0, 10, max_active_hint=100)


def test_dead_and_nonfinal_and_minus_inf(torch_cuda):
    from workloads.graphs import _from_arc_list
    torch = torch_cuda
    dead = _from_arc_list(2, 0, 2, [(0, 1, 1, 5, 0.0)], [INF, 0.0])
    refs = check_batch(torch, dead, np.zeros((1, 3, 2), np.float32), np.array([3], np.int32), 10.0, 10, max_active_hint=100)
    assert refs[0].dead
    nonfinal = _from_arc_list(2, 0, 1, [(0, 1, 1, 5, 1.0), (1, 1, 1, 0, 0.0)], [INF, INF])
    refs = check_batch(torch, nonfinal, np.full((1, 2, 1), -0.5, np.float32), np.array([2], np.int32), 10.0, 10, max_active_hint=100)
    assert not refs[0].reached_final
    g = _from_arc_list(3, 0, 2, [(0, 1, 1, 1, 0.0), (0, 2, 2, 2, 0.0), (1, 1, 1, 0, 0.0), (2, 2, 1, 0, 0.0)], np.zeros(3, np.float32))
    ll = np.array([[[-np.inf, -3.0], [-0.1, -0.2]]], np.float32)
    check_batch(torch, g, ll, np.array([2], np.int32), INF, IMAX, max_active_hint=100)


def test_word_truncation(torch_cuda, c1):
    refs = check_batch(torch_cuda, c1.graph, c1.loglikes, c1.lengths, c1.beam, c1.max_active, max_words=2)
    assert refs[0].truncated


def test_lattice_overflow_is_reported_not_fatal(torch_cuda, c1):
    from paper_2311_04996_amd import Decoder, FLAG_LATTICE_OVERFLOW, FLAG_DEAD, WfstError
    torch = torch_cuda
    ll = torch.from_numpy(c1.loglikes).cuda()
    dec = Decoder(c1.graph, max_channels=1, max_frames=100, max_active_hint=c1.max_active,
                  lattice_bytes_per_channel=8 * 5000)
    _, nwords, cost, flags = dec.decode_batch(ll, c1.lengths, c1.beam, c1.max_active)
    torch.cuda.synchronize()
    assert int(flags[0]) & FLAG_LATTICE_OVERFLOW and int(flags[0]) & FLAG_DEAD and int(nwords[0]) == 0
    dec.close()
    dec = Decoder(c1.graph, max_channels=1, max_frames=100, max_active_hint=c1.max_active,
                  lattice_bytes_per_channel=8 * 5000, outputs_on_host=True)
    with pytest.raises(WfstError) as e:
        dec.decode_batch(ll, c1.lengths, c1.beam, c1.max_active)
    assert e.value.code == -4
    # the channel is usable again after the failure
    dec.close()


def test_argument_errors(torch_cuda, c1):
    from paper_2311_04996_amd import Decoder, WfstError
    torch = torch_cuda
    dec = Decoder(c1.graph, max_channels=2, max_frames=50, max_active_hint=1000)
    ll = torch.from_numpy(c1.loglikes).cuda()
    with pytest.raises(WfstError) as e:
        dec.decode_batch(ll, c1.lengths, c1.beam, c1.max_active)       # 100 frames > max_frames
    assert e.value.code == -1
    with pytest.raises(WfstError) as e:
        dec.init_channel(2, 10.0, 100)
    assert e.value.code == -5
    with pytest.raises(WfstError) as e:
        dec.advance_chunk([0, 0], ll[:, :2].repeat(2, 1, 1).contiguous(), [1, 1])
    assert e.value.code == -5
    with pytest.raises(WfstError) as e:
        dec.decode_batch(ll[:, :50].contiguous(), [50], -1.0, 100)
    assert e.value.code == -1
    with pytest.raises(WfstError) as e:
        dec.set_launch_workgroups(-1)
    assert e.value.code == -1
    dec.close()


def test_host_outputs(torch_cuda, c1):
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder
    torch = torch_cuda
    dec = Decoder(c1.graph, max_channels=1, max_frames=100, max_active_hint=c1.max_active, outputs_on_host=True)
    words, nwords, cost, flags = dec.decode_batch(torch.from_numpy(c1.loglikes).cuda(), c1.lengths, c1.beam, c1.max_active)
    ref = Oracle(c1.graph).decode(c1.loglikes[0], beam=c1.beam, max_active=c1.max_active)
    assert words[0, :nwords[0]].tolist() == ref.words.tolist() and cost[0] == np.float32(ref.cost) and flags[0] == ref.flags
    w, c, f = dec.get_partial(0, finalize=True)
    assert w.tolist() == ref.words.tolist() and c == ref.cost
    dec.close()


# ------------------------------------------------------------------------------- config 2
@pytest.fixture(scope="module")
def c2_refs(c2):
    return oracle_batch(c2.graph, c2.loglikes, c2.lengths, c2.beam, c2.max_active)


def test_c2_medium_batch_matches_oracle(torch_cuda, c2, c2_refs):
    check_batch(torch_cuda, c2.graph, c2.loglikes, c2.lengths, c2.beam, c2.max_active, refs=c2_refs)


def test_c2_decoder_without_any_option(torch_cuda, c2, c2_refs):
    """A decoder with no option on (no digests, no token records, no cost offsets, no recycling, no
    boosting) runs the leanest instance of the kernel, the one the throughput is measured with:
    words, cost bits, flags and counters of the whole batch against the oracle, twice in a row."""
    from paper_2311_04996_amd import Decoder
    torch = torch_cuda
    dec = Decoder(c2.graph, max_channels=len(c2.lengths), max_frames=c2.loglikes.shape[1], max_active_hint=c2.max_active)
    ll = torch.from_numpy(c2.loglikes).cuda()
    for _ in range(2):
        dec.get_counters(reset=True)
        words, nwords, cost, flags = (t.cpu().numpy() for t in dec.decode_batch(ll, c2.lengths, c2.beam, c2.max_active))
        for b, r in enumerate(c2_refs):
            assert words[b, :nwords[b]].tolist() == r.words.tolist() and int(flags[b]) == r.flags, b
            assert cost[b] == np.float32(r.cost), b
        want = np.sum([r.counters for r in c2_refs], axis=0)
        assert dec.get_counters()[:7].tolist() == want[:7].tolist()
    dec.close()


@pytest.mark.parametrize("n_wg", [1, 5, 31, 32, 100])
def test_c2_fewer_workgroups_than_utterances(torch_cuda, c2, c2_refs, n_wg):
    """wfst_set_launch_workgroups: the launch gets n_wg workgroups, which take the 32 utterances one
    after the other from a counter on the device (each workgroup decodes several channels in a row,
    moving its pointers from one to the next).  Token sets of every frame, words, cost bits, flags
    and counters are the oracle's whatever n_wg is (32 and 100: one workgroup per utterance again)."""
    check_batch(torch_cuda, c2.graph, c2.loglikes, c2.lengths, c2.beam, c2.max_active, refs=c2_refs,
                launch_workgroups=n_wg)


def test_fewer_workgroups_with_boosting_and_lean_kernel(torch_cuda, c2, c2_refs):
    """The same through the other instances of the kernel: a decoder without any option (three
    calls in a row on one decoder, the workgroup count changed in between), and utterances that each
    have their own boosting acceptor (a workgroup loads the next channel's acceptor into LDS)."""
    from paper_2311_04996_amd import Decoder
    torch = torch_cuda
    dec = Decoder(c2.graph, max_channels=len(c2.lengths), max_frames=c2.loglikes.shape[1], max_active_hint=c2.max_active)
    ll = torch.from_numpy(c2.loglikes).cuda()
    for n_wg in (3, 0, 7):
        dec.set_launch_workgroups(n_wg)
        dec.get_counters(reset=True)
        words, nwords, cost, flags = (t.cpu().numpy() for t in dec.decode_batch(ll, c2.lengths, c2.beam, c2.max_active))
        for b, r in enumerate(c2_refs):
            assert words[b, :nwords[b]].tolist() == r.words.tolist() and int(flags[b]) == r.flags, (n_wg, b)
            assert cost[b] == np.float32(r.cost), (n_wg, b)
        want = np.sum([r.counters for r in c2_refs], axis=0)
        assert dec.get_counters()[:7].tolist() == want[:7].tolist()
    dec.close()
    from workloads import boost_fsts
    n = 6
    fsts = boost_fsts(9, n, int(c2.graph.meta["num_words"]), per_utt=100, max_len=4, score=-4.0, hot_words=40)
    lengths = np.minimum(c2.lengths[:n], 200)
    check_batch(torch_cuda, c2.graph, c2.loglikes[:n, :200], lengths, c2.beam, c2.max_active, boost_fsts=fsts,
                launch_workgroups=2)


def test_c2_alone_equals_in_batch(torch_cuda, c2, c2_refs):
    b = 5
    check_batch(torch_cuda, c2.graph, c2.loglikes[b:b + 1], c2.lengths[b:b + 1], c2.beam, c2.max_active,
                refs=c2_refs[b:b + 1])


def test_candidate_overflow_is_reported_not_fatal(torch_cuda, c2):
    """A candidate buffer far too small for the pruning settings: the utterances are flagged and
    stop (nothing faults), and the same decoder then decodes correctly with settings that fit."""
    from paper_2311_04996_amd import Decoder, FLAG_CAPACITY, FLAG_DEAD
    torch = torch_cuda
    n = 2
    ll = torch.from_numpy(np.ascontiguousarray(c2.loglikes[:n])).cuda()
    dec = Decoder(c2.graph, max_channels=n, max_frames=c2.loglikes.shape[1], max_active_hint=c2.max_active,
                  candidate_capacity=4096, record_digests=True)
    _, nwords, cost, flags = dec.decode_batch(ll, c2.lengths[:n], c2.beam, c2.max_active)
    torch.cuda.synchronize()
    for b in range(n):
        assert int(flags[b]) & FLAG_CAPACITY and int(flags[b]) & FLAG_DEAD and int(nwords[b]) == 0
    beam, max_active = 3.0, 100
    refs = oracle_batch(c2.graph, c2.loglikes[:n], c2.lengths[:n], beam, max_active)
    words, nwords, cost, flags = dec.decode_batch(ll, c2.lengths[:n], beam, max_active)
    torch.cuda.synchronize()
    for b, r in enumerate(refs):
        assert int(flags[b]) == r.flags and not int(flags[b]) & FLAG_CAPACITY
        assert words[b, :int(nwords[b])].cpu().numpy().tolist() == r.words.tolist()
        cnt, dig = dec.debug_frame_digests(b)
        assert (cnt == r.digest_count).all() and (dig == r.digest_sum).all()
    dec.close()


@pytest.mark.parametrize("chunk,n_wg", [(1, 0), (16, 0), (37, 0), (16, 3)])
def test_streaming_equals_offline(torch_cuda, c2, c2_refs, chunk, n_wg):
    """Per-stream state persists between chunks (Section 'Streaming inference'): any chunking
    gives the offline result bit for bit, and partial hypotheses depend on the frame count only.
    (n_wg = 3: the four channels of every launch are taken by three workgroups.)"""
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder
    torch = torch_cuda
    chans = [3, 0, 6, 1]                      # channel ids need not be ordered or dense
    utts = [0, 2, 4, 7]
    lens = np.minimum(c2.lengths[utts], 120 if chunk == 1 else 10**6)
    T = int(lens.max())
    dec = Decoder(c2.graph, max_channels=8, max_frames=T, max_active_hint=c2.max_active, record_digests=True)
    dec.set_launch_workgroups(n_wg)
    ll = torch.from_numpy(np.ascontiguousarray(c2.loglikes[utts, :T])).cuda()
    for ch in chans:
        dec.init_channel(ch, c2.beam, c2.max_active)
    o = Oracle(c2.graph)
    probe_at = {chunk * 2, chunk * 5}
    for t0 in range(0, T, chunk):
        nfr = np.clip(lens - t0, 0, chunk).astype(np.int32)
        block = torch.zeros((4, chunk, ll.shape[2]), device="cuda")
        block[:, :min(chunk, T - t0)] = ll[:, t0:t0 + chunk]
        dec.advance_chunk(chans, block, nfr)
        if t0 + chunk in probe_at:
            for i, ch in enumerate(chans[:2]):
                n = min(t0 + chunk, int(lens[i]))
                w, c, f = dec.get_partial(ch, finalize=False)
                r = o.decode(c2.loglikes[utts[i]], length=n, beam=c2.beam, max_active=c2.max_active, finalize=False)
                assert w.tolist() == r.words.tolist() and c == r.cost and f == r.flags
    bw, bn, bc, bf = dec.get_partial_batch(chans, finalize=True)           # all channels in one launch
    for i, ch in enumerate(chans):
        r = o.decode(c2.loglikes[utts[i]], length=int(lens[i]), beam=c2.beam, max_active=c2.max_active, want_digests=True)
        assert bw[i, :int(bn[i])].cpu().numpy().tolist() == r.words.tolist() and float(bc[i]) == r.cost and int(bf[i]) == r.flags
        cnt, dig = dec.debug_frame_digests(ch)
        assert (cnt == r.digest_count).all() and (dig == r.digest_sum).all()
        w, c, f = dec.get_partial(ch, finalize=True)
        assert w.tolist() == r.words.tolist() and c == r.cost and f == r.flags
    dec.close()


# ------------------------------------------------------------------------------- config 2, full dumps
def test_c2_token_dumps_of_every_frame(torch_cuda, c2):
    """Two utterances of config 2 streamed one frame at a time; after every frame the live token
    set is read back and compared with the oracle's dump, token by token (state, cost bits)."""
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder
    torch = torch_cuda
    utts, n_frames = [1, 9], 160
    o = Oracle(c2.graph)
    dec = Decoder(c2.graph, max_channels=2, max_frames=n_frames, max_active_hint=c2.max_active)
    ll = torch.from_numpy(np.ascontiguousarray(c2.loglikes[utts, :n_frames])).cuda()
    lens = np.minimum(c2.lengths[utts], n_frames)
    refs = [o.decode(c2.loglikes[u], length=int(n), beam=c2.beam, max_active=c2.max_active, want_frames=True)
            for u, n in zip(utts, lens)]
    for ch in range(2):
        dec.init_channel(ch, c2.beam, c2.max_active)
    for t in range(int(lens.max()) + 1):
        for ch in range(2):
            if t > lens[ch]:
                continue
            st, co = dec.debug_get_tokens(ch)
            got = np.stack([st.astype(np.int64), co.view(np.uint32).astype(np.int64)], axis=1)
            want = np.stack([refs[ch].frames[t][0].astype(np.int64),
                             refs[ch].frames[t][1].view(np.uint32).astype(np.int64)], axis=1)
            got, want = got[np.lexsort(got.T[::-1])], want[np.lexsort(want.T[::-1])]
            assert got.shape == want.shape, f"utt {utts[ch]} frame {t}: {len(got)} tokens, the oracle has {len(want)}"
            if not (got == want).all():
                i = int(np.nonzero((got != want).any(axis=1))[0][0])
                raise AssertionError(f"utt {utts[ch]} frame {t}: token {got[i].tolist()} vs the oracle's {want[i].tolist()}")
        if t < int(lens.max()):
            nfr = (t < lens).astype(np.int32)
            dec.advance_chunk([0, 1], ll[:, t:t + 1, :].contiguous(), nfr)
    dec.close()


# ------------------------------------------------------------------------------- config 3, full size
def test_c3_full_batch_every_utterance_against_oracle(torch_cuda, c3_graph):
    """The batch-256 configuration bench.py times (10 M states, 30 M arcs), decoded in one
    launch: EVERY utterance is compared with the oracle (token sets of every frame by count and
    digest, words, cost bits, flags) and the summed workload counters must be equal."""
    from paper_2311_04996_amd import Decoder
    from workloads import make_config
    torch = torch_cuda
    w = make_config("c3_large", graph=c3_graph)
    B, T, V = w.loglikes.shape
    print(f"c3_large: oracle on all {B} utterances ...", flush=True)
    refs = oracle_batch(w.graph, w.loglikes, w.lengths, w.beam, w.max_active, max_words=512)
    print("c3_large: GPU decode", flush=True)
    dec = Decoder(w.graph, max_channels=B, max_frames=T, max_words=512, max_active_hint=w.max_active,
                  record_digests=True)
    ll = torch.from_numpy(w.loglikes).cuda()
    words, nwords, cost, flags = dec.decode_batch(ll, w.lengths, w.beam, w.max_active)
    torch.cuda.synchronize()
    words, nwords, cost, flags = words.cpu().numpy(), nwords.cpu().numpy(), cost.cpu().numpy(), flags.cpu().numpy()
    not_bit_equal = 0
    for b, r in enumerate(refs):
        cnt, dig = dec.debug_frame_digests(b)
        assert len(cnt) == w.lengths[b] + 1
        bad = np.nonzero((cnt != r.digest_count) | (dig != r.digest_sum))[0]
        assert len(bad) == 0, f"utt {b}: token set differs first at frame {bad[0]}"
        assert words[b, :nwords[b]].tolist() == r.words.tolist(), f"utt {b}: words differ"
        assert int(flags[b]) == r.flags == 1, f"utt {b}: flags {flags[b]} vs {r.flags}"
        assert cost[b] == pytest.approx(r.cost, rel=1e-4)
        not_bit_equal += int(cost[b] != np.float32(r.cost))
    assert not_bit_equal == 0, f"{not_bit_equal} utterances whose cost is within 1e-4 but not bit-equal"
    want = np.sum([r.counters for r in refs], axis=0)
    got = dec.get_counters()
    assert got[:7].tolist() == want[:7].tolist(), (got, want)
    assert got[7] == int(w.lengths.sum())
    dec.close()
    # the launch configuration bench.py times: ONE decoder with three batch slots, each slot's batch on
    # its own stream, 128 workgroups per launch that take the utterances from the device-side queue;
    # six batches in flight three at a time, every result compared with the oracle again
    dec = Decoder(w.graph, max_channels=3 * B, max_frames=T, max_words=512, max_active_hint=w.max_active,
                  record_digests=True, batch_slots=3, lattice_by_length=True,
                  lattice_bytes_per_channel=int(8 * 1.5 * w.max_active * (float(w.lengths.mean()) + 2)))
    dec.set_launch_workgroups(128)
    streams = [torch.cuda.Stream() for _ in range(3)]
    torch.cuda.synchronize()
    for rnd in range(2):
        outs = [dec.decode_batch(ll, w.lengths, w.beam, w.max_active, stream=streams[k], slot=k) for k in range(3)]
        torch.cuda.synchronize()
        for k, out in enumerate(outs):
            ow, on, oc, of = (x.cpu().numpy() for x in out)
            for b, r in enumerate(refs):
                assert ow[b, :on[b]].tolist() == r.words.tolist() and oc[b] == np.float32(r.cost) and of[b] == r.flags, \
                    f"round {rnd}, slot {k}, utt {b}"
            for b in range(rnd, B, 16):
                cnt, dig = dec.debug_frame_digests(k * B + b)
                assert (cnt == refs[b].digest_count).all() and (dig == refs[b].digest_sum).all(), f"round {rnd}, slot {k}, utt {b}"
    got = dec.get_counters()
    assert got[:7].tolist() == (6 * want[:7]).tolist(), (got, want)
    dec.close()


# ------------------------------------------------------------------------------- config 4, full size
def test_c4_streaming_512_channels_against_oracle(torch_cuda, c3_graph):
    """The streaming configuration bench.py times: the config-3 graph, 512 concurrent channels,
    16-frame chunks, the partial hypotheses of all channels after EVERY chunk (alternately with
    wfst_advance_chunk + wfst_get_partial_batch and with wfst_advance_chunk_partial).  Every partial result of every channel
    (words, cost bits, flags) is compared with the oracle's decode of that prefix, and at the
    end the token sets of every frame of every channel by count and digest."""
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder
    from workloads import CONFIGS, ctc_loglikes
    torch = torch_cuda
    n, C, n_chunks = 512, 16, 6
    c = CONFIGS["c3_large"]
    g = c3_graph
    T = C * n_chunks
    beam, ma = float(c["beam"]), int(c["max_active"])
    lengths = np.full(n, T, np.int32)
    ll = ctc_loglikes(4, lengths, T, g.num_classes, **c["ll"])        # seed 4: the streaming configuration
    o = Oracle(g)
    print(f"c4_streaming: oracle on {n} channels x {n_chunks} prefixes ...", flush=True)

    def prefixes(ch):
        out = [o.decode(ll[ch], length=C * (k + 1), beam=beam, max_active=ma, max_words=512, finalize=False)
               for k in range(n_chunks - 1)]
        out.append(o.decode(ll[ch], length=T, beam=beam, max_active=ma, max_words=512, finalize=False,
                            want_digests=True))
        return out
    with ThreadPoolExecutor(16) as ex:
        refs = list(ex.map(prefixes, range(n)))
    print("c4_streaming: GPU", flush=True)
    chunks = torch.from_numpy(np.ascontiguousarray(
        ll.reshape(n, n_chunks, C, g.num_classes).transpose(1, 0, 2, 3))).cuda()
    dec = Decoder(g, max_channels=n, max_frames=T, max_words=512, max_active_hint=ma, outputs_on_host=True,
                  record_digests=True)
    chans = np.arange(n, dtype=np.int32)
    nfr = np.full(n, C, np.int32)
    dec.set_launch_workgroups(256)                                    # as bench.py: a workgroup per compute unit, channels from the queue
    dec.init_channels(chans, beam, ma)                                # one launch for the burst of new streams
    for k in range(n_chunks):
        if k % 2:                                                     # (bench.py's default: both in one launch)
            words, nwords, cost, flags = dec.advance_chunk_partial(chans, chunks[k], nfr, finalize=False)
        else:
            dec.advance_chunk(chans, chunks[k], nfr)
            words, nwords, cost, flags = dec.get_partial_batch(chans, finalize=False)
        for ch in range(n):
            r = refs[ch][k]
            assert words[ch, :nwords[ch]].tolist() == r.words.tolist(), f"chunk {k}, channel {ch}: words differ"
            assert cost[ch] == np.float32(r.cost) and int(flags[ch]) == r.flags, f"chunk {k}, channel {ch}"
    for ch in range(n):
        cnt, dig = dec.debug_frame_digests(ch)
        r = refs[ch][-1]
        assert (cnt == r.digest_count).all() and (dig == r.digest_sum).all(), f"channel {ch}: token sets differ"
    want = np.sum([refs[ch][-1].counters for ch in range(n)], axis=0)
    got = dec.get_counters()
    assert got[:7].tolist() == want[:7].tolist(), (got, want)
    dec.close()


# ------------------------------------------------------------------------------- internal paths
def test_many_duplicate_destinations(torch_cuda):
    """A small dense graph: ~50 candidates per destination state.  The candidates pre-selected
    for recombination then hold too few distinct states to decide the max-active cutoff, which
    forces the decoder's re-recombination of everything; the result must not change."""
    from workloads import ctc_loglikes, tlg_shaped_graph
    g = tlg_shaped_graph(11, 600, 30000, num_classes=33, alpha=3.0, k_max=200, p_eps=0.1, num_words=50)
    lengths = np.array([40, 25, 40], np.int32)
    ll = ctc_loglikes(11, lengths, 40, 33, sigma=2.0, p_blank=0.5, blank_boost=4.0, token_boost=3.0)
    from paper_2311_04996_amd import Decoder
    for ma in (100, 300, 550):
        check_batch(torch_cuda, g, ll, lengths, 17.0, ma, max_active_hint=2000)
    # the path under test was really taken
    dec = Decoder(g, max_channels=3, max_frames=40, max_active_hint=2000)
    dec.decode_batch(torch_cuda.from_numpy(ll).cuda(), lengths, 17.0, 550)
    assert dec.debug_phase_ticks()[15] > 0
    dec.close()


@pytest.mark.parametrize("sample", [1, 3, 64, 1000])
def test_results_do_not_depend_on_the_selection_sample(torch_cuda, c2, c2_refs, sample):
    """The pre-selection before recombination works from a sample of the candidates (one run of 64
    in 8 by default).  A coarse sample mis-estimates which candidates can survive and how many table
    passes they need: too few selected -> everything is recombined again; a pass that overfills the
    table -> the passes are planned again with twice as many.  Either way the result is the
    oracle's; with the coarse samples the second paths are really taken."""
    from paper_2311_04996_amd import Decoder
    check_batch(torch_cuda, c2.graph, c2.loglikes, c2.lengths, c2.beam, c2.max_active, refs=c2_refs,
                selection_sample=sample)
    if sample >= 64:
        dec = Decoder(c2.graph, max_channels=len(c2.lengths), max_frames=c2.loglikes.shape[1],
                      max_active_hint=c2.max_active, selection_sample=sample)
        dec.decode_batch(torch_cuda.from_numpy(c2.loglikes).cuda(), c2.lengths, c2.beam, c2.max_active)
        assert dec.debug_phase_ticks()[15] > 0
        dec.close()


def _stress_inputs(graph, T, seed, batch=2):
    from workloads import ctc_loglikes
    lengths = np.array([T, max(1, T - 3)][:batch], dtype=np.int32)
    ll = ctc_loglikes(seed, lengths, T, graph.num_classes, sigma=1.0, p_blank=0.5, blank_boost=2.0, token_boost=1.0)
    return ll, lengths


def test_more_high_degree_states_than_the_shared_list_holds(torch_cuda):
    """1,200 tokens with 600 arcs each: the list of states expanded segment by segment (512
    entries) overflows, so some are expanded by their own wave; 720 k candidates per frame for
    1,200 destinations also exercise the passes over many duplicates."""
    from workloads import dense_graph
    g = dense_graph(7, 1200, 600, 12)
    ll, lengths = _stress_inputs(g, 10, 11)
    check_batch(torch_cuda, g, ll, lengths, 30.0, 100000, max_active_hint=100000)
    check_batch(torch_cuda, g, ll, lengths, 6.0, 300, max_active_hint=100000)


def test_state_with_more_than_a_million_arcs(torch_cuda):
    """The emitting degree does not fit the packed header word: the exact degree is read."""
    from workloads import giant_state_graph
    g = giant_state_graph(8, 1_100_000, 3000, 12)
    ll, lengths = _stress_inputs(g, 8, 12)
    check_batch(torch_cuda, g, ll, lengths, 30.0, 100000, max_active_hint=131072)


def test_self_loop_candidates_that_tie_exactly_with_candidates_of_other_arcs(torch_cuda):
    """Tokens that stay on the usual self-loop of their state are never written as candidates; they
    meet the candidates of other arcs only if one of those goes to the same state.  Dyadic weights
    and log-likelihoods make the two tie exactly on cost nearly everywhere, so the arc ids decide,
    and the words (output labels sit on half of the arcs) show who won.  States with the
    self-loop alone, with more arcs after it, with epsilon arcs, with self-loops of other kinds
    (another label, a weight, an output label) and without any are all there."""
    from workloads import loop_tie_graph
    for seed, S, V in ((3, 400, 5), (4, 3000, 3), (5, 20000, 4), (6, 20000, 2)):
        g = loop_tie_graph(seed, S, V)
        rng = np.random.default_rng([seed, 77])
        T = 40
        lengths = np.array([T, T - 7, 1], np.int32)
        ll = (-0.5 * rng.integers(0, 7, size=(3, T, V))).astype(np.float32)
        for beam, ma in ((8.0, 100000), (4.0, 200), (6.0, 1500)):
            check_batch(torch_cuda, g, ll, lengths, beam, ma, max_active_hint=20000)
        boosts = [(np.arange(1, 30, 3, dtype=np.int32), np.full(10, -0.5, np.float32)),
                  (np.array([2, 5], np.int32), np.array([-1.0, 0.5], np.float32)), None]
        check_batch(torch_cuda, g, ll, lengths, 6.0, 1500, max_active_hint=20000, boosts=boosts)


def test_branchy_graph_where_no_state_has_the_self_loop_alone(torch_cuda):
    """Every state has the blank self-loop and one to three more arcs (the shape of the c3_branchy
    measurement at a tenth of its size): no token can skip the graph read, every token's
    self-loop candidate is implied, max-active binds on every frame."""
    from workloads import ctc_loglikes, random_lengths, tlg_shaped_graph
    g = tlg_shaped_graph(31, 1_000_000, 4_000_000, num_classes=129, alpha=1.8, k_max=5000, p_eps=0.2,
                         num_words=50_000, extra_lo=1, extra_hi=3)
    lengths = random_lengths(31, 12, 40, 160)
    T = int(lengths.max())
    ll = ctc_loglikes(31, lengths, T, 129, sigma=2.0, p_blank=0.65, blank_boost=6.0, token_boost=4.0)
    refs = check_batch(torch_cuda, g, ll, lengths, 17.0, 10000, max_active_hint=10000)
    assert sum(int(r.counters[5]) for r in refs) > 0.8 * int(lengths.sum())


def test_epsilon_rounds_larger_than_one_chunk_and_one_table(torch_cuda):
    """A closure round with 3,000 items and 9,000 arcs (not fused: several chunks of items, several
    table passes) after a fused round of one item with 3,000 arcs."""
    from workloads import eps_layers_graph
    g = eps_layers_graph(9, 3000, 12)
    ll, lengths = _stress_inputs(g, 10, 13)
    check_batch(torch_cuda, g, ll, lengths, 30.0, 100000, max_active_hint=20000)
    check_batch(torch_cuda, g, ll, lengths, 2.0, 500, max_active_hint=20000)


@pytest.mark.parametrize("dtype", ["float16", "bfloat16"])
def test_sixteen_bit_loglikes_equal_the_oracle_on_the_widened_values(torch_cuda, c1, c2, dtype):
    """Rows given as fp16 / bf16 are widened to fp32 when a frame is staged; everything after is
    the fp32 decoder, so the result is exactly the oracle's on the widened log-likelihoods."""
    torch = torch_cuda
    for w, n in ((c1, 1), (c2, 3)):
        ll16 = torch.from_numpy(np.ascontiguousarray(w.loglikes[:n])).to(getattr(torch, dtype))
        widened = ll16.to(torch.float32).numpy()
        assert not np.array_equal(widened, w.loglikes[:n])          # the rounding is real
        check_batch(torch, w.graph, widened, w.lengths[:n], w.beam, w.max_active,
                    max_active_hint=w.max_active, device_loglikes=ll16.cuda(), loglike_dtype=dtype)


def test_too_many_epsilon_arcs_on_one_state_is_a_bad_graph(torch_cuda):
    from paper_2311_04996_amd import Decoder, WfstError
    from workloads import eps_layers_graph
    with pytest.raises(WfstError) as e:
        Decoder(eps_layers_graph(9, 5000, 12), max_channels=1, max_frames=4)
    assert e.value.code == -2


def test_a_channel_that_lives_for_66000_frames(torch_cuda, c1):
    """A long stream: 66,000 frames of the tiny configuration in 660 chunks (costs grow to ~1e5,
    the lattice arena and the frame offsets are used far beyond an utterance's length)."""
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder
    torch = torch_cuda
    reps, T = 660, 100
    ll_host = np.tile(c1.loglikes[0], (reps, 1))
    ref = Oracle(c1.graph).decode(ll_host, beam=8.0, max_active=300, want_digests=True, max_words=64)
    dec = Decoder(c1.graph, max_channels=1, max_frames=reps * T, max_words=64, max_active_hint=300,
                  record_digests=True, lattice_bytes_per_channel=8 * 400 * (reps * T + 1))
    chunk = torch.from_numpy(c1.loglikes).cuda()
    dec.init_channel(0, 8.0, 300)
    o = Oracle(c1.graph)
    for k in range(reps):
        dec.advance_chunk([0], chunk, [T])
        if k in (4, 5, 329, 330):                 # partial results on the way (the traceback is incremental)
            w, c, f = dec.get_partial(0, finalize=False)
            r = o.decode(ll_host[:(k + 1) * T], beam=8.0, max_active=300, max_words=64, finalize=False)
            assert w.tolist() == r.words.tolist() and c == np.float32(r.cost) and f == r.flags, k
    cnt, dig = dec.debug_frame_digests(0)
    assert len(cnt) == reps * T + 1
    bad = np.nonzero((cnt != ref.digest_count) | (dig != ref.digest_sum))[0]
    assert len(bad) == 0, f"first difference at frame {bad[0]}"
    w, c, f = dec.get_partial(0, finalize=True)
    assert w.tolist() == ref.words.tolist() and c == ref.cost and f == ref.flags
    dec.close()


# ------------------------------------------------------------------------------- word boosting
def test_boost_on_micro_graphs(torch_cuda):
    """Output labels on emitting and epsilon arcs, dyadic weights and boosts (exact ties),
    a different table per utterance, one utterance without a table."""
    from workloads import micro_graph
    for seed in range(15):
        rng = np.random.default_rng(100 + seed)
        V, T, B = 3, 9, 4
        g = micro_graph(900 + seed, num_states=int(rng.integers(4, 40)), num_classes=V, max_deg=5, p_eps=0.4)
        ll = -(rng.integers(0, 40, size=(B, T, V)).astype(np.float32) / 8.0)
        lengths = rng.integers(1, T + 1, size=B).astype(np.int32)
        boosts = [(rng.choice(5, size=3, replace=False).astype(np.int32) + 1,
                   -(rng.integers(1, 9, size=3).astype(np.float32) / 4.0)) for _ in range(B)]
        boosts[1] = None
        for beam, ma in ((INF, IMAX), (3.0, 6)):
            check_batch(torch_cuda, g, ll, lengths, beam, ma, max_active_hint=1000, boosts=boosts)


def test_boost_changes_the_result_and_plain_decode_resets_it(torch_cuda, c1):
    """A boosted decode followed by a plain one on the same channel: the table must not linger."""
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder
    torch = torch_cuda
    ids = np.arange(1, 101, dtype=np.int32)
    boost = (ids, np.full(100, -2.0, np.float32))
    o = Oracle(c1.graph)
    plain = o.decode(c1.loglikes[0], beam=c1.beam, max_active=c1.max_active)
    boosted = o.decode(c1.loglikes[0], beam=c1.beam, max_active=c1.max_active, boost=boost)
    assert boosted.cost != plain.cost
    dec = Decoder(c1.graph, max_channels=1, max_frames=100, max_active_hint=c1.max_active, outputs_on_host=True)
    ll = torch.from_numpy(c1.loglikes).cuda()
    for want, b in ((boosted, [boost]), (plain, None), (boosted, [boost]), (plain, [None])):
        words, nwords, cost, flags = dec.decode_batch(ll, c1.lengths, c1.beam, c1.max_active, boosts=b)
        assert words[0, :nwords[0]].tolist() == want.words.tolist() and cost[0] == np.float32(want.cost)
    # streaming: the table is given when the stream is created
    dec.init_channel(0, c1.beam, c1.max_active, boost=boost)
    dec.advance_chunk([0], ll, [100])
    w, c, f = dec.get_partial(0, finalize=True)
    assert w.tolist() == boosted.words.tolist() and c == boosted.cost
    dec.close()


def test_boost_table_errors(torch_cuda, c1):
    from paper_2311_04996_amd import Decoder, WfstError
    dec = Decoder(c1.graph, max_channels=1, max_frames=10, max_active_hint=100)
    for bad in (([3, 3], [-1.0, -1.0]), ([0], [-1.0]), ([5], [float("nan")]),
                (np.arange(1, 1026), np.full(1025, -1.0))):
        with pytest.raises(WfstError) as e:
            dec.init_channel(0, 10.0, 100, boost=bad)
        assert e.value.code == -1
    dec.close()


def test_c5_boosted_medium_batch_matches_oracle(torch_cuda):
    """Configuration 5: the medium graph and batch, every utterance with its own table of 100
    vocabulary words at -2.0, applied on the fly (the product graph is never built)."""
    from workloads import make_config
    w = make_config("c5_boost")
    refs = check_batch(torch_cuda, w.graph, w.loglikes, w.lengths, w.beam, w.max_active, boosts=w.boosts)
    plain = oracle_batch(w.graph, w.loglikes[:4], w.lengths[:4], w.beam, w.max_active)
    assert any(r.cost != p.cost for r, p in zip(refs, plain)), "the tables must matter"


# ------------------------------------------------------------------------------- boosting acceptors with several states
def _dyadic_fst(rng, n_targets, vocab, max_len=3):
    from workloads import boost_trie, random_targets
    fst = boost_trie(random_targets(rng, n_targets, vocab, 1, max_len), -1.0)
    fst.arc_score[:] = -(rng.integers(1, 9, size=fst.num_arcs).astype(np.float32) / 4.0)
    return fst


def test_boost_fst_on_micro_graphs(torch_cuda):
    """Phrase targets over a vocabulary of 5 words: long matches, mismatches that fall back to the
    root, output labels on epsilon arcs, exact ties; hypotheses are (graph state, B state) pairs."""
    from workloads import micro_graph
    for seed in range(25):
        rng = np.random.default_rng(5000 + seed)
        V, T, B = 3, 9, 4
        g = micro_graph(1300 + seed, num_states=int(rng.integers(4, 40)), num_classes=V, max_deg=5, p_eps=0.4)
        ll = -(rng.integers(0, 40, size=(B, T, V)).astype(np.float32) / 8.0)
        lengths = rng.integers(0, T + 1, size=B).astype(np.int32)
        fsts = [_dyadic_fst(rng, int(rng.integers(1, 7)), np.arange(1, 6)) for _ in range(B)]
        fsts[1] = None
        for beam, ma in ((INF, IMAX), (3.0, 6), (1.0, 2)):
            check_batch(torch_cuda, g, ll, lengths, beam, ma, max_active_hint=1000, boost_fsts=fsts)


def test_boost_fst_token_pairs_of_every_frame(torch_cuda, c1):
    """The lexicon graph of config 1 with phrases of words that follow each other in it; streamed a
    frame at a time, every token set dumped as (graph state, B state, cost bits)."""
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder
    from workloads import boost_trie
    torch = torch_cuda
    g = c1.graph
    rng = np.random.default_rng(17)
    # word pairs and triples along arcs of the graph: a word's first arc leaves a state that another word's arcs enter
    words = np.unique(g.olabel[g.olabel > 0])
    targets = [rng.choice(words, size=int(rng.integers(1, 4))).tolist() for _ in range(60)]
    fst = boost_trie(targets, -3.0)
    assert fst.num_states > 10
    ref = Oracle(g).decode(c1.loglikes[0], beam=c1.beam, max_active=c1.max_active, boost_fst=fst, want_frames=True)
    assert any((b != 0).any() for b in ref.frames_b), "the workload must put tokens into inner states of B"
    dec = Decoder(g, max_channels=1, max_frames=100, max_active_hint=c1.max_active)
    ll = torch.from_numpy(c1.loglikes).cuda()
    dec.init_channel(0, c1.beam, c1.max_active, boost_fst=fst)
    for t in range(101):
        st, bs, co = dec.debug_get_token_pairs(0)
        got = sorted(zip(st.tolist(), bs.tolist(), co.view(np.uint32).tolist()))
        want = sorted(zip(ref.frames[t][0].tolist(), ref.frames_b[t].tolist(), ref.frames[t][1].view(np.uint32).tolist()))
        assert got == want, f"frame {t}"
        if t < 100:
            dec.advance_chunk([0], ll[:, t:t + 1, :].contiguous(), [1])
    w, c, f = dec.get_partial(0, finalize=True)
    assert w.tolist() == ref.words.tolist() and c == ref.cost and f == ref.flags
    dec.close()


def test_c5_boost_fst_medium_batch_matches_oracle(torch_cuda):
    """Config 5 as worded: config 2, every utterance composed on the fly with its own acceptor of
    100 targets of 1-4 output labels at -2.0 per matched label, failure arcs to the root."""
    from workloads import make_config
    w = make_config("c5_boost_fst")
    assert all(f.num_states > 50 for f in w.boost_fsts)
    refs = check_batch(torch_cuda, w.graph, w.loglikes, w.lengths, w.beam, w.max_active, boost_fsts=w.boost_fsts)
    plain = oracle_batch(w.graph, w.loglikes[:4], w.lengths[:4], w.beam, w.max_active)
    assert any((p.digest_sum != r.digest_sum).any() for p, r in zip(plain, refs))


def test_boost_fst_with_frequent_long_matches(torch_cuda, c2):
    """The config-2 graph with targets drawn from 40 hot words at -4.0: many hypotheses sit in inner
    states of B, so one graph state often carries several tokens."""
    from workloads import boost_fsts
    n = 6
    fsts = boost_fsts(9, n, int(c2.graph.meta["num_words"]), per_utt=100, max_len=4, score=-4.0, hot_words=40)
    lengths = np.minimum(c2.lengths[:n], 200)
    refs = check_batch(torch_cuda, c2.graph, c2.loglikes[:n, :200], lengths, c2.beam, c2.max_active, boost_fsts=fsts)
    assert sum(len(r.words) for r in refs) > 0


def test_boost_fst_streaming_equals_offline_and_errors(torch_cuda, c2):
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder, WfstError
    from workloads import BoostFst, boost_fsts
    torch = torch_cuda
    fst = boost_fsts(9, 1, int(c2.graph.meta["num_words"]), per_utt=100, max_len=4, score=-4.0, hot_words=40)[0]
    n = 90
    r = Oracle(c2.graph).decode(c2.loglikes[3], length=n, beam=c2.beam, max_active=c2.max_active, boost_fst=fst,
                                want_digests=True)
    dec = Decoder(c2.graph, max_channels=2, max_frames=n, max_active_hint=c2.max_active, record_digests=True,
                  keep_token_records=True)
    ll = torch.from_numpy(np.ascontiguousarray(c2.loglikes[3:4, :n])).cuda()
    dec.init_channel(1, c2.beam, c2.max_active, boost_fst=fst)
    for t0 in range(0, n, 16):
        k = min(16, n - t0)
        dec.advance_chunk([1], ll[:, t0:t0 + k].contiguous(), [k])
    w, c, f = dec.get_partial(1, finalize=True)
    cnt, dig = dec.debug_frame_digests(1)
    assert w.tolist() == r.words.tolist() and c == r.cost and f == r.flags
    assert (cnt == r.digest_count).all() and (dig == r.digest_sum).all()
    with pytest.raises(WfstError) as e:                       # lattices are over graph states only
        dec.get_lattice(1, ll[0], 2.0)
    assert e.value.code == -1
    many = BoostFst(5000, np.zeros(1, np.int32), np.ones(1, np.int32), np.zeros(1, np.int32), -np.ones(1, np.float32))
    with pytest.raises(WfstError) as e:                       # more states than the keys have room for
        dec.init_channel(0, 10.0, 100, boost_fst=many)
    assert e.value.code == -1
    twice = BoostFst(2, np.zeros(2, np.int32), np.array([7, 7], np.int32), np.array([1, 0], np.int32), -np.ones(2, np.float32))
    with pytest.raises(WfstError) as e:                       # not deterministic
        dec.init_channel(0, 10.0, 100, boost_fst=twice)
    assert e.value.code == -1
    dec.close()


def test_streams_set_up_together_each_with_its_own_acceptor(torch_cuda, c2):
    """wfst_init_channels_boost_fst: three streams set up in one launch, two with acceptors of their
    own and one without, advanced together with partial results in the same launch."""
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder
    from workloads import boost_fsts
    torch = torch_cuda
    fsts = boost_fsts(13, 2, int(c2.graph.meta["num_words"]), per_utt=100, max_len=4, score=-3.0, hot_words=40) + [None]
    n, pick = 64, [2, 5, 8]
    ll = torch.from_numpy(np.ascontiguousarray(c2.loglikes[pick, :n])).cuda()
    dec = Decoder(c2.graph, max_channels=4, max_frames=n, max_words=64, max_active_hint=c2.max_active, record_digests=True)
    chans = np.array([2, 0, 3], np.int32)
    dec.init_channels(chans, c2.beam, c2.max_active, boost_fsts=fsts)
    for t0 in range(0, n, 16):
        out = dec.advance_chunk_partial(chans, ll[:, t0:t0 + 16].contiguous(), [16, 16, 16], finalize=t0 + 16 == n)
    torch.cuda.synchronize()
    words, nwords, cost, flags = (t.cpu().numpy() for t in out)
    o = Oracle(c2.graph)
    for i in range(3):
        r = o.decode(c2.loglikes[pick[i]], length=n, beam=c2.beam, max_active=c2.max_active, max_words=64,
                     boost_fst=fsts[i], want_digests=True)
        cnt, dig = dec.debug_frame_digests(int(chans[i]))
        assert (cnt == r.digest_count).all() and (dig == r.digest_sum).all(), i
        assert words[i, :nwords[i]].tolist() == r.words.tolist() and cost[i] == np.float32(r.cost) and flags[i] == r.flags, i
    dec.close()


# ------------------------------------------------------------------------------- cost offsets
def test_cost_offsets_match_the_oracle_with_the_same_option(torch_cuda, c1, c2):
    """Token costs rebased after every prune step: token sets (rebased costs), words, cost and
    flags equal the oracle's with cost_offset, on the tiny configuration, micro graphs with
    ties and negative epsilon weights, boosted utterances and part of the medium batch."""
    from workloads import micro_graph
    check_batch(torch_cuda, c1.graph, c1.loglikes, c1.lengths, c1.beam, c1.max_active, cost_offset=True)
    check_batch(torch_cuda, c1.graph, c1.loglikes, c1.lengths, 4.0, 50, max_active_hint=2000, cost_offset=True)
    for seed in range(8):
        rng = np.random.default_rng(5000 + seed)
        V, T, B = 3, 9, 4
        g = micro_graph(2000 + seed, num_states=int(rng.integers(4, 40)), num_classes=V, max_deg=5, p_eps=0.4)
        ll = -(rng.integers(0, 40, size=(B, T, V)).astype(np.float32) / 8.0)
        lengths = rng.integers(1, T + 1, size=B).astype(np.int32)
        boosts = [(rng.choice(5, size=3, replace=False).astype(np.int32) + 1,
                   -(rng.integers(1, 9, size=3).astype(np.float32) / 4.0)) for _ in range(B)]
        boosts[2] = None
        for beam, ma in ((INF, IMAX), (3.0, 6)):
            check_batch(torch_cuda, g, ll, lengths, beam, ma, max_active_hint=1000, boosts=boosts, cost_offset=True)
    n = 6
    check_batch(torch_cuda, c2.graph, c2.loglikes[:n], c2.lengths[:n], c2.beam, c2.max_active, cost_offset=True)


def test_cost_offsets_in_a_streamed_channel(torch_cuda, c2):
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder
    torch = torch_cuda
    b = 1
    L = int(c2.lengths[b])
    ref = Oracle(c2.graph).decode(c2.loglikes[b], length=L, beam=c2.beam, max_active=c2.max_active,
                                  want_digests=True, cost_offset=True)
    dec = Decoder(c2.graph, max_channels=1, max_frames=L, max_active_hint=c2.max_active, record_digests=True,
                  cost_offset=True)
    ll = torch.from_numpy(c2.loglikes[b:b + 1]).cuda()
    dec.init_channel(0, c2.beam, c2.max_active)
    for t0 in range(0, L, 37):
        n = min(37, L - t0)
        dec.advance_chunk([0], ll[:, t0:t0 + n].contiguous(), [n])
    cnt, dig = dec.debug_frame_digests(0)
    assert (cnt == ref.digest_count).all() and (dig == ref.digest_sum).all()
    w, c, f = dec.get_partial(0, finalize=True)
    assert w.tolist() == ref.words.tolist() and c == np.float32(ref.cost) and f == ref.flags
    dec.close()


# ------------------------------------------------------------------------------- a sweep of small configurations
def test_random_small_configurations(torch_cuda):
    """Thirty seeded combinations of graph shape (epsilon share up to 45 %, hubs of up to 700 arcs),
    class count, beam, max-active, batch and length mix (0- and 1-frame utterances included),
    half of them with cost offsets, a third with 16-bit rows, three quarters with fewer workgroups
    than utterances (1, 2 or 3 for up to 6 utterances)."""
    from workloads import ctc_loglikes, tlg_shaped_graph
    torch = torch_cuda
    for seed in range(30):
        rng = np.random.default_rng(9100 + seed)
        S = int(rng.integers(300, 6000))
        V = int(rng.choice([2, 5, 33, 129, 700]))
        g = tlg_shaped_graph(4000 + seed, S, int(S * rng.uniform(1.5, 6.0)), num_classes=V,
                             alpha=float(rng.uniform(1.6, 3.0)), k_max=int(rng.choice([20, 200, 700])),
                             p_eps=float(rng.uniform(0.0, 0.45)), num_words=200)
        B = int(rng.integers(1, 7))
        T = int(rng.integers(1, 40))
        lengths = rng.integers(0, T + 1, size=B).astype(np.int32)
        lengths[int(rng.integers(0, B))] = T
        ll = ctc_loglikes(seed, lengths, T, V, sigma=float(rng.uniform(0.5, 3.0)), p_blank=float(rng.uniform(0.2, 0.8)),
                          blank_boost=float(rng.uniform(1, 6)), token_boost=float(rng.uniform(1, 5)))
        beam = float(rng.choice([0.5, 3.0, 9.0, 17.0, 40.0]))
        ma = int(rng.choice([1, 7, 100, 1500, 20000]))
        kw = {"cost_offset": bool(seed % 2), "launch_workgroups": (0, 1, 2, 3)[(seed // 2) % 4]}
        if seed % 3 == 0:
            dt = "float16" if seed % 2 else "bfloat16"
            dev = torch.from_numpy(ll).to(getattr(torch, dt)).cuda()
            check_batch(torch, g, dev.float().cpu().numpy(), lengths, beam, ma, max_active_hint=4000,
                        device_loglikes=dev, loglike_dtype=dt, **kw)
        else:
            check_batch(torch, g, ll, lengths, beam, ma, max_active_hint=4000, **kw)


def test_boost_tables_change_from_call_to_call_without_waiting(torch_cuda):
    """Boosted batches back to back on one decoder, a different table per utterance and per call,
    no synchronisation between the calls: the tables are staged in pinned memory that the
    previous call's copies may still be reading."""
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder
    from workloads import ctc_loglikes, tlg_shaped_graph
    torch = torch_cuda
    g = tlg_shaped_graph(77, 3000, 15000, num_classes=33, p_eps=0.2, num_words=60, p_olabel=0.5)
    B, T = 6, 30
    lengths = np.full(B, T, np.int32)
    ll = ctc_loglikes(78, lengths, T, 33, sigma=1.5, p_blank=0.5, blank_boost=3.0, token_boost=2.0)
    dev = torch.from_numpy(ll).cuda()
    rng = np.random.default_rng(79)
    calls = [[(rng.choice(60, size=20, replace=False).astype(np.int32) + 1,
               -rng.uniform(0.5, 4.0, size=20).astype(np.float32)) for _ in range(B)] for _ in range(6)]
    dec = Decoder(g, max_channels=B, max_frames=T, max_active_hint=2000)
    outs = [dec.decode_batch(dev, lengths, 12.0, 1500, boosts=bs) for bs in calls]
    torch.cuda.synchronize()
    o = Oracle(g)
    for bs, out in zip(calls, outs):
        words, nwords, cost = out[0].cpu().numpy(), out[1].cpu().numpy(), out[2].cpu().numpy()
        for b in range(B):
            r = o.decode(ll[b], beam=12.0, max_active=1500, boost=bs[b])
            assert words[b, :nwords[b]].tolist() == r.words.tolist() and cost[b] == np.float32(r.cost)
    dec.close()


def test_lattice_arena_overflow_in_a_batch_does_not_touch_the_neighbours(torch_cuda, c2):
    """An arena too small for the long utterances of the batch: they stop with the overflow flag
    (also when it strikes in the middle of an epsilon closure), and the utterances that fit -
    whose arenas lie right behind the overflowing ones - still equal the oracle."""
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder, FLAG_LATTICE_OVERFLOW
    torch = torch_cuda
    n = 8
    lengths = c2.lengths[:n].copy()
    fit = int(np.sort(lengths)[n // 2])                       # about half of them fit
    entries = int(1.05 * 9000 * (fit + 1))
    dec = Decoder(c2.graph, max_channels=n, max_frames=int(lengths.max()), max_active_hint=c2.max_active,
                  lattice_bytes_per_channel=8 * entries)
    ll = torch.from_numpy(np.ascontiguousarray(c2.loglikes[:n])).cuda()
    words, nwords, cost, flags = [t.cpu().numpy() for t in dec.decode_batch(ll, lengths, c2.beam, c2.max_active)]
    dec.close()
    o = Oracle(c2.graph)
    n_over = 0
    for b in range(n):
        if flags[b] & FLAG_LATTICE_OVERFLOW:
            n_over += 1
            assert nwords[b] == 0
            continue
        r = o.decode(c2.loglikes[b], length=int(lengths[b]), beam=c2.beam, max_active=c2.max_active)
        assert words[b, :nwords[b]].tolist() == r.words.tolist() and cost[b] == np.float32(r.cost) and flags[b] == r.flags
    assert 0 < n_over < n


def test_partial_results_after_every_chunk_equal_the_oracle_on_the_prefix(torch_cuda, c2):
    """The traceback is incremental (it stops where it meets the path of the previous one):
    after every chunk the partial hypothesis, with and without final costs, must be exactly the
    oracle's result on the frames consumed so far; also with a word limit that truncates, and
    with a caller buffer of another size (which takes the full walk)."""
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder
    torch = torch_cuda
    b = 2
    L = min(int(c2.lengths[b]), 230)
    o = Oracle(c2.graph)
    for max_words, chunk in ((256, 16), (5, 23)):
        dec = Decoder(c2.graph, max_channels=2, max_frames=L, max_words=max_words, max_active_hint=c2.max_active)
        ll = torch.from_numpy(c2.loglikes[b:b + 1, :L]).cuda()
        dec.init_channel(1, c2.beam, c2.max_active)
        for t0 in range(0, L, chunk):
            n = min(chunk, L - t0)
            dec.advance_chunk([1], ll[:, t0:t0 + n].contiguous(), [n])
            for fin in (False, True, False):
                w, c, f = dec.get_partial(1, finalize=fin)
                r = o.decode(c2.loglikes[b], length=t0 + n, beam=c2.beam, max_active=c2.max_active,
                             max_words=max_words, finalize=fin)
                assert w.tolist() == r.words.tolist() and c == np.float32(r.cost) and f == r.flags, (t0, fin)
            if t0 % (3 * chunk) == 0:            # a buffer of another size: no marks, full walk, same words
                w, c, f = dec.get_partial(1, finalize=False, cap=max_words + 3) if max_words == 5 else (None, None, None)
                if w is not None:
                    r = o.decode(c2.loglikes[b], length=t0 + n, beam=c2.beam, max_active=c2.max_active,
                                 max_words=max_words + 3, finalize=False)
                    assert w.tolist() == r.words.tolist() and f == r.flags
        dec.close()


def test_advance_and_partial_in_one_launch(torch_cuda, c2):
    """wfst_advance_chunk_partial: the frames of a chunk and the partial hypotheses of the same
    channels in one launch; after every chunk exactly the oracle's result on the frames so far, for
    channels that advance by different numbers of frames (one of them by none), device and host
    outputs, and a final call that applies the final costs."""
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder
    torch = torch_cuda
    pick = [1, 4, 6]
    L = 150
    ll = torch.from_numpy(np.ascontiguousarray(c2.loglikes[pick, :L])).cuda()
    o = Oracle(c2.graph)
    chunk = 20
    for host in (False, True):
        dec = Decoder(c2.graph, max_channels=4, max_frames=L, max_words=64, max_active_hint=c2.max_active,
                      outputs_on_host=host)
        chans = np.array([3, 0, 2], np.int32)
        dec.init_channels(chans, c2.beam, c2.max_active)
        done = np.zeros(3, np.int64)
        step = np.array([20, 13, 0], np.int32)                   # the third channel only advances every other chunk
        for k in range(6):
            nfr = step.copy()
            nfr[2] = 20 if k % 2 else 0
            buf = torch.zeros((3, chunk, c2.graph.num_classes), dtype=torch.float32, device="cuda")
            for i in range(3):
                buf[i, :nfr[i]] = ll[i, done[i]:done[i] + nfr[i]]
            fin = k == 5
            words, nwords, cost, flags = dec.advance_chunk_partial(chans, buf, nfr, finalize=fin)
            done += nfr
            if not host:
                torch.cuda.synchronize()
                words, nwords, cost, flags = (t.cpu().numpy() for t in (words, nwords, cost, flags))
            for i in range(3):
                r = o.decode(c2.loglikes[pick[i]], length=int(done[i]), beam=c2.beam, max_active=c2.max_active,
                             max_words=64, finalize=fin)
                assert words[i, :nwords[i]].tolist() == r.words.tolist(), (host, k, i)
                assert cost[i] == np.float32(r.cost) and int(flags[i]) == r.flags, (host, k, i)
            # the separate call afterwards reports the same
            w2 = dec.get_partial_batch(chans, finalize=fin)
            if not host:
                torch.cuda.synchronize()
                w2 = tuple(t.cpu().numpy() for t in w2)
            assert (w2[1] == nwords).all() and (w2[2] == cost).all() and (w2[3] == flags).all()
        dec.close()


# ------------------------------------------------------------------------------- batch slots, shared lattice memory
def test_batches_in_flight_on_one_decoder(torch_cuda, c2, c2_refs):
    """One decoder, three batch slots: three batches decoded at the same time on three streams,
    the slot's lattice memory shared out by utterance length (sized for the mean length); every
    result equals the oracle's.  Then streaming on a slot a batch decode has used."""
    from paper_2311_04996_amd import Decoder, WfstError
    torch = torch_cuda
    B, T = 8, int(c2.lengths[:24].max())
    mean_frames = float(c2.lengths[:24].mean())
    dec = Decoder(c2.graph, max_channels=3 * B, max_frames=T, max_active_hint=c2.max_active, record_digests=True,
                  batch_slots=3, lattice_by_length=True,
                  lattice_bytes_per_channel=int(8 * 1.35 * 8200 * (mean_frames + 2)))
    plain = Decoder(c2.graph, max_channels=B, max_frames=T, max_active_hint=c2.max_active)
    assert dec.device_bytes() < 3 * plain.device_bytes() * 0.75      # shared graph, arenas for the mean length
    plain.close()
    lls = [torch.from_numpy(np.ascontiguousarray(c2.loglikes[k * B:(k + 1) * B, :T])).cuda() for k in range(3)]
    streams = [torch.cuda.Stream() for _ in range(3)]
    torch.cuda.synchronize()
    for rep in range(2):
        outs = [dec.decode_batch(lls[k], c2.lengths[k * B:(k + 1) * B], c2.beam, c2.max_active, stream=streams[k], slot=k)
                for k in range(3)]
        torch.cuda.synchronize()
        for k, out in enumerate(outs):
            words, nwords, cost, flags = (x.cpu().numpy() for x in out)
            for b in range(B):
                r = c2_refs[k * B + b]
                assert words[b, :nwords[b]].tolist() == r.words.tolist() and cost[b] == np.float32(r.cost) and flags[b] == r.flags
                cnt, dig = dec.debug_frame_digests(k * B + b)
                assert (cnt == r.digest_count).all() and (dig == r.digest_sum).all(), (rep, k, b)
            assert dec.slot_kernel_ms(k) > 0
    # a channel of slot 1 as a stream: its slot's memory goes back to equal shares, the other channels
    # of that slot must be initialised again before use
    from oracle import Oracle
    ch = B + 2
    dec.init_channel(ch, c2.beam, c2.max_active)
    n = 48
    dec.advance_chunk([ch], lls[0][:1, :n].contiguous(), [n])
    w, c, f = dec.get_partial(ch, finalize=True)
    r = Oracle(c2.graph).decode(c2.loglikes[0], length=n, beam=c2.beam, max_active=c2.max_active)
    assert w.tolist() == r.words.tolist() and c == np.float32(r.cost) and f == r.flags
    with pytest.raises(WfstError) as e:
        dec.advance_chunk([B + 3], lls[0][:1, :n].contiguous(), [n])
    assert e.value.code == -5
    with pytest.raises(WfstError) as e:                          # a batch larger than a slot
        dec.decode_batch(torch.cat([lls[0], lls[1]]), c2.lengths[:2 * B], c2.beam, c2.max_active, slot=0)
    assert e.value.code == -5
    dec.close()


# ------------------------------------------------------------------------------- streams of any length
def test_recycled_lattice_stream_ten_times_the_window(torch_cuda, c2):
    """recycle_lattice: a channel streams 2,000 frames through a window of 200 frames (per-frame
    tables) and a lattice arena of about 250 frames of tokens, in chunks of 16 with a partial
    result after every chunk.  The partials (and the final result) equal the oracle's on the
    prefix, and no overflow is flagged: the arena is a ring behind what results still need."""
    from oracle import Oracle
    from paper_2311_04996_amd import Decoder, FLAG_LATTICE_OVERFLOW, FLAG_CAPACITY
    torch = torch_cuda
    window, total, chunk = 200, 2000, 16
    utts = [4, 11]
    lls = [np.concatenate([c2.loglikes[u, :c2.lengths[u]]] * (total // int(c2.lengths[u]) + 1))[:total] for u in utts]
    o = Oracle(c2.graph)
    checkpoints = [16, 208, 400, 992, 1600, 2000]
    with ThreadPoolExecutor(16) as ex:
        refs = list(ex.map(lambda a: o.decode(lls[a[0]], length=a[1], beam=c2.beam, max_active=c2.max_active,
                                              max_words=512, finalize=False),
                           [(i, n) for i in range(2) for n in checkpoints]))
    refs = {(i, n): r for (i, n), r in zip([(i, n) for i in range(2) for n in checkpoints], refs)}
    dec = Decoder(c2.graph, max_channels=2, max_frames=window, max_words=512, max_active_hint=c2.max_active,
                  recycle_lattice=True, lattice_bytes_per_channel=8 * 8200 * 250)
    dev = torch.from_numpy(np.stack(lls)).cuda()
    dec.init_channels([0, 1], c2.beam, c2.max_active)
    for t0 in range(0, total, chunk):
        n = min(chunk, total - t0)
        dec.advance_chunk([0, 1], dev[:, t0:t0 + n].contiguous(), [n, n])
        words, nwords, cost, flags = (x.cpu().numpy() for x in dec.get_partial_batch([0, 1], finalize=False))
        assert not (flags & (FLAG_LATTICE_OVERFLOW | FLAG_CAPACITY)).any(), t0
        if t0 + n in checkpoints:
            for i in range(2):
                r = refs[(i, t0 + n)]
                assert words[i, :nwords[i]].tolist() == r.words.tolist(), (i, t0 + n)
                assert cost[i] == np.float32(r.cost) and flags[i] == r.flags, (i, t0 + n)
    assert len(refs[(0, total)].words) > 40
    dec.close()


def test_recycled_lattice_reports_a_result_asked_for_too_late(torch_cuda, c2):
    """No result for longer than the ring holds: the traceback cannot reach the start any more, which
    is reported as a flag (nothing faults); a decoder whose arena holds the stream is fine."""
    from paper_2311_04996_amd import Decoder, FLAG_LATTICE_OVERFLOW, WfstError
    torch = torch_cuda
    total = 600
    u = int(np.argmax(c2.lengths))
    ll = torch.from_numpy(np.concatenate([c2.loglikes[u, :c2.lengths[u]]] * 2)[None, :total].copy()).cuda()
    dec = Decoder(c2.graph, max_channels=1, max_frames=100, max_words=64, max_active_hint=c2.max_active,
                  recycle_lattice=True, lattice_bytes_per_channel=8 * 8200 * 120)
    dec.init_channel(0, c2.beam, c2.max_active)
    for t0 in range(0, total, 100):
        dec.advance_chunk([0], ll[:, t0:t0 + 100].contiguous(), [100])
    w, c, f = dec.get_partial(0, finalize=False)
    assert f & FLAG_LATTICE_OVERFLOW and len(w) == 0 and np.isfinite(c)
    dec.close()
    with pytest.raises(WfstError) as e:                       # too little memory for two token sets
        Decoder(c2.graph, max_channels=1, max_frames=100, max_active_hint=c2.max_active, recycle_lattice=True,
                lattice_bytes_per_channel=8 * 20000)
    assert e.value.code == -1


# ------------------------------------------------------------------------------- narrow arc records
def _with_binary16_emitting_weights(g):
    """The graph the decoder decodes with narrow_arcs: emitting arcs' weights rounded to IEEE binary16."""
    from workloads.graphs import Graph
    w = g.weight.copy()
    e = g.ilabel != 0
    w[e] = w[e].astype(np.float16).astype(np.float32)
    return Graph(g.num_states, g.start_state, g.num_classes, g.row_offsets, g.next_state, g.ilabel, g.olabel, w,
                 g.final_cost, g.meta)


def test_narrow_arc_records_equal_the_oracle_on_the_rounded_weights(torch_cuda, c1, c2):
    """8-byte emitting-arc records (binary16 weights): bit-exact against the oracle fed the graph with
    the rounded weights; and the rounding is real (the plain graph gives other token sets).  Config 1,
    part of config 2 (hub states, boosting reads output labels from the full records), a dense graph
    whose states all have 600 arcs, micro graphs with ties."""
    from workloads import dense_graph, micro_graph
    for w, n, T in ((c1, 1, 100), (c2, 4, 150)):
        g16 = _with_binary16_emitting_weights(w.graph)
        assert not np.array_equal(g16.weight, w.graph.weight)
        lengths = np.minimum(w.lengths[:n], T)
        refs = oracle_batch(g16, w.loglikes[:n, :T], lengths, w.beam, w.max_active)
        check_batch(torch_cuda, w.graph, w.loglikes[:n, :T], lengths, w.beam, w.max_active, refs=refs, narrow_arcs=True)
        plain = oracle_batch(w.graph, w.loglikes[:1, :T], lengths[:1], w.beam, w.max_active)
        assert (plain[0].digest_sum != refs[0].digest_sum).any()
    from workloads import boost_tables
    g16 = _with_binary16_emitting_weights(c2.graph)
    boosts = boost_tables(5, 2, int(c2.graph.meta["num_words"]), 100, -2.0)
    lengths = np.minimum(c2.lengths[:2], 100)
    refs = oracle_batch(g16, c2.loglikes[:2, :100], lengths, c2.beam, c2.max_active, boosts=boosts)
    check_batch(torch_cuda, c2.graph, c2.loglikes[:2, :100], lengths, c2.beam, c2.max_active, refs=refs, boosts=boosts,
                narrow_arcs=True)
    g = dense_graph(7, 1200, 600, 12)
    ll, lengths = _stress_inputs(g, 10, 11)
    refs = oracle_batch(_with_binary16_emitting_weights(g), ll, lengths, 6.0, 300)
    check_batch(torch_cuda, g, ll, lengths, 6.0, 300, max_active_hint=100000, refs=refs, narrow_arcs=True)
    for seed in range(8):
        rng = np.random.default_rng(seed)
        g = micro_graph(seed, num_states=int(rng.integers(4, 40)), num_classes=3, max_deg=5, p_eps=0.4, dyadic=False)
        ll = -(rng.integers(0, 40, size=(3, 9, 3)).astype(np.float32) / 8.0)
        lengths = rng.integers(0, 10, size=3).astype(np.int32)
        refs = oracle_batch(_with_binary16_emitting_weights(g), ll, lengths, 3.0, 6)
        check_batch(torch_cuda, g, ll, lengths, 3.0, 6, max_active_hint=1000, refs=refs, narrow_arcs=True)
