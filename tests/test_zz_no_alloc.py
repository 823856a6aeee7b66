"""The entry point that allocates nothing (wfst_get_lattice_noalloc) against the entry point it is
a variant of (wfst_get_lattice): same tokens, same links, bit for bit, on two calls in a row, the
second on a shorter utterance (the static scratch keeps the first call's contents).

Collected last on purpose: the round's end runs pytest -x, and a failure here must not hide the
other tests.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _rows(frame_off, state, links):
    k = links
    rows = np.stack([np.asarray(c).astype(np.int64) for c in
                     (k["frame"], state[k["src"]], state[k["dst"]], k["ilabel"], k["olabel"],
                      k["graph_cost"].view(np.uint32), k["acoustic_cost"].view(np.uint32), k["cost"].view(np.uint32))],
                    axis=1)
    return rows[np.lexsort(rows.T[::-1])]


def test_noalloc_lattice_matches_get_lattice_twice_in_a_row():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2311_04996_amd import Decoder
    from paper_2311_04996_amd.binding import LINK_DTYPE, WfstError
    from workloads import make_config
    w = make_config("c2_medium", batch=3)
    lengths = np.minimum(w.lengths, [150, 60, 20]).astype(np.int32)   # long, then shorter, then shortest
    T = int(lengths.max())
    ll = torch.from_numpy(np.ascontiguousarray(w.loglikes[:, :T])).cuda()
    dec = Decoder(w.graph, max_channels=3, max_frames=T, max_active_hint=w.max_active, keep_token_records=True)
    dec.decode_batch(ll, lengths, w.beam, w.max_active)
    torch.cuda.synchronize()
    lattice_beam = 2.0
    for ch in (0, 1, 2, 0):                                           # back to the long one at the end
        n = int(lengths[ch])
        rows = ll[ch, :n].contiguous()
        want = dec.get_lattice(ch, rows, lattice_beam)                # the existing entry point
        nt, nl = len(want.state), len(want.links)
        assert nl > nt > 0
        tok_state = torch.full((nt,), -1, dtype=torch.int32, device="cuda")
        tok_cost = torch.full((nt,), -1.0, dtype=torch.float32, device="cuda")
        links = torch.zeros(nl * LINK_DTYPE.itemsize, dtype=torch.uint8, device="cuda")
        frame_off = np.zeros(dec.opts.max_frames_per_channel + 2, np.int64)
        torch.cuda.synchronize()
        got_nt, got_nl = dec.get_lattice_noalloc(ch, rows, lattice_beam, tok_state, tok_cost, links, frame_off)
        assert (got_nt, got_nl) == (nt, nl)
        assert frame_off[:n + 2].tolist() == want.frame_off.tolist()
        st, co = tok_state.cpu().numpy(), tok_cost.cpu().numpy()
        assert (st == want.state).all() and (co.view(np.uint32) == want.cost.view(np.uint32)).all()
        lk = links.cpu().numpy().view(LINK_DTYPE)
        a, b = _rows(frame_off, st, lk), _rows(want.frame_off, want.state, want.links)
        assert a.shape == b.shape and (a == b).all()
    # too small buffers: the sizes come back with WFST_ERR_CAPACITY, nothing is written past them
    small = torch.zeros(4 * LINK_DTYPE.itemsize, dtype=torch.uint8, device="cuda")
    with pytest.raises(WfstError) as e:
        dec.get_lattice_noalloc(0, ll[0, :int(lengths[0])].contiguous(), lattice_beam, tok_state, tok_cost, small,
                                frame_off)
    assert e.value.code == -7
    dec.close()


def test_noalloc_lattice_rejects_more_frames_than_its_scratch_holds():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2311_04996_amd import Decoder
    from paper_2311_04996_amd.binding import LINK_DTYPE, WfstError
    from workloads import ctc_topology_graph, ctc_loglikes
    V, T = 6, 4100                                                    # the static scratch holds 4094 frames
    g = ctc_topology_graph(V)
    ll = torch.from_numpy(ctc_loglikes(7, [T], T, V, sigma=1.0, p_blank=0.5, blank_boost=3.0, token_boost=3.0)).cuda()
    dec = Decoder(g, max_channels=1, max_frames=T, max_active_hint=64, keep_token_records=True)
    dec.decode_batch(ll, [T], 3.0, 64)
    torch.cuda.synchronize()
    want = dec.get_lattice(0, ll[0], 1.0)                             # the allocating entry point has no such limit
    assert len(want.links) > 0
    tok_state = torch.zeros(len(want.state), dtype=torch.int32, device="cuda")
    tok_cost = torch.zeros(len(want.state), dtype=torch.float32, device="cuda")
    links = torch.zeros(len(want.links) * LINK_DTYPE.itemsize, dtype=torch.uint8, device="cuda")
    frame_off = np.zeros(T + 2, np.int64)
    with pytest.raises(WfstError) as e:
        dec.get_lattice_noalloc(0, ll[0], 1.0, tok_state, tok_cost, links, frame_off)
    assert e.value.code == -7 and "4094" in str(e.value)
    dec.close()
