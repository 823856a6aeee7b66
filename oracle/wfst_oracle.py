"""ctypes loader for the C oracle in wfst_oracle.c (test infrastructure only)."""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_LIB = os.path.join(_HERE, "liboracle.so")
_SRC = os.path.join(_HERE, "wfst_oracle.c")


def build_oracle(force: bool = False) -> str:
    """Compile the oracle with strict fp32 semantics (no contraction, no fast-math)."""
    if force or not os.path.exists(ORACLE_LIB) or os.path.getmtime(ORACLE_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math",
                               "-fPIC", "-shared", "-o", ORACLE_LIB, _SRC, "-lm"])
    return ORACLE_LIB


class _Graph(C.Structure):
    _fields_ = [("num_states", C.c_int32), ("start_state", C.c_int32), ("num_classes", C.c_int32),
                ("num_arcs", C.c_int64), ("row_offsets", C.c_void_p), ("next_state", C.c_void_p),
                ("ilabel", C.c_void_p), ("olabel", C.c_void_p), ("weight", C.c_void_p),
                ("final_cost", C.c_void_p)]


class _Opts(C.Structure):
    _fields_ = [("beam", C.c_float), ("max_active", C.c_int32), ("max_words", C.c_int32),
                ("finalize", C.c_int32), ("worklist_order", C.c_int32), ("order_seed", C.c_uint64),
                ("boost_n", C.c_int32), ("boost_ids", C.c_void_p), ("boost_scores", C.c_void_p),
                ("cost_offset", C.c_int32),
                ("bfst_states", C.c_int32), ("bfst_arcs", C.c_int32), ("bfst_from", C.c_void_p),
                ("bfst_label", C.c_void_p), ("bfst_to", C.c_void_p), ("bfst_score", C.c_void_p)]


class _Result(C.Structure):
    _fields_ = [("nwords", C.c_int32), ("cost", C.c_float), ("flags", C.c_int32),
                ("path_len", C.c_int32), ("counters", C.c_int64 * 8)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        build_oracle()
        _lib = C.CDLL(ORACLE_LIB)
        _lib.oracle_prepare.restype = C.c_void_p
        _lib.oracle_prepare.argtypes = [C.POINTER(_Graph)]
        _lib.oracle_free.argtypes = [C.c_void_p]
        _lib.oracle_num_emitting.restype = C.c_int64
        _lib.oracle_num_emitting.argtypes = [C.c_void_p]
        _lib.oracle_num_epsilon.restype = C.c_int64
        _lib.oracle_num_epsilon.argtypes = [C.c_void_p]
        _lib.oracle_arc_original_index.restype = C.c_int64
        _lib.oracle_arc_original_index.argtypes = [C.c_void_p, C.c_int64]
        _lib.oracle_cutoff.restype = C.c_int32
        _lib.oracle_cutoff.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_int32,
                                       C.POINTER(C.c_float), C.POINTER(C.c_int32), C.c_void_p]
        _lib.oracle_keep.restype = C.c_int32
        _lib.oracle_keep.argtypes = [C.c_float, C.c_float, C.c_float, C.c_int32]
        _lib.oracle_eps_closure.restype = C.c_int32
        _lib.oracle_eps_closure.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                            C.c_float, C.c_float, C.c_int32, C.c_int32,
                                            C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_int32]
        _lib.oracle_decode.restype = C.c_int32
        _lib.oracle_decode.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                       C.POINTER(_Opts), C.c_void_p, C.POINTER(_Result),
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        _lib.oracle_lattice_links.restype = C.c_int64
        _lib.oracle_lattice_links.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                              C.POINTER(_Opts), C.c_float, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p]
    return _lib


def oracle_cutoff(costs, beam: float, max_active: int):
    """(best, k_keep, n_in_beam, hist[256]) of a set of recombined token costs."""
    lib = _load()
    c = np.ascontiguousarray(costs, dtype=np.float32)
    best, kk = C.c_float(), C.c_int32()
    hist = np.zeros(256, dtype=np.int32)
    n_in = lib.oracle_cutoff(c.ctypes.data, len(c), beam, max_active, C.byref(best),
                             C.byref(kk), hist.ctypes.data)
    return best.value, kk.value, n_in, hist


def oracle_keep(c: float, best: float, beam: float, k_keep: int) -> bool:
    return bool(_load().oracle_keep(c, best, beam, k_keep))


@dataclass
class OracleResult:
    words: np.ndarray
    cost: float
    flags: int
    counters: np.ndarray
    path_arcs: np.ndarray | None = None          # global arc ids, in path order
    digest_count: np.ndarray | None = None       # [len+1]
    digest_sum: np.ndarray | None = None         # [len+1] uint64
    frames: list | None = field(default=None)    # per closed set: (states, costs)
    frames_b: list | None = field(default=None)  # per closed set: the tokens' boosting-acceptor states
    frame_best: np.ndarray | None = None         # [len+1] offsets the sets were rebased by (cost offsets)

    @property
    def reached_final(self) -> bool:
        return bool(self.flags & 1)

    @property
    def truncated(self) -> bool:
        return bool(self.flags & 2)

    @property
    def dead(self) -> bool:
        return bool(self.flags & 4)


@dataclass
class OracleLattice:
    """Token sets A_0..A_T (set_off, states, costs) and the links between them.  A link's src /
    dst are positions inside their sets: the source of an emitting link (arc < num_emitting)
    lies in A_{frame-1}, of an epsilon link in A_frame."""
    result: OracleResult
    set_off: np.ndarray
    states: np.ndarray
    costs: np.ndarray
    frame: np.ndarray
    src: np.ndarray
    dst: np.ndarray
    arc: np.ndarray
    cost: np.ndarray
    num_emitting: int

    def src_global(self) -> np.ndarray:
        """Index of every link's source token in the concatenated token arrays."""
        emit = self.arc < self.num_emitting
        return self.set_off[self.frame - emit.astype(np.int32)] + self.src

    def dst_global(self) -> np.ndarray:
        return self.set_off[self.frame] + self.dst


class Oracle:
    """Prepared graph + decode calls.  `graph` is a workloads.Graph (or any object with the
    same array attributes); the arrays are only read."""

    def __init__(self, graph):
        lib = _load()
        self._keep = [np.ascontiguousarray(graph.row_offsets, dtype=np.int64),
                      np.ascontiguousarray(graph.next_state, dtype=np.int32),
                      np.ascontiguousarray(graph.ilabel, dtype=np.int32),
                      np.ascontiguousarray(graph.olabel, dtype=np.int32),
                      np.ascontiguousarray(graph.weight, dtype=np.float32),
                      None if graph.final_cost is None else
                      np.ascontiguousarray(graph.final_cost, dtype=np.float32)]
        g = _Graph(graph.num_states, graph.start_state, graph.num_classes,
                   int(self._keep[0][-1]), *[None if a is None else a.ctypes.data for a in self._keep])
        self.V = graph.num_classes
        self._p = lib.oracle_prepare(C.byref(g))
        if not self._p:
            raise ValueError("oracle_prepare rejected the graph")
        self.num_emitting = lib.oracle_num_emitting(self._p)
        self.num_epsilon = lib.oracle_num_epsilon(self._p)

    def __del__(self):
        if getattr(self, "_p", None) and _lib is not None:
            _lib.oracle_free(self._p)
            self._p = None

    def original_arc(self, gid: int) -> int:
        return int(_load().oracle_arc_original_index(self._p, int(gid)))

    def decode(self, loglikes, length=None, beam=17.0, max_active=10000, max_words=1024,
               finalize=True, worklist_order=0, order_seed=0, want_path=False,
               want_digests=False, want_frames=False, frames_cap=None, boost=None,
               cost_offset=False, boost_fst=None) -> OracleResult:
        """boost: optional (word_ids, scores) table of the utterance (Section "Word boosting").
        boost_fst: optional boosting acceptor with several states (reading R12 in the C source), an
        object with num_states and arrays arc_from, arc_label, arc_to, arc_score.
        cost_offset: rebase the token costs after every prune step (reading R11 in the C source)."""
        lib = _load()
        ll = np.asarray(loglikes, dtype=np.float32)
        assert ll.ndim == 2 and ll.shape[1] == self.V and ll.strides[1] == 4
        n = ll.shape[0] if length is None else int(length)
        assert n <= ll.shape[0]
        if boost is not None:
            b_ids = np.ascontiguousarray(boost[0], dtype=np.int32)
            b_sc = np.ascontiguousarray(boost[1], dtype=np.float32)
            assert b_ids.shape == b_sc.shape
            o = _Opts(beam, max_active, max_words, int(bool(finalize)), worklist_order, order_seed,
                      len(b_ids), b_ids.ctypes.data, b_sc.ctypes.data, int(bool(cost_offset)))
        else:
            o = _Opts(beam, max_active, max_words, int(bool(finalize)), worklist_order, order_seed, 0, None, None,
                      int(bool(cost_offset)))
        if boost_fst is not None:
            assert boost is None
            f_from = np.ascontiguousarray(boost_fst.arc_from, dtype=np.int32)
            f_lab = np.ascontiguousarray(boost_fst.arc_label, dtype=np.int32)
            f_to = np.ascontiguousarray(boost_fst.arc_to, dtype=np.int32)
            f_sc = np.ascontiguousarray(boost_fst.arc_score, dtype=np.float32)
            assert f_from.shape == f_lab.shape == f_to.shape == f_sc.shape
            o.bfst_states, o.bfst_arcs = int(boost_fst.num_states), len(f_from)
            o.bfst_from, o.bfst_label = f_from.ctypes.data, f_lab.ctypes.data
            o.bfst_to, o.bfst_score = f_to.ctypes.data, f_sc.ctypes.data
        res = _Result()
        words = np.zeros(max(1, max_words), dtype=np.int32)
        dc = np.zeros(n + 1, dtype=np.int32) if want_digests else None
        ds = np.zeros(n + 1, dtype=np.uint64) if want_digests else None
        pcap = 8 * (n + 8) + 64
        path = np.zeros(pcap, dtype=np.int32) if want_path else None
        if want_frames:
            cap = frames_cap or (n + 1) * max(4096, 4 * min(max_active, 1 << 20))
            doff = np.zeros(n + 2, dtype=np.int64)
            dst = np.zeros(cap, dtype=np.int32)
            dco = np.zeros(cap, dtype=np.float32)
            dbs = np.zeros(cap, dtype=np.int32)
        else:
            cap, doff, dst, dco, dbs = 0, None, None, None, None
        ptr = lambda a: None if a is None else a.ctypes.data
        fbest = np.zeros(n + 1, dtype=np.float32) if want_frames else None
        rc = lib.oracle_decode(self._p, ll.ctypes.data, ll.strides[0] // 4, n, C.byref(o),
                               words.ctypes.data, C.byref(res), ptr(dc), ptr(ds), ptr(path), pcap,
                               ptr(doff), ptr(dst), ptr(dco), cap, ptr(fbest), ptr(dbs))
        if rc != 0:
            raise RuntimeError(f"oracle_decode failed: {rc}")
        frames = frames_b = None
        if want_frames:
            frames = [(dst[doff[t]:doff[t + 1]].copy(), dco[doff[t]:doff[t + 1]].copy())
                      for t in range(n + 1)]
            frames_b = [dbs[doff[t]:doff[t + 1]].copy() for t in range(n + 1)]
        return OracleResult(words[:res.nwords].copy(), float(res.cost), int(res.flags),
                            np.array(list(res.counters), dtype=np.int64),
                            None if path is None else path[:res.path_len].copy(), dc, ds, frames, frames_b, fbest)

    def lattice(self, loglikes, length=None, beam=17.0, max_active=10000, lattice_beam=np.inf,
                boost=None, cost_offset=False) -> "OracleLattice":
        """Decode, then list the lattice links between the stored token sets (reading R10 in
        the C source): every arc between two stored tokens whose cost through the arc is within
        `lattice_beam` of the destination token's cost."""
        lib = _load()
        ll = np.asarray(loglikes, dtype=np.float32)
        n = ll.shape[0] if length is None else int(length)
        cap = (n + 1) * max(4096, 4 * min(max_active, 1 << 20))
        while True:                                   # the closure can grow a set well past max_active
            try:
                res = self.decode(ll, n, beam, max_active, want_frames=True, want_path=True, boost=boost,
                                  frames_cap=cap, cost_offset=cost_offset)
                break
            except RuntimeError as e:
                if "-2" not in str(e) or cap > (1 << 31):
                    raise
                cap *= 4
        off = np.zeros(n + 2, np.int64)
        off[1:] = np.cumsum([len(s) for s, _ in res.frames])
        st = np.ascontiguousarray(np.concatenate([s for s, _ in res.frames]), dtype=np.int32)
        co = np.ascontiguousarray(np.concatenate([c for _, c in res.frames]), dtype=np.float32)
        if boost is not None:
            b_ids = np.ascontiguousarray(boost[0], dtype=np.int32)
            b_sc = np.ascontiguousarray(boost[1], dtype=np.float32)
            o = _Opts(beam, max_active, 0, 1, 0, 0, len(b_ids), b_ids.ctypes.data, b_sc.ctypes.data, int(cost_offset))
        else:
            o = _Opts(beam, max_active, 0, 1, 0, 0, 0, None, None, int(cost_offset))
        fb = np.ascontiguousarray(res.frame_best, dtype=np.float32) if cost_offset else None
        args = (self._p, ll.ctypes.data, ll.strides[0] // 4, n, C.byref(o), float(lattice_beam),
                off.ctypes.data, st.ctypes.data, co.ctypes.data, None if fb is None else fb.ctypes.data)
        m = lib.oracle_lattice_links(*args, 0, None, None, None, None, None)
        if m < 0:
            raise RuntimeError("oracle_lattice_links rejected its arguments")
        fr, src, dst, arc = (np.zeros(m, np.int32) for _ in range(4))
        cost = np.zeros(m, np.float32)
        m2 = lib.oracle_lattice_links(*args, m, fr.ctypes.data, src.ctypes.data, dst.ctypes.data,
                                      arc.ctypes.data, cost.ctypes.data)
        assert m2 == m
        return OracleLattice(res, off, st, co, fr, src, dst, arc, cost, self.num_emitting)

    def eps_closure(self, states, costs, best, beam, k_keep=256, order=0, seed=0):
        lib = _load()
        st = np.ascontiguousarray(states, dtype=np.int32)
        co = np.ascontiguousarray(costs, dtype=np.float32)
        cap = max(1024, 64 * len(st) + 65536)
        os_, oc = np.zeros(cap, np.int32), np.zeros(cap, np.float32)
        op, oa = np.zeros(cap, np.int32), np.zeros(cap, np.int32)
        n = lib.oracle_eps_closure(self._p, st.ctypes.data, co.ctypes.data, len(st), best, beam,
                                   k_keep, order, seed, os_.ctypes.data, oc.ctypes.data,
                                   op.ctypes.data, oa.ctypes.data, cap)
        if n < 0:
            raise RuntimeError("closure output overflow")
        return os_[:n].copy(), oc[:n].copy(), op[:n].copy(), oa[:n].copy()
