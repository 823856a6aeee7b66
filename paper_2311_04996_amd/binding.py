"""Thin ctypes binding over libwfstdec.so (include/wfst_decoder.h).

Argument marshalling only: every step of decoding runs in the HIP kernels.  PyTorch supplies
device memory and streams.  There is no CPU fallback: if the library is missing or cannot
be loaded, importing this module's entry points raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from .build import LIB_PATH

WFST_OK = 0
ERRORS = {-1: "INVALID_ARG", -2: "BAD_GRAPH", -3: "OOM", -4: "LATTICE_OVERFLOW",
          -5: "BAD_CHANNEL", -6: "HIP", -7: "CAPACITY"}
FLAG_REACHED_FINAL, FLAG_TRUNCATED, FLAG_DEAD, FLAG_LATTICE_OVERFLOW, FLAG_CAPACITY = 1, 2, 4, 8, 16
LOGLIKE_DTYPES = {"float32": 0, "float16": 1, "bfloat16": 2}

EXPORTS = ["wfst_decoder_create", "wfst_decoder_destroy", "wfst_decode_batch", "wfst_decode_batch_boosted",
           "wfst_decode_batch_boost_fst", "wfst_decode_batch_slot", "wfst_slot_kernel_ms", "wfst_init_channel", "wfst_init_channel_boost_fst", "wfst_init_channels", "wfst_init_channels_boost_fst",
           "wfst_advance_chunk", "wfst_advance_chunk_partial", "wfst_get_partial", "wfst_get_partial_batch", "wfst_get_lattice",
           "wfst_get_lattice_noalloc", "wfst_get_lattice_batch",
           "wfst_debug_frame_digests",
           "wfst_debug_get_tokens", "wfst_debug_get_token_pairs", "wfst_get_counters", "wfst_debug_phase_ticks", "wfst_debug_set_phase_timing", "wfst_set_launch_workgroups", "wfst_device_bytes",
           "wfst_last_kernel_ms", "wfst_last_error"]


class WfstError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"{ERRORS.get(code, code)}: {msg}")
        self.code = code


class wfst_graph_csr(C.Structure):
    _fields_ = [("num_states", C.c_int32), ("start_state", C.c_int32), ("num_classes", C.c_int32),
                ("num_arcs", C.c_int64), ("row_offsets", C.c_void_p), ("next_state", C.c_void_p),
                ("ilabel", C.c_void_p), ("olabel", C.c_void_p), ("weight", C.c_void_p),
                ("final_cost", C.c_void_p)]


class wfst_boost_table(C.Structure):
    _fields_ = [("n", C.c_int32), ("word_ids", C.c_void_p), ("scores", C.c_void_p)]


def _boost_struct(boost):
    """(word_ids, scores) -> (wfst_boost_table, arrays to keep alive)."""
    ids = np.ascontiguousarray(boost[0], dtype=np.int32)
    sc = np.ascontiguousarray(boost[1], dtype=np.float32)
    assert ids.shape == sc.shape and ids.ndim == 1
    return wfst_boost_table(len(ids), ids.ctypes.data, sc.ctypes.data), (ids, sc)


class wfst_boost_fst(C.Structure):
    _fields_ = [("n_states", C.c_int32), ("n_arcs", C.c_int32), ("arc_from", C.c_void_p),
                ("arc_label", C.c_void_p), ("arc_to", C.c_void_p), ("arc_score", C.c_void_p)]


def _fst_struct(fst):
    """Object with num_states, arc_from, arc_label, arc_to, arc_score -> (wfst_boost_fst, arrays to keep alive)."""
    a = (np.ascontiguousarray(fst.arc_from, dtype=np.int32), np.ascontiguousarray(fst.arc_label, dtype=np.int32),
         np.ascontiguousarray(fst.arc_to, dtype=np.int32), np.ascontiguousarray(fst.arc_score, dtype=np.float32))
    assert a[0].shape == a[1].shape == a[2].shape == a[3].shape and a[0].ndim == 1
    return wfst_boost_fst(int(fst.num_states), len(a[0]), *[x.ctypes.data for x in a]), a


class wfst_opts(C.Structure):
    _fields_ = [("max_channels", C.c_int32), ("max_frames_per_channel", C.c_int32),
                ("max_words", C.c_int32), ("lattice_bytes_per_channel", C.c_int64),
                ("outputs_on_host", C.c_int32), ("max_active_hint", C.c_int32),
                ("candidate_capacity", C.c_int32), ("record_digests", C.c_int32),
                ("loglike_dtype", C.c_int32), ("keep_token_records", C.c_int32), ("cost_offset", C.c_int32),
                ("batch_slots", C.c_int32), ("recycle_lattice", C.c_int32), ("lattice_by_length", C.c_int32),
                ("narrow_arcs", C.c_int32), ("selection_sample", C.c_int32)]


class wfst_lattice_link(C.Structure):
    _fields_ = [("src", C.c_int32), ("dst", C.c_int32), ("ilabel", C.c_int32), ("olabel", C.c_int32),
                ("graph_cost", C.c_float), ("acoustic_cost", C.c_float), ("cost", C.c_float),
                ("frame", C.c_int32)]


LINK_DTYPE = np.dtype([("src", np.int32), ("dst", np.int32), ("ilabel", np.int32), ("olabel", np.int32),
                       ("graph_cost", np.float32), ("acoustic_cost", np.float32), ("cost", np.float32),
                       ("frame", np.int32)])


_lib = None


def load_library():
    """Loads the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2311_04996_amd.build` "
                           "(or __graft_entry__.build()) first; there is no CPU fallback")
    # PyTorch ships its own HIP runtime; import it first so that this library binds to the
    # same libamdhip64 instance (two runtimes in one process do not share the device).
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    p, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    lib.wfst_decoder_create.argtypes = [C.POINTER(wfst_graph_csr), C.POINTER(wfst_opts), C.POINTER(p)]
    lib.wfst_decoder_destroy.argtypes = [p]
    lib.wfst_decode_batch.argtypes = [p, p, p, i32, i32, i32, f32, i32, p, p, p, p, p]
    lib.wfst_decode_batch_boosted.argtypes = [p, p, p, i32, i32, i32, f32, i32, p, p, p, p, p, p]
    lib.wfst_init_channel.argtypes = [p, i32, f32, i32, p, p]
    lib.wfst_init_channel_boost_fst.argtypes = [p, i32, f32, i32, p, p]
    lib.wfst_decode_batch_boost_fst.argtypes = [p, p, p, i32, i32, i32, f32, i32, p, p, p, p, p, p]
    lib.wfst_debug_get_token_pairs.argtypes = [p, i32, p, p, p, i32, p]
    lib.wfst_init_channels.argtypes = [p, p, i32, f32, i32, p, p]
    lib.wfst_init_channels_boost_fst.argtypes = [p, p, i32, f32, i32, p, p]
    lib.wfst_advance_chunk.argtypes = [p, p, i32, p, p, i32, i32, p]
    lib.wfst_advance_chunk_partial.argtypes = [p, p, i32, p, p, i32, i32, i32, p, p, p, p, p]
    lib.wfst_get_partial.argtypes = [p, i32, i32, p, i32, p, p, p, p]
    lib.wfst_get_partial_batch.argtypes = [p, p, i32, i32, p, p, p, p, p]
    lib.wfst_debug_frame_digests.argtypes = [p, i32, p, p, i32, p]
    lib.wfst_debug_get_tokens.argtypes = [p, i32, p, p, i32, p]
    lib.wfst_get_counters.argtypes = [p, p, i32]
    lib.wfst_debug_phase_ticks.argtypes = [p, p, i32]
    lib.wfst_debug_set_phase_timing.argtypes = [p, i32]
    lib.wfst_set_launch_workgroups.argtypes = [p, i32]
    lib.wfst_device_bytes.argtypes = [p]
    lib.wfst_device_bytes.restype = i64
    lib.wfst_last_kernel_ms.argtypes = [p]
    lib.wfst_last_kernel_ms.restype = f32
    lib.wfst_slot_kernel_ms.argtypes = [p, i32]
    lib.wfst_slot_kernel_ms.restype = f32
    lib.wfst_decode_batch_slot.argtypes = [p, i32, p, p, i32, i32, i32, f32, i32, p, p, p, p, p, p, p]
    lib.wfst_last_error.argtypes = [p]
    lib.wfst_last_error.restype = C.c_char_p
    lib.wfst_get_lattice.argtypes = [p, i32, p, f32, p, p, i64, p, p, i64, p, p, p]
    lib.wfst_get_lattice_noalloc.argtypes = lib.wfst_get_lattice.argtypes
    lib.wfst_get_lattice_batch.argtypes = [p, p, i32, p, i32, f32, p, p, i64, p, p, i64, p, p, p]
    for name in EXPORTS:
        if name not in ("wfst_device_bytes", "wfst_last_kernel_ms", "wfst_slot_kernel_ms", "wfst_last_error"):
            getattr(lib, name).restype = i32
    _lib = lib
    return lib


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _on(stream):
    """Context in which torch allocates (and zero-fills) on the stream the kernel will run on: a
    fill queued on another stream could land after the kernel has written its outputs."""
    import contextlib
    import torch
    return contextlib.nullcontext() if stream is None else torch.cuda.stream(stream)


class Decoder:
    """Owns one wfst_decoder handle.  Method names mirror the C entry points."""

    def __init__(self, graph, max_channels, max_frames, max_words=256, max_active_hint=10000,
                 lattice_bytes_per_channel=0, outputs_on_host=False, candidate_capacity=0,
                 record_digests=False, loglike_dtype="float32", keep_token_records=False, cost_offset=False,
                 batch_slots=0, recycle_lattice=False, lattice_by_length=False, narrow_arcs=False, selection_sample=0):
        self.lib = load_library()
        arrs = [np.ascontiguousarray(graph.row_offsets, dtype=np.int64),
                np.ascontiguousarray(graph.next_state, dtype=np.int32),
                np.ascontiguousarray(graph.ilabel, dtype=np.int32),
                np.ascontiguousarray(graph.olabel, dtype=np.int32),
                np.ascontiguousarray(graph.weight, dtype=np.float32),
                None if graph.final_cost is None else np.ascontiguousarray(graph.final_cost, dtype=np.float32)]
        g = wfst_graph_csr(graph.num_states, graph.start_state, graph.num_classes, int(arrs[0][-1]),
                           *[None if a is None else a.ctypes.data for a in arrs])
        self.opts = wfst_opts(max_channels, max_frames, max_words, lattice_bytes_per_channel,
                              int(outputs_on_host), max_active_hint, candidate_capacity,
                              int(record_digests), LOGLIKE_DTYPES[loglike_dtype], int(keep_token_records),
                              int(cost_offset), int(batch_slots), int(recycle_lattice), int(lattice_by_length),
                              int(narrow_arcs), int(selection_sample))
        self.loglike_dtype = loglike_dtype
        self.V = graph.num_classes
        self.max_words = max_words
        self.outputs_on_host = bool(outputs_on_host)
        h = C.c_void_p()
        rc = self.lib.wfst_decoder_create(C.byref(g), C.byref(self.opts), C.byref(h))
        if rc != WFST_OK:
            raise WfstError(rc, self.lib.wfst_last_error(None).decode())
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.wfst_decoder_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != WFST_OK:
            raise WfstError(rc, self.lib.wfst_last_error(self.h).decode())

    # ---- offline
    def decode_batch(self, loglikes, lengths, beam, max_active, stream=None, out=None, boosts=None, boost_fsts=None,
                     slot=None):
        """loglikes: CUDA float32 tensor [B, T, V]; lengths: int32 host array [B].
        boosts: optional list of B entries, each None or a (word_ids, scores) table.
        boost_fsts: optional list of B entries, each None or a boosting acceptor (an object with
        num_states, arc_from, arc_label, arc_to, arc_score).
        Returns (words [B, max_words], nwords [B], cost [B], flags [B]); torch CUDA tensors, or
        numpy arrays when the decoder was created with outputs_on_host."""
        import torch
        assert loglikes.is_cuda and loglikes.dtype == getattr(torch, self.loglike_dtype) and loglikes.is_contiguous()
        B, T, V = loglikes.shape
        lengths = np.ascontiguousarray(lengths, dtype=np.int32)
        assert lengths.shape == (B,)
        if out is None:
            if self.outputs_on_host:
                out = (np.zeros((B, self.max_words), np.int32), np.zeros(B, np.int32),
                       np.zeros(B, np.float32), np.zeros(B, np.int32))
            else:
                dev = loglikes.device
                with _on(stream):
                    out = (torch.zeros((B, self.max_words), dtype=torch.int32, device=dev),
                           torch.zeros(B, dtype=torch.int32, device=dev),
                           torch.zeros(B, dtype=torch.float32, device=dev),
                           torch.zeros(B, dtype=torch.int32, device=dev))
        ptr = (lambda a: a.ctypes.data) if self.outputs_on_host else (lambda t: t.data_ptr())
        if slot is not None:                       # wfst_decode_batch_slot: several batches in flight on one decoder
            keep = arr_t = arr_f = None
            if boosts is not None:
                keep = [None if t is None else _boost_struct(t) for t in boosts]
                arr_t = (C.c_void_p * B)(*[None if k is None else C.addressof(k[0]) for k in keep])
            if boost_fsts is not None:
                keep = [None if f is None else _fst_struct(f) for f in boost_fsts]
                arr_f = (C.c_void_p * B)(*[None if k is None else C.addressof(k[0]) for k in keep])
            self._check(self.lib.wfst_decode_batch_slot(self.h, int(slot), loglikes.data_ptr(), lengths.ctypes.data, B, T, V,
                                                        beam, max_active, arr_t, arr_f, _stream_ptr(stream),
                                                        ptr(out[0]), ptr(out[1]), ptr(out[2]), ptr(out[3])))
            return out
        if boost_fsts is not None:
            assert boosts is None and len(boost_fsts) == B
            keep = [None if f is None else _fst_struct(f) for f in boost_fsts]
            arr = (C.c_void_p * B)(*[None if k is None else C.addressof(k[0]) for k in keep])
            self._check(self.lib.wfst_decode_batch_boost_fst(self.h, loglikes.data_ptr(), lengths.ctypes.data, B, T, V,
                                                             beam, max_active, arr, _stream_ptr(stream),
                                                             ptr(out[0]), ptr(out[1]), ptr(out[2]), ptr(out[3])))
            return out
        if boosts is None:
            self._check(self.lib.wfst_decode_batch(self.h, loglikes.data_ptr(), lengths.ctypes.data, B, T, V,
                                                   beam, max_active, _stream_ptr(stream),
                                                   ptr(out[0]), ptr(out[1]), ptr(out[2]), ptr(out[3])))
            return out
        assert len(boosts) == B
        keep = [None if t is None else _boost_struct(t) for t in boosts]
        arr = (C.c_void_p * B)(*[None if k is None else C.addressof(k[0]) for k in keep])
        self._check(self.lib.wfst_decode_batch_boosted(self.h, loglikes.data_ptr(), lengths.ctypes.data, B, T, V,
                                                       beam, max_active, arr, _stream_ptr(stream),
                                                       ptr(out[0]), ptr(out[1]), ptr(out[2]), ptr(out[3])))
        return out

    # ---- streaming
    def init_channel(self, ch, beam, max_active, stream=None, boost=None, boost_fst=None):
        """boost: None or a (word_ids, scores) table for this stream; boost_fst: None or a boosting
        acceptor with several states."""
        if boost_fst is not None:
            assert boost is None
            t, keep = _fst_struct(boost_fst)
            self._check(self.lib.wfst_init_channel_boost_fst(self.h, ch, beam, max_active, C.byref(t), _stream_ptr(stream)))
        elif boost is None:
            self._check(self.lib.wfst_init_channel(self.h, ch, beam, max_active, None, _stream_ptr(stream)))
        else:
            t, keep = _boost_struct(boost)
            self._check(self.lib.wfst_init_channel(self.h, ch, beam, max_active, C.byref(t), _stream_ptr(stream)))

    def init_channels(self, channels, beam, max_active, stream=None, boosts=None, boost_fsts=None):
        """wfst_init_channels: reset several channels in one launch; boosts: None or one entry
        per channel, each None or a (word_ids, scores) table; boost_fsts (instead): None or one
        entry per channel, each None or a boosting acceptor (wfst_init_channels_boost_fst)."""
        channels = np.ascontiguousarray(channels, dtype=np.int32)
        n = len(channels)
        arr = None
        if boost_fsts is not None:
            assert boosts is None and len(boost_fsts) == n
            keep = [None if f is None else _fst_struct(f) for f in boost_fsts]
            arr = (C.c_void_p * n)(*[None if k is None else C.addressof(k[0]) for k in keep])
            self._check(self.lib.wfst_init_channels_boost_fst(self.h, channels.ctypes.data, n, beam, max_active, arr,
                                                              _stream_ptr(stream)))
            return
        if boosts is not None:
            assert len(boosts) == n
            keep = [None if t is None else _boost_struct(t) for t in boosts]
            arr = (C.c_void_p * n)(*[None if k is None else C.addressof(k[0]) for k in keep])
        self._check(self.lib.wfst_init_channels(self.h, channels.ctypes.data, n, beam, max_active, arr,
                                                _stream_ptr(stream)))

    def advance_chunk(self, channels, loglikes, nframes, stream=None):
        """loglikes: CUDA float32 [n, C, V]; channels, nframes: host int32 [n]."""
        import torch
        assert loglikes.is_cuda and loglikes.dtype == getattr(torch, self.loglike_dtype) and loglikes.is_contiguous()
        n, Cn, V = loglikes.shape
        channels = np.ascontiguousarray(channels, dtype=np.int32)
        nframes = np.ascontiguousarray(nframes, dtype=np.int32)
        assert channels.shape == (n,) and nframes.shape == (n,)
        self._check(self.lib.wfst_advance_chunk(self.h, channels.ctypes.data, n, loglikes.data_ptr(),
                                                nframes.ctypes.data, Cn, V, _stream_ptr(stream)))

    def _partial_outputs(self, n, stream):
        import torch
        if self.outputs_on_host:
            return (np.zeros((n, self.max_words), np.int32), np.zeros(n, np.int32),
                    np.zeros(n, np.float32), np.zeros(n, np.int32))
        with _on(stream):
            return (torch.zeros((n, self.max_words), dtype=torch.int32, device="cuda"),
                    torch.zeros(n, dtype=torch.int32, device="cuda"),
                    torch.zeros(n, dtype=torch.float32, device="cuda"),
                    torch.zeros(n, dtype=torch.int32, device="cuda"))

    def advance_chunk_partial(self, channels, loglikes, nframes, finalize=False, stream=None, out=None):
        """wfst_advance_chunk_partial: advance_chunk and get_partial_batch in one launch.  Returns
        (words [n, max_words], nwords [n], cost [n], flags [n]) like get_partial_batch."""
        import torch
        assert loglikes.is_cuda and loglikes.dtype == getattr(torch, self.loglike_dtype) and loglikes.is_contiguous()
        n, Cn, V = loglikes.shape
        channels = np.ascontiguousarray(channels, dtype=np.int32)
        nframes = np.ascontiguousarray(nframes, dtype=np.int32)
        assert channels.shape == (n,) and nframes.shape == (n,)
        if out is None:
            out = self._partial_outputs(n, stream)
        ptr = (lambda a: a.ctypes.data) if self.outputs_on_host else (lambda t: t.data_ptr())
        self._check(self.lib.wfst_advance_chunk_partial(self.h, channels.ctypes.data, n, loglikes.data_ptr(),
                                                        nframes.ctypes.data, Cn, V, int(finalize),
                                                        ptr(out[0]), ptr(out[1]), ptr(out[2]), ptr(out[3]),
                                                        _stream_ptr(stream)))
        return out

    def get_partial(self, ch, finalize=False, stream=None, cap=None):
        """Returns (words ndarray, cost, flags) of the channel's best hypothesis so far (at most
        `cap` words, default the decoder's max_words)."""
        import torch
        cap = self.max_words if cap is None else int(cap)
        if self.outputs_on_host:
            w, n = np.zeros(cap, np.int32), np.zeros(1, np.int32)
            c, f = np.zeros(1, np.float32), np.zeros(1, np.int32)
            self._check(self.lib.wfst_get_partial(self.h, ch, int(finalize), w.ctypes.data, cap, n.ctypes.data,
                                                  c.ctypes.data, f.ctypes.data, _stream_ptr(stream)))
            return w[:n[0]].copy(), float(c[0]), int(f[0])
        with _on(stream):
            w = torch.zeros(cap, dtype=torch.int32, device="cuda")
            n = torch.zeros(1, dtype=torch.int32, device="cuda")
            c = torch.zeros(1, dtype=torch.float32, device="cuda")
            f = torch.zeros(1, dtype=torch.int32, device="cuda")
        self._check(self.lib.wfst_get_partial(self.h, ch, int(finalize), w.data_ptr(), cap, n.data_ptr(),
                                              c.data_ptr(), f.data_ptr(), _stream_ptr(stream)))
        if stream is not None:
            stream.synchronize()                 # the copies below run on torch's current stream
        k = int(n.item())
        return w[:k].cpu().numpy(), float(c.item()), int(f.item())

    def get_partial_batch(self, channels, finalize=False, stream=None, out=None):
        """Best hypotheses of several channels in one launch.  Returns (words [n, max_words],
        nwords [n], cost [n], flags [n]) as CUDA tensors, or numpy arrays with outputs_on_host."""
        import torch
        channels = np.ascontiguousarray(channels, dtype=np.int32)
        n = len(channels)
        if out is None:
            if self.outputs_on_host:
                out = (np.zeros((n, self.max_words), np.int32), np.zeros(n, np.int32),
                       np.zeros(n, np.float32), np.zeros(n, np.int32))
            else:
                with _on(stream):
                    out = (torch.zeros((n, self.max_words), dtype=torch.int32, device="cuda"),
                           torch.zeros(n, dtype=torch.int32, device="cuda"),
                           torch.zeros(n, dtype=torch.float32, device="cuda"),
                           torch.zeros(n, dtype=torch.int32, device="cuda"))
        ptr = (lambda a: a.ctypes.data) if self.outputs_on_host else (lambda t: t.data_ptr())
        self._check(self.lib.wfst_get_partial_batch(self.h, channels.ctypes.data, n, int(finalize),
                                                    ptr(out[0]), ptr(out[1]), ptr(out[2]), ptr(out[3]),
                                                    _stream_ptr(stream)))
        return out

    def get_lattice_noalloc(self, ch, loglikes, lattice_beam, tok_state, tok_cost, links, frame_off, stream=None):
        """wfst_get_lattice_noalloc: every buffer is the caller's (tok_state int32 / tok_cost float32
        CUDA tensors, links a CUDA uint8 tensor of 32-byte records, frame_off a host int64 array).
        Returns (n_tokens, n_links); raises on any status but OK."""
        nt, nl = C.c_int64(), C.c_int64()
        self._check(self.lib.wfst_get_lattice_noalloc(
            self.h, ch, loglikes.data_ptr(), float(lattice_beam), tok_state.data_ptr(), tok_cost.data_ptr(),
            tok_state.numel(), frame_off.ctypes.data, links.data_ptr(), links.numel() // LINK_DTYPE.itemsize,
            C.byref(nt), C.byref(nl), _stream_ptr(stream)))
        return nt.value, nl.value

    def get_lattice(self, ch, loglikes, lattice_beam, stream=None, tok_cap=None, link_cap=None, on_device=False):
        """wfst_get_lattice for channel `ch`; `loglikes` [frames, V] is the utterance's device
        tensor it was decoded with.  Returns a `Lattice` (host arrays), or with on_device=True the
        tuple (frame_off, state tensor, cost tensor, link bytes tensor, n_tokens, n_links) with the
        outputs left in device memory.  Without capacities the call is made twice: once to
        learn the sizes, once with buffers of that size."""
        import torch
        from .lattice import Lattice
        assert loglikes.is_cuda and loglikes.dtype == getattr(torch, self.loglike_dtype) and loglikes.is_contiguous()
        assert loglikes.ndim == 2 and loglikes.shape[1] == self.V
        off = np.zeros(self.opts.max_frames_per_channel + 2, np.int64)
        nt, nl = C.c_int64(), C.c_int64()

        def call(tc, lc):
            with _on(stream):
                st = torch.zeros(max(tc, 1), dtype=torch.int32, device="cuda")
                co = torch.zeros(max(tc, 1), dtype=torch.float32, device="cuda")
                lk = torch.zeros(max(lc, 1) * LINK_DTYPE.itemsize, dtype=torch.uint8, device="cuda")
            rc = self.lib.wfst_get_lattice(self.h, ch, loglikes.data_ptr(), float(lattice_beam),
                                           st.data_ptr(), co.data_ptr(), tc, off.ctypes.data, lk.data_ptr(), lc,
                                           C.byref(nt), C.byref(nl), _stream_ptr(stream))
            return rc, st, co, lk

        if tok_cap is None or link_cap is None:
            rc, *_ = call(0, 0)
            if rc not in (WFST_OK, -7) or (rc == -7 and nt.value == 0 and nl.value == 0):
                self._check(rc)
            tok_cap, link_cap = nt.value, nl.value
        rc, st, co, lk = call(tok_cap, link_cap)
        self._check(rc)
        if on_device:
            return off[:loglikes.shape[0] + 2].copy(), st, co, lk, nt.value, nl.value
        links = lk.cpu().numpy()[:nl.value * LINK_DTYPE.itemsize].view(LINK_DTYPE).copy()
        return Lattice(off[:loglikes.shape[0] + 2].copy(), st.cpu().numpy()[:nt.value].copy(),
                       co.cpu().numpy()[:nt.value].copy(), links)

    def get_lattice_batch(self, channels, loglikes, lengths, lattice_beam, stream=None, tok_cap=None, link_cap=None,
                          on_device=False):
        """wfst_get_lattice_batch: the lattices of several channels in one call.  `loglikes` [n, T, V] is
        the device tensor the channels were decoded with (channel channels[k] = row k, which has
        consumed lengths[k] frames).  Returns a list
        of `Lattice` (host arrays), or with on_device=True the tuple (frame_off [n, T+2], tok_first,
        link_first, state tensor, cost tensor, link bytes tensor) with the outputs left in device
        memory.  Without capacities the call is made twice: once to learn the sizes."""
        import torch
        from .lattice import Lattice
        channels = np.ascontiguousarray(channels, dtype=np.int32)
        n = len(channels)
        assert loglikes.is_cuda and loglikes.dtype == getattr(torch, self.loglike_dtype) and loglikes.is_contiguous()
        assert loglikes.ndim == 3 and loglikes.shape[0] == n and loglikes.shape[2] == self.V
        T = int(loglikes.shape[1])
        off = np.zeros((n, T + 2), np.int64)
        tf, lf = np.zeros(n + 1, np.int64), np.zeros(n + 1, np.int64)

        def call(tc, lc):
            with _on(stream):
                st = torch.zeros(max(tc, 1), dtype=torch.int32, device="cuda")
                co = torch.zeros(max(tc, 1), dtype=torch.float32, device="cuda")
                lk = torch.zeros(max(lc, 1) * LINK_DTYPE.itemsize, dtype=torch.uint8, device="cuda")
            rc = self.lib.wfst_get_lattice_batch(self.h, channels.ctypes.data, n, loglikes.data_ptr(), T,
                                                 float(lattice_beam), st.data_ptr(), co.data_ptr(), tc,
                                                 off.ctypes.data, lk.data_ptr(), lc, tf.ctypes.data, lf.ctypes.data,
                                                 _stream_ptr(stream))
            return rc, st, co, lk

        if tok_cap is None or link_cap is None:
            rc, *_ = call(0, 0)
            if rc not in (WFST_OK, -7) or (rc == -7 and tf[n] == 0 and lf[n] == 0):
                self._check(rc)
            tok_cap, link_cap = int(tf[n]), int(lf[n])
        rc, st, co, lk = call(tok_cap, link_cap)
        self._check(rc)
        if on_device:
            return off, tf.copy(), lf.copy(), st, co, lk
        sth, coh = st.cpu().numpy(), co.cpu().numpy()
        lkh = lk.cpu().numpy()[:int(lf[n]) * LINK_DTYPE.itemsize].view(LINK_DTYPE)
        out = []
        for k in range(n):
            out.append(Lattice(off[k, :int(lengths[k]) + 2].copy(), sth[tf[k]:tf[k + 1]].copy(),
                               coh[tf[k]:tf[k + 1]].copy(), lkh[lf[k]:lf[k + 1]].copy()))
        return out

    # ---- hooks
    def debug_frame_digests(self, ch):
        cap = self.opts.max_frames_per_channel + 1
        dig, cnt, n = np.zeros(cap, np.uint64), np.zeros(cap, np.int32), C.c_int32()
        self._check(self.lib.wfst_debug_frame_digests(self.h, ch, dig.ctypes.data, cnt.ctypes.data, cap, C.byref(n)))
        return cnt[:n.value].copy(), dig[:n.value].copy()

    def debug_get_tokens(self, ch, cap=1 << 20):
        st, co, n = np.zeros(cap, np.int32), np.zeros(cap, np.float32), C.c_int32()
        self._check(self.lib.wfst_debug_get_tokens(self.h, ch, st.ctypes.data, co.ctypes.data, cap, C.byref(n)))
        return st[:n.value].copy(), co[:n.value].copy()

    def debug_get_token_pairs(self, ch, cap=1 << 20):
        """(graph states, boosting-acceptor states, costs) of the channel's current token set."""
        st, bs, co, n = np.zeros(cap, np.int32), np.zeros(cap, np.int32), np.zeros(cap, np.float32), C.c_int32()
        self._check(self.lib.wfst_debug_get_token_pairs(self.h, ch, st.ctypes.data, bs.ctypes.data, co.ctypes.data,
                                                        cap, C.byref(n)))
        return st[:n.value].copy(), bs[:n.value].copy(), co[:n.value].copy()

    def get_counters(self, reset=False):
        c = np.zeros(8, np.int64)
        self._check(self.lib.wfst_get_counters(self.h, c.ctypes.data, int(reset)))
        return c

    def set_launch_workgroups(self, n):
        """At most n workgroups per launch from now on (0: one per utterance); see the header."""
        self._check(self.lib.wfst_set_launch_workgroups(self.h, int(n)))

    def debug_set_phase_timing(self, on=True):
        self._check(self.lib.wfst_debug_set_phase_timing(self.h, int(bool(on))))

    def debug_phase_ticks(self, reset=False):
        t = np.zeros(16, np.int64)
        self._check(self.lib.wfst_debug_phase_ticks(self.h, t.ctypes.data, int(reset)))
        return t

    def device_bytes(self):
        return int(self.lib.wfst_device_bytes(self.h))

    def last_kernel_ms(self):
        return float(self.lib.wfst_last_kernel_ms(self.h))

    def slot_kernel_ms(self, slot):
        return float(self.lib.wfst_slot_kernel_ms(self.h, int(slot)))
