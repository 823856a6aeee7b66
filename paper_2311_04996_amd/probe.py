"""ctypes binding over libwfstprobe.so (include/wfst_probe.h): measured ceilings of the GPU."""
from __future__ import annotations

import ctypes as C
import os

from .build import PROBE_LIB_PATH

EXPORTS = ["wfst_probe_copy", "wfst_probe_random_lines", "wfst_probe_atomics"]
_lib = None


def load_probe_library():
    global _lib
    if _lib is None:
        if not os.path.exists(PROBE_LIB_PATH):
            raise RuntimeError(f"{PROBE_LIB_PATH} is missing: run `python -m paper_2311_04996_amd.build` first")
        import torch  # noqa: F401  (one HIP runtime per process: bind to torch's)
        lib = C.CDLL(PROBE_LIB_PATH)
        lib.wfst_probe_copy.argtypes = [C.c_int64, C.c_int32, C.POINTER(C.c_double)]
        lib.wfst_probe_random_lines.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.POINTER(C.c_double)]
        lib.wfst_probe_atomics.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.POINTER(C.c_double)]
        for name in EXPORTS:
            getattr(lib, name).restype = C.c_int32
        _lib = lib
    return _lib


def _call(fn, *args):
    out = C.c_double()
    if fn(*args, C.byref(out)) != 0:
        raise RuntimeError(f"{fn.__name__} failed")
    return out.value


def probe_copy(nbytes=1 << 30, reps=5):
    """GB/s (read + written) of a plain device copy."""
    return _call(load_probe_library().wfst_probe_copy, nbytes, reps)


def probe_random_lines(footprint=1 << 32, workgroups=1024, loads_per_lane=256):
    """Random 128-byte line requests per second."""
    return _call(load_probe_library().wfst_probe_random_lines, footprint, workgroups, loads_per_lane)


def probe_atomics(footprint=1 << 30, workgroups=1024, atomics_per_lane=64):
    """Random 64-bit global atomics per second."""
    return _call(load_probe_library().wfst_probe_atomics, footprint, workgroups, atomics_per_lane)
