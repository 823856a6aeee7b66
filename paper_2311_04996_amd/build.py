"""Build step: compiles the HIP decoder for gfx950 into libwfstdec.so next to this file."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
LIB_PATH = os.path.join(_HERE, "libwfstdec.so")
SOURCES = [os.path.join(_HERE, "csrc", "wfst_decoder.hip")]
HEADERS = [os.path.join(ROOT, "include", "wfst_decoder.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                       # costs are compared bit for bit: no FMA contraction
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"),
]


def build_library(verbose: bool = False) -> str:
    """Always recompiles.  Returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB_PATH] + SOURCES
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd, stderr=None if verbose else subprocess.DEVNULL)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
