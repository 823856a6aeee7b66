"""MI355X-native WFST beam-search decoder for CTC models (HIP kernels behind a C ABI)."""
from .binding import (Decoder, WfstError, load_library, EXPORTS, FLAG_REACHED_FINAL, FLAG_TRUNCATED,
                      FLAG_DEAD, FLAG_LATTICE_OVERFLOW, FLAG_CAPACITY)
from .build import build_library, LIB_PATH
from .lattice import Lattice

__all__ = ["Decoder", "Lattice", "WfstError", "load_library", "build_library", "LIB_PATH", "EXPORTS",
           "FLAG_REACHED_FINAL", "FLAG_TRUNCATED", "FLAG_DEAD", "FLAG_LATTICE_OVERFLOW", "FLAG_CAPACITY"]
