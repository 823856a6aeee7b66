"""CPU-only checks of the C-ABI library: it loads and exports every declared symbol."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2311_04996_amd import LIB_PATH, build_library, load_library
    if not os.path.exists(LIB_PATH):
        build_library()
    return load_library()


def declared_functions(header="wfst_decoder.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(wfst_[a-z_]+)\s*\(", text)))


def test_every_header_is_covered():
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["wfst_decoder.h", "wfst_probe.h"]


def test_probe_library_exports_what_its_header_declares():
    from paper_2311_04996_amd.build import PROBE_LIB_PATH, build_library
    from paper_2311_04996_amd.probe import EXPORTS, load_probe_library
    if not os.path.exists(PROBE_LIB_PATH):
        build_library()
    lib = load_probe_library()
    names = declared_functions("wfst_probe.h")
    assert names == sorted(EXPORTS) and len(names) == 3
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/wfst_probe.h but not exported"
    out = ctypes.c_double()
    assert lib.wfst_probe_copy(0, 1, ctypes.byref(out)) == -1          # bad arguments: rejected before any GPU call
    assert lib.wfst_probe_random_lines(1 << 30, 0, 64, ctypes.byref(out)) == -1
    assert lib.wfst_probe_atomics(1 << 30, 4, 64, None) == -1


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/wfst_decoder.h but not exported"


def test_binding_lists_the_same_names():
    from paper_2311_04996_amd import EXPORTS
    assert sorted(EXPORTS) == declared_functions()


def test_link_record_layout():
    import numpy as np
    from paper_2311_04996_amd.binding import LINK_DTYPE, wfst_lattice_link
    assert ctypes.sizeof(wfst_lattice_link) == 32 == LINK_DTYPE.itemsize
    for name, _ in wfst_lattice_link._fields_:
        assert getattr(wfst_lattice_link, name).offset == LINK_DTYPE.fields[name][1]


def test_null_arguments_are_errors_not_crashes(lib):
    h = ctypes.c_void_p()
    assert lib.wfst_decoder_create(None, None, ctypes.byref(h)) == -1
    assert b"null" in lib.wfst_last_error(None)
    assert lib.wfst_decoder_destroy(None) == 0
    assert lib.wfst_device_bytes(None) == 0


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2311_04996_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower(), (f, "mentions the oracle")


def _create(lib, arcs, S, V, final=None, loglike_dtype=0):
    import numpy as np
    from paper_2311_04996_amd.binding import wfst_graph_csr, wfst_opts
    from workloads.graphs import _from_arc_list
    g = _from_arc_list(S, 0, V, arcs, np.zeros(S, np.float32) if final is None else final)
    keep = [g.row_offsets, g.next_state, g.ilabel, g.olabel, g.weight, g.final_cost]
    cg = wfst_graph_csr(g.num_states, g.start_state, g.num_classes, g.num_arcs,
                        *[a.ctypes.data for a in keep])
    o = wfst_opts(1, 10, 8, 0, 0, 100, 0, 0, loglike_dtype)
    h = ctypes.c_void_p()
    rc = lib.wfst_decoder_create(ctypes.byref(cg), ctypes.byref(o), ctypes.byref(h))
    return rc, lib.wfst_last_error(None).decode()


def test_bad_graphs_are_rejected_before_touching_the_gpu(lib):
    rc, msg = _create(lib, [(0, 1, 0, 0, 1.0), (1, 0, 0, 0, -1.0)], 2, 1)
    assert rc == -2 and "cycle" in msg
    rc, msg = _create(lib, [(0, 1, 2, 0, 1.0)], 2, 1)
    assert rc == -2 and "ilabel" in msg
    rc, msg = _create(lib, [(0, 1, 1, 0, float("inf"))], 2, 1)
    assert rc == -2 and "weight" in msg
    rc, msg = _create(lib, [(0, 1, 1, -3, 0.5)], 2, 1)
    assert rc == -2 and "olabel" in msg
    # more epsilon arcs out of one state than the state header's 12-bit field holds
    rc, msg = _create(lib, [(0, 1, 0, 0, 0.5)] * 5000, 2, 1)
    assert rc == -2 and "epsilon arcs" in msg
    rc, msg = _create(lib, [(0, 1, 1, 0, 0.5)], 2, 1, loglike_dtype=7)
    assert rc == -1 and "loglike_dtype" in msg


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 on its own."""
    import subprocess
    src = tmp_path / "h.c"
    src.write_text('#include "wfst_decoder.h"\n#include "wfst_probe.h"\nint main(void) { wfst_opts o; wfst_lattice_link l; (void)o; (void)l;'
                   ' return sizeof(wfst_lattice_link) == 32 ? 0 : 1; }\n')
    exe = tmp_path / "h"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror",
                           "-I" + os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    assert subprocess.call([str(exe)]) == 0
