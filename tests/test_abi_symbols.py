"""Host-side checks of the C-ABI library: it loads without a GPU, exports every function that
include/mixgcn.h declares, and the Python structs match the header's layout."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mixgcn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mixgcn_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_six_calls():
    names = declared_functions()
    for f in ("mixgcn_build_csr", "mixgcn_normalize", "mixgcn_aggregate", "mixgcn_update",
              "mixgcn_layer_fwd", "mixgcn_layer_bwd"):
        assert f in names


def test_library_exports_every_declared_symbol():
    import paper_2501_01951_amd as m

    lib = m.load_library()
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in mixgcn.h but not exported"
    assert lib.mixgcn_version() == 100
    assert lib.mixgcn_strerror(-1) == b"invalid argument"
    assert lib.mixgcn_strerror(0) == b"ok"


def test_struct_layouts_match_header():
    from paper_2501_01951_amd.binding import LayerDesc, _GraphView

    # mixgcn_layer_desc: 2 x int32, 4 x int64, 4 x int32
    assert ctypes.sizeof(LayerDesc) == 2 * 4 + 4 * 8 + 4 * 4
    assert LayerDesc.ld_h.offset == 8 and LayerDesc.ld_w.offset == 32 and LayerDesc.dtype.offset == 40
    # mixgcn_graph_view: 2 x uint32, int64, 8 pointers
    assert ctypes.sizeof(_GraphView) == 8 + 8 + 8 * 8
    assert _GraphView.rowptr.offset == 16


def test_argument_errors_need_no_gpu():
    """Calls that fail validation before touching the device."""
    import paper_2501_01951_amd as m

    lib = m.load_library()
    out = ctypes.c_void_p()
    assert lib.mixgcn_build_csr(None, None, 0, 0, 3, None, ctypes.byref(out)) == -1  # n_nodes == 0
    assert b"n_nodes" in lib.mixgcn_last_error()
    assert lib.mixgcn_build_csr(None, None, 5, 10, 3, None, ctypes.byref(out)) == -1  # null edges
    assert lib.mixgcn_build_csr(None, None, 0, 10, 1 << 9, None, ctypes.byref(out)) == -1  # flag
    assert lib.mixgcn_normalize(None, 0, None) == -1
    assert lib.mixgcn_graph_free(None) == 0
    assert lib.mixgcn_update(9, 0, None, 0, None, 0, None, 0, 1, 1, 1, None, 0, 0.0, None) == -1
    assert lib.mixgcn_update(0, 0, None, 4, None, 4, None, 4, 1, 4, 4, None, 0, 0.0, None) == -1
