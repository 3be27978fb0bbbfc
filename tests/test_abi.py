"""The C-ABI library loads and exports every symbol include/rgnn.h declares (no GPU needed)."""
import os
import re

from paper_2412_04747_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _ensure_built():
    if not os.path.exists(B.LIB_PATH):
        from paper_2412_04747_amd import build
        build.build()


def test_header_symbols_are_exported():
    _ensure_built()
    header = open(os.path.join(ROOT, "include", "rgnn.h")).read()
    declared = set(re.findall(r"\b(rgnn_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert hasattr(lib, name), name


def test_index_enum_matches_binding():
    header = open(os.path.join(ROOT, "include", "rgnn.h")).read()
    enum = re.findall(r"RGNN_IDX_([A-Z_]+)\s*=\s*(\d+)", header)
    names = [n.lower() for n, _ in enum if n != "COUNT"]
    assert names == B.INDEX_NAMES
    assert [int(v) for _, v in enum] == list(range(len(enum)))


def test_argument_errors_without_gpu():
    _ensure_built()
    import ctypes as C
    lib = B.lib()
    g = C.c_void_p()
    # bad sizes are rejected before any device call
    st = lib.rgnn_graph_create(C.byref(g), C.c_int64(-1), C.c_int32(1), C.c_int32(1), C.c_int64(0), 0, None, None,
                               None, None, None, None, 0)
    assert st == 1 and g.value is None and b"num_nodes" in lib.rgnn_last_error()
    st = lib.rgnn_graph_create(C.byref(g), C.c_int64(4), C.c_int32(2), C.c_int32(1), C.c_int64(0), 0, None, None,
                               None, None, None, None, 0)
    assert st == 1 and b"ntype" in lib.rgnn_last_error()
    assert lib.rgnn_graph_destroy(None) == 0
    assert lib.rgnn_graph_info(None, None) == 1
