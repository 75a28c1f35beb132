"""CPU-only: the shared library loads and exports every function the header declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "flatformer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ff_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = _declared()
    for must in ("ff_flatten", "ff_group_attention", "ff_gather", "ff_scatter", "ff_fwa_block"):
        assert must in names


def test_library_exports_every_declared_symbol():
    import paper_2301_08739_amd as ff
    if not os.path.exists(ff.library_path()):
        pytest.skip("library not built (run __graft_entry__.build())")
    lib = ctypes.CDLL(ff.library_path())
    for name in _declared():
        assert hasattr(lib, name), name
    assert set(_declared()) == set(ff.exported_symbols())
    ff.load_library()
    assert ff.ff_version() >= 100
    assert ff.ff_status_string(0) == "ok" and "unsupported" in ff.ff_status_string(-2)


def test_host_side_workspace_queries_need_no_gpu():
    import paper_2301_08739_amd as ff
    if not os.path.exists(ff.library_path()):
        pytest.skip("library not built")
    g = ff.Geometry(1, 468, 468, 13, 13)
    a = ff.ff_flatten_workspace_bytes(30000, g)
    b = ff.ff_flatten_workspace_bytes(60000, g)
    assert 0 < a < b
    assert ff.ff_flatten_workspace_bytes(-1, g) == 0
    assert ff.ff_flatten_workspace_bytes(10, ff.Geometry(1, 468, 468, 0, 13)) == 0
