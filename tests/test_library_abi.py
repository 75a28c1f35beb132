"""CPU-only: the shared library loads and exports every function the header declares."""
import ctypes
import os
import re
import shutil
import subprocess

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
    # and nothing else with C linkage leaks out of the library
    nm = shutil.which("nm")
    if nm:
        out = subprocess.run([nm, "-D", "--defined-only", ff.library_path()], capture_output=True, text=True, check=True).stdout
        c_funcs = {ln.split()[2] for ln in out.splitlines() if len(ln.split()) == 3 and ln.split()[1] == "T" and not ln.split()[2].startswith("_")}
        assert c_funcs == set(_declared()), sorted(c_funcs ^ set(_declared()))
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


def test_argument_errors_are_reported_before_any_launch():
    """Every entry point checks its arguments on the host and returns a status code; these calls
    never reach a kernel launch, so they run without a GPU."""
    import paper_2301_08739_amd as ff
    from paper_2301_08739_amd.binding import _LayerWeightsC, VoxelGrid
    if not os.path.exists(ff.library_path()):
        pytest.skip("library not built")
    lib = ff.load_library()
    g = ff.Geometry(1, 468, 468, 13, 13)
    gp = ctypes.byref(g)
    one = ctypes.c_void_p(256)                     # a non-null, aligned address that is never dereferenced
    null = ctypes.c_void_p(0)
    # flatten: bad tail mode, bad shift, G < 1, missing outputs
    assert lib.ff_flatten(one, 10, gp, 0, 0, 4, 7, one, one, one, null, one, 1 << 20, null) == -1
    assert lib.ff_flatten(one, 10, gp, 0, 3, 4, 0, one, one, one, null, one, 1 << 20, null) == -1
    assert lib.ff_flatten(one, 10, gp, 0, 0, 0, 0, one, one, one, null, one, 1 << 20, null) == -1
    assert lib.ff_flatten(one, 10, gp, 0, 0, 4, 0, one, null, one, null, one, 1 << 20, null) == -1
    assert lib.ff_flatten(one, 10, gp, 0, 0, 4, 0, one, one, one, null, one, 16, null) == -3     # workspace too small
    # the same with a third coordinate: bad tail, bad z window, key too wide, workspace too small
    g3 = ff.Geometry3(1, 468, 468, 40, 13, 13, 4)
    g3p = ctypes.byref(g3)
    assert lib.ff_flatten3d(one, 10, g3p, 0, 0, 4, 7, one, one, one, one, 1 << 20, null) == -1
    assert lib.ff_flatten3d(one, 10, ctypes.byref(ff.Geometry3(1, 468, 468, 40, 13, 13, 0)), 0, 0, 4, 0, one, one, one,
                            one, 1 << 20, null) == -1
    assert lib.ff_flatten3d(one, 10, ctypes.byref(ff.Geometry3(65535, 65535, 65535, 65535, 1, 1, 1)), 0, 0, 4, 0, one,
                            one, one, one, 1 << 20, null) == -2
    assert lib.ff_flatten3d(one, 10, g3p, 0, 0, 4, 0, one, one, one, one, 16, null) == -3
    assert 0 < lib.ff_flatten3d_workspace_bytes(30000, g3p) < lib.ff_flatten3d_workspace_bytes(60000, g3p)
    assert lib.ff_fwa_block3d(one, 10, g3p, 64, 9, ctypes.byref(_LayerWeightsC()), 1, 1, one, ctypes.c_void_p(1 << 20), one,
                              1 << 30, null) == -1
    # layer: incomplete weights, C not divisible by heads, overlapping buffers, workspace missing
    w = _LayerWeightsC()
    wp = ctypes.byref(w)
    assert lib.ff_group_attention(one, one, 10, one, one, one, 3, wp, 4, 1, 0, one, 1 << 20, null) == -1
    for k, _ in _LayerWeightsC._fields_[:12]:
        setattr(w, k, 256)
    w.C, w.F, w.heads, w.ln_eps = 128, 256, 7, 1e-5
    assert lib.ff_group_attention(one, ctypes.c_void_p(1 << 20), 10, one, one, one, 3, wp, 4, 1, 0, one, 1 << 20, null) == -2
    w.heads = 8
    assert lib.ff_group_attention(one, one, 10, one, one, one, 3, wp, 4, 1, 0, one, 1 << 20, null) == -1  # in == out
    assert lib.ff_group_attention(one, ctypes.c_void_p(1 << 20), 10, one, one, one, 3, wp, 2000, 1, 0, one, 1 << 20, null) == -2
    assert lib.ff_group_attention(one, ctypes.c_void_p(1 << 20), 10, one, one, one, 3, wp, 64, 1, 0, null, 0, null) == -3
    assert lib.ff_group_attention(one, ctypes.c_void_p(1 << 20), 10, one, one, one, 3, wp, 64, 5, 0, one, 1 << 20, null) == -1  # dtype
    assert lib.ff_pack_weights(wp, 0, one, null) == -2                                             # fp32 has no packed form
    assert lib.ff_pack_weights_bytes(wp, 1) == lib.ff_pack_weights_bytes(wp, 2) > 256 * 1024
    # rows, dense map, voxelisation, block
    assert lib.ff_gather(one, one, one, 10, 100, 1, null) == -2                                    # row bytes not a multiple of 16
    assert lib.ff_scatter(one, one, one, -1, 128, 1, null) == -1
    assert lib.ff_bev_scatter(one, one, 10, gp, 128, 1, null, null) == -1
    v = VoxelGrid(0.0, 0.0, 0.0, 0.32)
    assert lib.ff_voxelize(one, null, one, 10, 4, gp, ctypes.byref(v), one, one, one, null, one, 1 << 30, null) == -1
    assert lib.ff_fwa_block(one, 10, gp, 64, 9, wp, 1, 1, one, ctypes.c_void_p(1 << 20), one, 1 << 30, null) == -1   # tail mode
    assert lib.ff_fwa_block(one, 10, gp, 64, 0, wp, 1, 1, one, ctypes.c_void_p(1 << 20), one, 16, null) == -3


def test_bench_only_library_exports_its_two_entry_points():
    import paper_2301_08739_amd as ff
    path = os.path.join(os.path.dirname(ff.library_path()), "libffpeaks.so")
    if not os.path.exists(path):
        pytest.skip("library not built (run __graft_entry__.build())")
    lib = ctypes.CDLL(path)
    assert hasattr(lib, "ffpeak_stream_copy") and hasattr(lib, "ffpeak_mfma_bf16")
