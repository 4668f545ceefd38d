"""Host-only checks of the C-ABI library: it loads, exports every symbol the header
declares, and validates arguments before touching the GPU (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "molgrid_hip.h")
LIB = os.path.join(ROOT, "paper_1912_04822_amd", "libmolgrid_hip.so")


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(LIB):
        from paper_1912_04822_amd import build
        build.build_library()
    return ctypes.CDLL(LIB)


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mg_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(L, n), n
    from paper_1912_04822_amd import molgrid
    assert sorted(molgrid.EXPORTS) == names


def make(L, *args):
    h = ctypes.c_void_p()
    L.mg_gridmaker_create.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_float,
                                      ctypes.c_float, ctypes.c_int, ctypes.c_int, ctypes.c_float,
                                      ctypes.c_float]
    rc = L.mg_gridmaker_create(ctypes.byref(h), *args)
    return rc, h


def test_create_validates_and_reports_points_per_side(L):
    rc, h = make(L, 0.5, 23.5, 0, 0, 1.0, 1.0)         # the paper's defaults
    assert rc == 0 and h.value
    d = ctypes.c_int()
    L.mg_gridmaker_points_per_side.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_int)]
    assert L.mg_gridmaker_points_per_side(h, ctypes.byref(d)) == 0 and d.value == 48
    L.mg_gridmaker_destroy.argtypes = [ctypes.c_void_p]
    L.mg_gridmaker_destroy(h)
    for res, dim, D in [(0.25, 23.75, 96), (0.5, 11.5, 24), (0.75, 9.0, 13), (1.0, 0.0, 1)]:
        rc, h = make(L, res, dim, 0, 1, 1.0, 1.0)
        assert rc == 0
        L.mg_gridmaker_points_per_side(h, ctypes.byref(d))
        assert d.value == D
        L.mg_gridmaker_destroy(h)
    bad = [(0.0, 23.5, 0, 0, 1.0, 1.0), (-0.5, 23.5, 0, 0, 1.0, 1.0),
           (float("nan"), 23.5, 0, 0, 1.0, 1.0), (0.5, float("inf"), 0, 0, 1.0, 1.0),
           (0.5, 23.5, 0, 0, 0.0, 1.0), (0.5, 23.5, 0, 0, 1.0, 0.0),
           (0.5, 23.5, 0, 0, 1.0, float("nan")), (0.5, -1.0, 0, 0, 1.0, 1.0)]
    for args in bad:
        rc, h = make(L, *args)
        assert rc == -3 and not h.value, args                   # MG_EPARAM
    rc, h = make(L, 0.01, 100.0, 0, 0, 1.0, 1.0)                # D = 10001 > MG_MAX_POINTS
    assert rc == -2
    assert L.mg_gridmaker_create(None, ctypes.c_float(0.5), ctypes.c_float(23.5), 0, 0,
                                 ctypes.c_float(1.0), ctypes.c_float(1.0)) == -1


def test_calls_reject_bad_arguments_before_any_launch(L):
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.mg_forward_index.argtypes = [vp, ci, ci, ci] + [vp] * 8 + [vp, sz, vp]
    L.mg_backward_index.argtypes = [vp, ci, ci, ci] + [vp] * 9 + [vp, sz, vp]
    L.mg_forward_vector.argtypes = [vp, ci, ci, ci] + [vp] * 8 + [vp, sz, vp]
    L.mg_workspace_bytes.argtypes = [vp, ci, ci, ci, ctypes.POINTER(sz)]
    rc, h = make(L, 0.5, 23.5, 0, 1, 1.0, 1.0)
    assert rc == 0
    n = sz()
    assert L.mg_workspace_bytes(h, 50, 2040, 28, ctypes.byref(n)) == 0
    # records 16 B + atom index 4 B + channel 4 B + liveness 1 B per atom; group table, plane spans and channel
    # order per (example, type); pose and centre per example; the tag
    assert 50 * 2040 * 25 <= n.value <= 50 * 2040 * 25 + 50 * 28 * (16 + 48 * 8 + 4) + 50 * 64 + 128
    assert L.mg_workspace_bytes(h, 0, 2040, 28, ctypes.byref(n)) == -2
    # a subgrid decomposition: S^3 virtual examples per example, plus the gradient staging
    L.mg_gridmaker_create_subgrids.argtypes = [ctypes.POINTER(vp), ctypes.c_float, ctypes.c_float,
                                               ci, ci, ci, ctypes.c_float, ctypes.c_float]
    hs = vp()
    assert L.mg_gridmaker_create_subgrids(ctypes.byref(hs), 0.5, 11.5, 2, 0, 1, 1.0, 1.0) == 0
    m = sz()
    assert L.mg_workspace_bytes(hs, 50, 2040, 28, ctypes.byref(m)) == 0
    assert m.value >= 8 * 50 * 2040 * (20 + 12 + 28 * 4)
    s_ = ci()
    L.mg_gridmaker_subgrids_per_side.argtypes = [vp, ctypes.POINTER(ci)]
    assert L.mg_gridmaker_subgrids_per_side(hs, ctypes.byref(s_)) == 0 and s_.value == 2
    assert L.mg_gridmaker_subgrids_per_side(h, ctypes.byref(s_)) == 0 and s_.value == 1
    assert L.mg_workspace_bytes(hs, 9000, 10, 4, ctypes.byref(m)) == -2      # 72000 virtual examples
    for bad in (0, -3, 17):
        assert L.mg_gridmaker_create_subgrids(ctypes.byref(vp()), 0.5, 11.5, bad, 0, 1, 1.0, 1.0) == -2
    L.mg_gridmaker_destroy.argtypes = [vp]
    L.mg_gridmaker_destroy(hs)
    assert L.mg_workspace_bytes(h, 50, 2040, 28, None) == -1
    assert L.mg_workspace_bytes(None, 50, 2040, 28, ctypes.byref(n)) == -1
    fake = vp(0x1000)       # never dereferenced: validation fails first
    # NULL required pointers
    assert L.mg_forward_index(h, 1, 1, 1, None, fake, fake, None, None, None, None, fake, fake,
                              1 << 20, None) == -1
    assert L.mg_forward_index(h, 1, 1, 1, fake, fake, fake, None, None, None, None, None, fake,
                              1 << 20, None) == -1
    # bad shapes
    assert L.mg_forward_index(h, 0, 1, 1, fake, fake, fake, None, None, None, None, fake, fake,
                              1 << 20, None) == -2
    assert L.mg_forward_index(h, 1, 1, -4, fake, fake, fake, None, None, None, None, fake, fake,
                              1 << 20, None) == -2
    assert L.mg_forward_index(h, 70000, 1, 1, fake, fake, fake, None, None, None, None, fake, fake,
                              1 << 30, None) == -2
    # workspace missing / too small / misaligned
    assert L.mg_forward_index(h, 1, 100, 4, fake, fake, fake, None, None, None, None, fake, None,
                              1 << 20, None) == -4
    assert L.mg_forward_index(h, 1, 100, 4, fake, fake, fake, None, None, None, None, fake, fake,
                              16, None) == -4
    assert L.mg_forward_index(h, 1, 100, 4, fake, fake, fake, None, None, None, None, fake,
                              vp(0x1008), 1 << 20, None) == -4
    # misaligned float array
    assert L.mg_forward_index(h, 1, 100, 4, vp(0x1002), fake, fake, None, None, None, None, fake,
                              fake, 1 << 20, None) == -7
    # backward is not defined in binary mode; vector types need radii per type
    rc, hb = make(L, 0.5, 23.5, 1, 1, 1.0, 1.0)
    assert L.mg_backward_index(hb, 1, 1, 1, fake, fake, fake, None, None, None, None, fake, fake,
                               fake, 1 << 20, None) == -6
    rc, hp = make(L, 0.5, 23.5, 0, 0, 1.0, 1.0)
    assert L.mg_forward_vector(hp, 1, 1, 1, fake, fake, fake, None, None, None, None, fake, fake,
                               1 << 20, None) == -6
    L.mg_strerror.restype = ctypes.c_char_p
    for code in range(-8, 1):
        assert len(L.mg_strerror(code)) > 1
    assert b"unknown" in L.mg_strerror(-99)
    L.mg_set_option.argtypes = [ctypes.c_char_p, ci]
    assert L.mg_set_option(b"tile_floats", 2048) == 0
    assert L.mg_set_option(b"tile_floats", 0) == 0
    assert L.mg_set_option(b"tile_floats", 1000) == -3
    assert L.mg_set_option(b"nope", 0) == -3
    # the timing aids (which write wrong grids) are not in the library as built by default
    assert L.mg_set_option(b"debug", 1) == -3
    assert L.mg_set_option(b"prep_stop", 3) == -3
    for key, bad in ((b"waves_per_tile", 3), (b"waves_per_tile", 8), (b"xcd_run", -1),
                     (b"lds_floor", -2), (b"keep_alive", -1), (b"tile_order", -1)):
        assert L.mg_set_option(key, bad) == -3
    for key, good, bad, default in ((b"keep_alive", 0, 2, 1), (b"tile_order", 1, 2, 0),
                                    (b"single_launch", 0, 2, 1), (b"keep_alive_stride", 4, 3, 1),
                                    (b"lds_floor", 8192, 70000, -1), (b"xcd_run", 8, 12, 0)):
        assert L.mg_set_option(key, good) == 0
        assert L.mg_set_option(key, bad) == -3
        assert L.mg_set_option(key, default) == 0
    for hh in (h, hb, hp):
        L.mg_gridmaker_destroy(hh)


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU; with --gpus above 1 it says so and exits (before touching a GPU)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_static_workspace_call_refuses_sizes_beyond_its_array_on_the_host(L):
    """mg_forward_index_static holds its workspace in an 8 MiB static device array; a problem
    whose tables do not fit is refused before the device is asked for anything."""
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.mg_forward_index_static.argtypes = [vp, ci, ci, ci] + [vp] * 8 + [vp]
    L.mg_workspace_bytes.argtypes = [vp, ci, ci, ci, ctypes.POINTER(sz)]
    rc, h = make(L, 0.5, 23.5, 0, 1, 1.0, 1.0)
    assert rc == 0
    n = sz()
    assert L.mg_workspace_bytes(h, 400, 2040, 28, ctypes.byref(n)) == 0 and n.value > 8 << 20
    fake = vp(4096)         # never dereferenced: the size check comes first
    assert L.mg_forward_index_static(h, 400, 2040, 28, fake, fake, fake, None, None, None, None,
                                     fake, None) == -4          # MG_EWORKSPACE
    assert L.mg_forward_index_static(None, 1, 1, 1, fake, fake, fake, None, None, None, None,
                                     fake, None) == -1          # MG_ENULL
    assert L.mg_forward_index_static(h, 0, 1, 1, fake, fake, fake, None, None, None, None,
                                     fake, None) == -2          # MG_ESHAPE
    assert L.mg_forward_index_static(h, 1, 1, 1, None, fake, fake, None, None, None, None,
                                     fake, None) == -1          # no coords
    L.mg_gridmaker_destroy.argtypes = [vp]
    L.mg_gridmaker_destroy(h)
