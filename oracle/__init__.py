"""CPU oracle for the atom-to-grid path -- TEST INFRASTRUCTURE, not product code.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares nothing with the HIP library
(``paper_1912_04822_amd``) and neither imports the other.

The arithmetic lives in ``molgrid_oracle.c`` (plain C, double precision, one
fixed float sequence for the binary predicate); this module only compiles that
file with gcc and marshals numpy arrays into it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "molgrid_oracle.c")
_LIB = os.path.join(_HERE, "libmolgrid_oracle.so")

_lib: Optional[ctypes.CDLL] = None

_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off: no fused multiply-add."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.orc_cutoff.restype = ctypes.c_double
        L.orc_cutoff.argtypes = [ctypes.c_double]
        L.orc_density.restype = ctypes.c_double
        L.orc_density.argtypes = [ctypes.c_double, ctypes.c_double]
        L.orc_density_deriv.restype = ctypes.c_double
        L.orc_density_deriv.argtypes = [ctypes.c_double, ctypes.c_double]
        L.orc_points_per_side.restype = ctypes.c_int
        L.orc_points_per_side.argtypes = [ctypes.c_double, ctypes.c_double]
        L.orc_quat_to_matrix.restype = None
        L.orc_quat_to_matrix.argtypes = [_f32p, _f64p]
        _lib = L
    return _lib


def _f32(a, shape=None):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _i32(a, shape=None):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.int32)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _p(a, typ):
    return a.ctypes.data_as(typ) if a is not None else typ()


# --------------------------------------------------------------------------
# scalar functions
# --------------------------------------------------------------------------

def cutoff(g: float) -> float:
    return lib().orc_cutoff(float(g))


def density(x: float, g: float = 1.0) -> float:
    return lib().orc_density(float(x), float(g))


def density_deriv(x: float, g: float = 1.0) -> float:
    return lib().orc_density_deriv(float(x), float(g))


def points_per_side(resolution: float, dimension: float) -> int:
    return lib().orc_points_per_side(float(resolution), float(dimension))


def quat_to_matrix(q) -> np.ndarray:
    q = _f32(q, (4,))
    R = np.empty(9, dtype=np.float64)
    lib().orc_quat_to_matrix(_p(q, _f32p), _p(R, _f64p))
    return R.reshape(3, 3)


# --------------------------------------------------------------------------
# batch functions
# --------------------------------------------------------------------------

def transform(coords, centers=None, quats=None, translations=None, as_float=True):
    """x' = R(q)(x - c) + c + t per example.  Returns float32 (rounded once) or float64."""
    coords = _f32(coords)
    B, N, _ = coords.shape
    centers = _f32(centers, (B, 3))
    quats = _f32(quats, (B, 4))
    translations = _f32(translations, (B, 3))
    o32 = np.empty((B, N, 3), np.float32) if as_float else None
    o64 = None if as_float else np.empty((B, N, 3), np.float64)
    lib().orc_transform(ctypes.c_int(B), ctypes.c_int(N), _p(coords, _f32p),
                        _p(centers, _f32p), _p(quats, _f32p), _p(translations, _f32p),
                        _p(o32, _f32p), _p(o64, _f64p))
    return o32 if as_float else o64


def transform_inverse(coords, centers=None, quats=None, translations=None, as_float=True):
    """x = R(q)^T ((x' - t) - c) + c per example.  Returns float32 (rounded once) or float64."""
    coords = _f32(coords)
    B, N, _ = coords.shape
    centers = _f32(centers, (B, 3))
    quats = _f32(quats, (B, 4))
    translations = _f32(translations, (B, 3))
    o32 = np.empty((B, N, 3), np.float32) if as_float else None
    o64 = None if as_float else np.empty((B, N, 3), np.float64)
    lib().orc_transform_inverse(ctypes.c_int(B), ctypes.c_int(N), _p(coords, _f32p),
                                _p(centers, _f32p), _p(quats, _f32p), _p(translations, _f32p),
                                _p(o32, _f32p), _p(o64, _f64p))
    return o32 if as_float else o64


def philox4x32_10(counter, key) -> np.ndarray:
    """One block of the Philox-4x32-10 bijection: 4 counter words, 2 key words -> 4 words."""
    c = np.ascontiguousarray(counter, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    o = np.empty(4, np.uint32)
    u32p = ctypes.POINTER(ctypes.c_uint32)
    lib().orc_philox4x32_10(c.ctypes.data_as(u32p), k.ctypes.data_as(u32p), o.ctypes.data_as(u32p))
    return o


def draw_transforms(seed: int, draw: int, B: int, random_rotation: bool = True,
                    max_translation: float = 0.0):
    """Per-example random quaternions [B,4] (w,x,y,z) and translations [B,3] (float32)."""
    q = np.empty((B, 4), np.float32)
    t = np.empty((B, 3), np.float32)
    lib().orc_draw_transforms(ctypes.c_uint64(seed & (2**64 - 1)), ctypes.c_uint64(draw & (2**64 - 1)),
                              ctypes.c_int(B), ctypes.c_int(1 if random_rotation else 0),
                              ctypes.c_double(max_translation), _p(q, _f32p), _p(t, _f32p))
    return q, t


def _common(coords, natoms, centers, quats, translations):
    coords = _f32(coords)
    B, N, three = coords.shape
    assert three == 3
    return (coords, B, N, _i32(natoms, (B,)), _f32(centers, (B, 3)), _f32(quats, (B, 4)),
            _f32(translations, (B, 3)))


def forward_index(coords, types, radii, T, resolution, dimension, *, grm=1.0,
                  radius_scale=1.0, radius_type_indexed=True, natoms=None, centers=None,
                  quats=None, translations=None, box=True, coords_as_float=True,
                  out_dtype=np.float32, threads=0, return_threads=False):
    """Real-valued density grid [B,T,D,D,D] for index-typed atoms."""
    coords, B, N, natoms, centers, quats, translations = _common(
        coords, natoms, centers, quats, translations)
    types = _i32(types, (B, N))
    radii = _f32(radii, (T,) if radius_type_indexed else (B, N))
    D = points_per_side(resolution, dimension)
    f64 = np.dtype(out_dtype) == np.float64
    out = np.empty((B, T, D, D, D), np.float64 if f64 else np.float32)
    rc = lib().orc_forward_index(
        ctypes.c_int(B), ctypes.c_int(N), ctypes.c_int(T), ctypes.c_double(resolution),
        ctypes.c_double(dimension), ctypes.c_double(grm), ctypes.c_double(radius_scale),
        ctypes.c_int(int(radius_type_indexed)), ctypes.c_int(int(coords_as_float)),
        ctypes.c_int(int(box)), _p(coords, _f32p), _p(types, _i32p), _p(radii, _f32p),
        _p(natoms, _i32p), _p(centers, _f32p), _p(quats, _f32p), _p(translations, _f32p),
        _p(None if f64 else out, _f32p), _p(out if f64 else None, _f64p),
        ctypes.c_int(threads))
    if rc < 0:
        raise MemoryError("oracle allocation failed")
    return (out, rc) if return_threads else out


def forward_vector(coords, weights, radii, resolution, dimension, *, grm=1.0,
                   radius_scale=1.0, natoms=None, centers=None, quats=None,
                   translations=None, box=True, coords_as_float=True,
                   out_dtype=np.float32, threads=0, return_threads=False):
    """Real-valued density grid [B,T,D,D,D] for vector-typed atoms (weights [B,N,T])."""
    coords, B, N, natoms, centers, quats, translations = _common(
        coords, natoms, centers, quats, translations)
    weights = _f32(weights)
    T = weights.shape[2]
    assert weights.shape == (B, N, T)
    radii = _f32(radii, (T,))
    D = points_per_side(resolution, dimension)
    f64 = np.dtype(out_dtype) == np.float64
    out = np.empty((B, T, D, D, D), np.float64 if f64 else np.float32)
    rc = lib().orc_forward_vector(
        ctypes.c_int(B), ctypes.c_int(N), ctypes.c_int(T), ctypes.c_double(resolution),
        ctypes.c_double(dimension), ctypes.c_double(grm), ctypes.c_double(radius_scale),
        ctypes.c_int(int(coords_as_float)), ctypes.c_int(int(box)), _p(coords, _f32p),
        _p(weights, _f32p), _p(radii, _f32p), _p(natoms, _i32p), _p(centers, _f32p),
        _p(quats, _f32p), _p(translations, _f32p),
        _p(None if f64 else out, _f32p), _p(out if f64 else None, _f64p),
        ctypes.c_int(threads))
    if rc < 0:
        raise MemoryError("oracle allocation failed")
    return (out, rc) if return_threads else out


def forward_binary(coords, radii, T, resolution, dimension, *, types=None, weights=None,
                   radius_scale=1.0, radius_type_indexed=True, natoms=None, centers=None,
                   quats=None, translations=None, box=True, threads=0):
    """Binary occupancy grid [B,T,D,D,D] float32 in {0,1} (float predicate, fixed order)."""
    coords, B, N, natoms, centers, quats, translations = _common(
        coords, natoms, centers, quats, translations)
    assert (types is None) != (weights is None)
    types = _i32(types, (B, N))
    weights = _f32(weights, (B, N, T)) if weights is not None else None
    radii = _f32(radii, (T,) if (radius_type_indexed or types is None) else (B, N))
    D = points_per_side(resolution, dimension)
    out = np.empty((B, T, D, D, D), np.float32)
    lib().orc_forward_binary(
        ctypes.c_int(B), ctypes.c_int(N), ctypes.c_int(T), ctypes.c_float(resolution),
        ctypes.c_float(dimension), ctypes.c_float(radius_scale),
        ctypes.c_int(int(radius_type_indexed)), ctypes.c_int(int(box)), _p(coords, _f32p),
        _p(types, _i32p), _p(weights, _f32p), _p(radii, _f32p), _p(natoms, _i32p),
        _p(centers, _f32p), _p(quats, _f32p), _p(translations, _f32p), _p(out, _f32p),
        ctypes.c_int(threads))
    return out


def binary_knife_edges(coords, radii, T, resolution, dimension, *, types=None, weights=None,
                       radius_scale=1.0, radius_type_indexed=True, natoms=None, centers=None,
                       quats=None, translations=None, eps=1e-5):
    """uint8 mask [B,T,D,D,D]: voxels where some atom of the channel has |d^2 - r^2| < eps in
    double, i.e. where the float predicate of the binary mode is decided by rounding."""
    coords, B, N, natoms, centers, quats, translations = _common(
        coords, natoms, centers, quats, translations)
    assert (types is None) != (weights is None)
    types = _i32(types, (B, N))
    weights = _f32(weights, (B, N, T)) if weights is not None else None
    radii = _f32(radii, (T,) if (radius_type_indexed or types is None) else (B, N))
    D = points_per_side(resolution, dimension)
    mask = np.empty((B, T, D, D, D), np.uint8)
    lib().orc_binary_knife_edges(
        ctypes.c_int(B), ctypes.c_int(N), ctypes.c_int(T), ctypes.c_float(resolution),
        ctypes.c_float(dimension), ctypes.c_float(radius_scale),
        ctypes.c_int(int(radius_type_indexed)), ctypes.c_double(eps), _p(coords, _f32p),
        _p(types, _i32p), _p(weights, _f32p), _p(radii, _f32p), _p(natoms, _i32p),
        _p(centers, _f32p), _p(quats, _f32p), _p(translations, _f32p),
        mask.ctypes.data_as(ctypes.POINTER(ctypes.c_ubyte)))
    return mask


def _grad_ptrs(grad_out, shape):
    if grad_out.dtype == np.float64:
        G = np.ascontiguousarray(grad_out)
        assert G.shape == shape
        return G, _f32p(), _p(G, _f64p)
    G = _f32(grad_out, shape)
    return G, _p(G, _f32p), _f64p()


def backward_index(coords, types, radii, T, resolution, dimension, grad_out, *, grm=1.0,
                   radius_scale=1.0, radius_type_indexed=True, natoms=None, centers=None,
                   quats=None, translations=None, box=True, coords_as_float=True,
                   threads=0):
    """dL/dcoords [B,N,3] float64 for L = sum(grad_out * forward_index(...))."""
    coords, B, N, natoms, centers, quats, translations = _common(
        coords, natoms, centers, quats, translations)
    types = _i32(types, (B, N))
    radii = _f32(radii, (T,) if radius_type_indexed else (B, N))
    D = points_per_side(resolution, dimension)
    G, g32, g64 = _grad_ptrs(grad_out, (B, T, D, D, D))
    out = np.empty((B, N, 3), np.float64)
    lib().orc_backward_index(
        ctypes.c_int(B), ctypes.c_int(N), ctypes.c_int(T), ctypes.c_double(resolution),
        ctypes.c_double(dimension), ctypes.c_double(grm), ctypes.c_double(radius_scale),
        ctypes.c_int(int(radius_type_indexed)), ctypes.c_int(int(coords_as_float)),
        ctypes.c_int(int(box)), _p(coords, _f32p), _p(types, _i32p), _p(radii, _f32p),
        _p(natoms, _i32p), _p(centers, _f32p), _p(quats, _f32p), _p(translations, _f32p),
        g32, g64, _p(out, _f64p), ctypes.c_int(threads))
    return out


def backward_vector(coords, weights, radii, resolution, dimension, grad_out, *, grm=1.0,
                    radius_scale=1.0, natoms=None, centers=None, quats=None,
                    translations=None, box=True, coords_as_float=True, threads=0):
    """(dL/dcoords [B,N,3], dL/dweights [B,N,T]) float64 for vector-typed atoms."""
    coords, B, N, natoms, centers, quats, translations = _common(
        coords, natoms, centers, quats, translations)
    weights = _f32(weights)
    T = weights.shape[2]
    radii = _f32(radii, (T,))
    D = points_per_side(resolution, dimension)
    G, g32, g64 = _grad_ptrs(grad_out, (B, T, D, D, D))
    gc = np.empty((B, N, 3), np.float64)
    gw = np.empty((B, N, T), np.float64)
    lib().orc_backward_vector(
        ctypes.c_int(B), ctypes.c_int(N), ctypes.c_int(T), ctypes.c_double(resolution),
        ctypes.c_double(dimension), ctypes.c_double(grm), ctypes.c_double(radius_scale),
        ctypes.c_int(int(coords_as_float)), ctypes.c_int(int(box)), _p(coords, _f32p),
        _p(weights, _f32p), _p(radii, _f32p), _p(natoms, _i32p), _p(centers, _f32p),
        _p(quats, _f32p), _p(translations, _f32p), g32, g64, _p(gc, _f64p), _p(gw, _f64p),
        ctypes.c_int(threads))
    return gc, gw


# --------------------------------------------------------------------------
# Subgrid decomposition (the paper: size extensiveness with cubic grids "by performing a
# subgrid decomposition").  Reading: a cube of S*D lattice points per side, spacing
# `resolution`, centred on the example's centre, presented as S^3 grids of D points per
# side; subgrid (sx,sy,sz) holds lattice points [sx*D,(sx+1)*D) x ... .  Written as a
# composition of the functions above: transform once (rotation about the example's centre),
# then one plain forward per subgrid about that subgrid's centre.
# --------------------------------------------------------------------------

def subgrid_centers(centers, S: int, D: int, resolution: float) -> np.ndarray:
    """[B,S,S,S,3] float32 centres: c + ((float)s - (S-1)/2) * ((float)D * res), all in float."""
    c = _f32(centers)
    B = c.shape[0]
    step = np.float32(D) * np.float32(resolution)
    mid = np.float32(0.5) * np.float32(S - 1)
    off = (np.arange(S, dtype=np.float32) - mid) * step              # float product
    out = np.empty((B, S, S, S, 3), np.float32)
    out[..., 0] = c[:, None, None, None, 0] + off[None, :, None, None]
    out[..., 1] = c[:, None, None, None, 1] + off[None, None, :, None]
    out[..., 2] = c[:, None, None, None, 2] + off[None, None, None, :]
    return out


def _virtual(arr, S3):
    return None if arr is None else np.repeat(np.asarray(arr), S3, axis=0)


def forward_subgrids(coords, radii, S, resolution, dimension, *, T=None, types=None, weights=None,
                     binary=False, grm=1.0, radius_scale=1.0, radius_type_indexed=True,
                     natoms=None, centers=None, quats=None, translations=None):
    """[B,S,S,S,T,D,D,D]: every subgrid by the plain forward about its own centre."""
    coords = _f32(coords)
    B, N, _ = coords.shape
    D = points_per_side(resolution, dimension)
    S3 = S ** 3
    cen = _f32(centers, (B, 3)) if centers is not None else np.zeros((B, 3), np.float32)
    moved = transform(coords, centers, quats, translations)          # float, rounded once
    gc = subgrid_centers(cen, S, D, resolution).reshape(B * S3, 3)
    vc, vn = _virtual(moved, S3), _virtual(natoms, S3)
    vr = radii if radius_type_indexed else _virtual(radii, S3)
    if binary:
        out = forward_binary(vc, vr, T, resolution, dimension, types=_virtual(types, S3),
                             weights=_virtual(weights, S3), radius_scale=radius_scale,
                             radius_type_indexed=radius_type_indexed, natoms=vn, centers=gc)
    elif weights is not None:
        out = forward_vector(vc, _virtual(weights, S3), vr, resolution, dimension, grm=grm,
                             radius_scale=radius_scale, natoms=vn, centers=gc)
    else:
        out = forward_index(vc, _virtual(types, S3), vr, T, resolution, dimension, grm=grm,
                            radius_scale=radius_scale, radius_type_indexed=radius_type_indexed,
                            natoms=vn, centers=gc)
    return out.reshape((B, S, S, S) + out.shape[1:])


def backward_subgrids(coords, radii, S, resolution, dimension, grad_out, *, T=None, types=None,
                      weights=None, grm=1.0, radius_scale=1.0, radius_type_indexed=True,
                      natoms=None, centers=None, quats=None, translations=None):
    """dL/dcoords [B,N,3] (and dL/dweights [B,N,T] for vector types), summed over subgrids and
    rotated back to the caller's frame."""
    coords = _f32(coords)
    B, N, _ = coords.shape
    D = points_per_side(resolution, dimension)
    S3 = S ** 3
    cen = _f32(centers, (B, 3)) if centers is not None else np.zeros((B, 3), np.float32)
    moved = transform(coords, centers, quats, translations)
    gc = subgrid_centers(cen, S, D, resolution).reshape(B * S3, 3)
    vc, vn = _virtual(moved, S3), _virtual(natoms, S3)
    vr = radii if radius_type_indexed else _virtual(radii, S3)
    G = np.asarray(grad_out)
    G = G.reshape((B * S3,) + G.shape[4:])
    gw = None
    if weights is not None:
        g, gw = backward_vector(vc, _virtual(weights, S3), vr, resolution, dimension, G, grm=grm,
                                radius_scale=radius_scale, natoms=vn, centers=gc)
        gw = gw.reshape(B, S3, N, -1).sum(1)
    else:
        g = backward_index(vc, _virtual(types, S3), vr, T, resolution, dimension, G, grm=grm,
                           radius_scale=radius_scale, radius_type_indexed=radius_type_indexed,
                           natoms=vn, centers=gc)
    g = g.reshape(B, S3, N, 3).sum(1)                                # in the transformed frame
    out = np.empty_like(g)
    for b in range(B):                                               # back by R^T
        R = quat_to_matrix(quats[b]) if quats is not None else np.eye(3)
        out[b] = g[b] @ R
    return (out, gw) if weights is not None else out
