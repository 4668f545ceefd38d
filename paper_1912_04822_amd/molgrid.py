"""Thin ctypes binding over the C-ABI HIP library (``include/molgrid_hip.h``).

Argument marshalling only: every step of the path runs in the library's
kernels.  PyTorch supplies device memory and the stream.  There is no CPU
fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmolgrid_hip.so")

MG_OK = 0
EXPORTS = [
    "mg_gridmaker_create", "mg_gridmaker_create_subgrids", "mg_gridmaker_subgrids_per_side",
    "mg_gridmaker_destroy", "mg_gridmaker_points_per_side",
    "mg_workspace_bytes", "mg_transform_forward", "mg_transform_backward", "mg_draw_transforms",
    "mg_forward_index", "mg_forward_index_static", "mg_forward_vector", "mg_forward_index_f64", "mg_forward_vector_f64",
    "mg_backward_index_f64", "mg_backward_vector_f64",
    "mg_backward_index", "mg_backward_vector", "mg_strerror", "mg_last_hip_error",
    "mg_prepare", "mg_forward_index_prepared", "mg_forward_vector_prepared",
    "mg_backward_index_prepared", "mg_backward_vector_prepared",
    "mg_set_option", "mg_time_next_kernel",
]

_lib: Optional[ctypes.CDLL] = None


class MolgridError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (code %d)" % (where, strerror(code), code))


def lib(path: Optional[str] = None) -> ctypes.CDLL:
    """Load libmolgrid_hip.so (built by ``paper_1912_04822_amd.build``); raise if absent.
    ``path`` (first call only) names another build of the same library, e.g. the measurement
    build with the timing aids."""
    global _lib
    if _lib is None:
        path = path or LIB_PATH
        if not os.path.exists(path):
            raise FileNotFoundError(
                "HIP library not built: %s (run python -m paper_1912_04822_amd.build)" % path)
        L = ctypes.CDLL(path)
        vp, ci, cf, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        L.mg_gridmaker_create.restype = ci
        L.mg_gridmaker_create.argtypes = [ctypes.POINTER(vp), cf, cf, ci, ci, cf, cf]
        L.mg_gridmaker_create_subgrids.restype = ci
        L.mg_gridmaker_create_subgrids.argtypes = [ctypes.POINTER(vp), cf, cf, ci, ci, ci, cf, cf]
        L.mg_gridmaker_subgrids_per_side.restype = ci
        L.mg_gridmaker_subgrids_per_side.argtypes = [vp, ctypes.POINTER(ci)]
        L.mg_gridmaker_destroy.restype = None
        L.mg_gridmaker_destroy.argtypes = [vp]
        L.mg_gridmaker_points_per_side.restype = ci
        L.mg_gridmaker_points_per_side.argtypes = [vp, ctypes.POINTER(ci)]
        L.mg_workspace_bytes.restype = ci
        L.mg_workspace_bytes.argtypes = [vp, ci, ci, ci, ctypes.POINTER(sz)]
        L.mg_transform_forward.restype = ci
        L.mg_transform_forward.argtypes = [ci, ci, vp, vp, vp, vp, vp, vp]
        L.mg_transform_backward.restype = ci
        L.mg_transform_backward.argtypes = [ci, ci, vp, vp, vp, vp, vp, vp]
        L.mg_draw_transforms.restype = ci
        L.mg_draw_transforms.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ci, ci, cf, vp, vp, vp]
        L.mg_forward_index.restype = ci
        L.mg_forward_index.argtypes = [vp, ci, ci, ci] + [vp] * 8 + [vp, sz, vp]
        L.mg_forward_index_static.restype = ci
        L.mg_forward_index_static.argtypes = [vp, ci, ci, ci] + [vp] * 8 + [vp]
        L.mg_forward_vector.restype = ci
        L.mg_forward_vector.argtypes = [vp, ci, ci, ci] + [vp] * 8 + [vp, sz, vp]
        for name, src in (("mg_forward_index_f64", "mg_forward_index"),
                          ("mg_forward_vector_f64", "mg_forward_vector")):
            getattr(L, name).restype = ci
            getattr(L, name).argtypes = [vp, ci, ci, ci] + [vp] * 8 + [vp, sz, vp]
        L.mg_backward_index_f64.restype = ci
        L.mg_backward_index_f64.argtypes = [vp, ci, ci, ci] + [vp] * 9 + [vp, sz, vp]
        L.mg_backward_vector_f64.restype = ci
        L.mg_backward_vector_f64.argtypes = [vp, ci, ci, ci] + [vp] * 10 + [vp, sz, vp]
        L.mg_backward_index.restype = ci
        L.mg_backward_index.argtypes = [vp, ci, ci, ci] + [vp] * 9 + [vp, sz, vp]
        L.mg_backward_vector.restype = ci
        L.mg_backward_vector.argtypes = [vp, ci, ci, ci] + [vp] * 10 + [vp, sz, vp]
        L.mg_prepare.restype = ci
        L.mg_prepare.argtypes = [vp, ci, ci, ci] + [vp] * 7 + [vp, sz, vp]
        L.mg_forward_index_prepared.restype = ci
        L.mg_forward_index_prepared.argtypes = [vp, ci, ci, ci, vp, vp, sz, vp]
        L.mg_forward_vector_prepared.restype = ci
        L.mg_forward_vector_prepared.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp, sz, vp]
        L.mg_backward_index_prepared.restype = ci
        L.mg_backward_index_prepared.argtypes = [vp, ci, ci, ci, vp, vp, vp, sz, vp]
        L.mg_backward_vector_prepared.restype = ci
        L.mg_backward_vector_prepared.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp, vp, vp, sz, vp]
        L.mg_strerror.restype = ctypes.c_char_p
        L.mg_strerror.argtypes = [ci]
        L.mg_last_hip_error.restype = ci
        L.mg_last_hip_error.argtypes = []
        L.mg_set_option.restype = ci
        L.mg_set_option.argtypes = [ctypes.c_char_p, ci]
        L.mg_time_next_kernel.restype = ci
        L.mg_time_next_kernel.argtypes = [vp, vp]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().mg_strerror(int(code)).decode()


def set_option(key: str, value: int) -> None:
    rc = lib().mg_set_option(key.encode(), int(value))
    if rc != MG_OK:
        raise MolgridError(rc, "mg_set_option")


def mg_time_next_kernel(start_event: Optional[int], stop_event: Optional[int]) -> None:
    """Have the next forward/backward call record these hipEvent_t handles around its main kernel."""
    lib().mg_time_next_kernel(ctypes.c_void_p(start_event), ctypes.c_void_p(stop_event))


def _ptr(t: Optional[torch.Tensor], dtype, name: str, shape=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must be a device tensor" % name)
    if t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def mg_transform_forward(coords, centers=None, quats=None, translations=None, out=None):
    """x' = R(q)(x - c) + c + t per example; [B,N,3] float32 device tensors."""
    B, N, _ = coords.shape
    if out is None:
        out = torch.empty_like(coords)
    rc = lib().mg_transform_forward(
        B, N, _ptr(coords, torch.float32, "coords", (B, N, 3)),
        _ptr(centers, torch.float32, "centers", (B, 3)), _ptr(quats, torch.float32, "quats", (B, 4)),
        _ptr(translations, torch.float32, "translations", (B, 3)),
        _ptr(out, torch.float32, "out", (B, N, 3)), _stream())
    if rc != MG_OK:
        raise MolgridError(rc, "mg_transform_forward")
    return out


def mg_transform_backward(coords, centers=None, quats=None, translations=None, out=None):
    """x = R(q)^T ((x' - t) - c) + c per example; [B,N,3] float32 device tensors."""
    B, N, _ = coords.shape
    if out is None:
        out = torch.empty_like(coords)
    rc = lib().mg_transform_backward(
        B, N, _ptr(coords, torch.float32, "coords", (B, N, 3)),
        _ptr(centers, torch.float32, "centers", (B, 3)), _ptr(quats, torch.float32, "quats", (B, 4)),
        _ptr(translations, torch.float32, "translations", (B, 3)),
        _ptr(out, torch.float32, "out", (B, N, 3)), _stream())
    if rc != MG_OK:
        raise MolgridError(rc, "mg_transform_backward")
    return out


def mg_draw_transforms(seed: int, draw: int, B: int, random_rotation: bool = True,
                       max_translation: float = 0.0, quats=None, translations=None, device=None):
    """Per-example random quaternions [B,4] and translations [B,3] drawn on the device."""
    if quats is None:
        quats = torch.empty((B, 4), dtype=torch.float32, device=device or "cuda")
    if translations is None:
        translations = torch.empty((B, 3), dtype=torch.float32, device=quats.device)
    rc = lib().mg_draw_transforms(
        int(seed) & (2 ** 64 - 1), int(draw) & (2 ** 64 - 1), B, 1 if random_rotation else 0,
        float(max_translation), _ptr(quats, torch.float32, "quats", (B, 4)),
        _ptr(translations, torch.float32, "translations", (B, 3)), _stream())
    if rc != MG_OK:
        raise MolgridError(rc, "mg_draw_transforms")
    return quats, translations


class GridMaker:
    """Handle over ``mg_gridmaker`` (GridMaker constructor listing of the paper)."""

    def __init__(self, resolution=0.5, dimension=23.5, binary=False, radius_type_indexed=False,
                 radius_scale=1.0, gaussian_radius_multiple=1.0, subgrids_per_side=1):
        self._h = ctypes.c_void_p()
        if subgrids_per_side == 1:
            rc = lib().mg_gridmaker_create(ctypes.byref(self._h), resolution, dimension,
                                           int(binary), int(radius_type_indexed), radius_scale,
                                           gaussian_radius_multiple)
        else:
            rc = lib().mg_gridmaker_create_subgrids(
                ctypes.byref(self._h), resolution, dimension, int(subgrids_per_side), int(binary),
                int(radius_type_indexed), radius_scale, gaussian_radius_multiple)
        if rc != MG_OK:
            self._h = ctypes.c_void_p()
            raise MolgridError(rc, "mg_gridmaker_create")
        sps = ctypes.c_int()
        lib().mg_gridmaker_subgrids_per_side(self._h, ctypes.byref(sps))
        self.S = sps.value
        d = ctypes.c_int()
        lib().mg_gridmaker_points_per_side(self._h, ctypes.byref(d))
        self.D = d.value
        self.binary = bool(binary)
        self.radius_type_indexed = bool(radius_type_indexed)
        # workspaces the binding allocated, one per (device, stream): calls on different
        # streams may run at the same time and must not share tables
        self._ws = {}

    def __del__(self):
        h = getattr(self, "_h", None)
        if h is not None and h.value and _lib is not None:
            _lib.mg_gridmaker_destroy(h)
            self._h = ctypes.c_void_p()

    def workspace_bytes(self, B: int, N: int, T: int) -> int:
        n = ctypes.c_size_t()
        rc = lib().mg_workspace_bytes(self._h, B, N, T, ctypes.byref(n))
        if rc != MG_OK:
            raise MolgridError(rc, "mg_workspace_bytes")
        return n.value

    def grid_shape(self, B: int, T: int):
        """[B,T,D,D,D], or [B,S,S,S,T,D,D,D] for a GridMaker with S > 1 subgrids per side."""
        D, S = self.D, self.S
        return (B, T, D, D, D) if S == 1 else (B, S, S, S, T, D, D, D)

    def _workspace(self, B, N, T, device, workspace):
        need = self.workspace_bytes(B, N, T)
        if workspace is not None:
            return workspace, workspace.numel() * workspace.element_size()
        key = (str(device), torch.cuda.current_stream().cuda_stream)    # the stream the call uses
        ws = self._ws.get(key)
        if ws is None or ws.numel() < need:
            ws = torch.empty(need, dtype=torch.uint8, device=device)
            self._ws[key] = ws
        return ws, ws.numel()

    def _common(self, coords, natoms, centers, quats, translations):
        B, N, _ = coords.shape
        return (B, N, _ptr(coords, torch.float32, "coords", (B, N, 3)),
                _ptr(natoms, torch.int32, "natoms", (B,)),
                _ptr(centers, torch.float32, "centers", (B, 3)),
                _ptr(quats, torch.float32, "quats", (B, 4)),
                _ptr(translations, torch.float32, "translations", (B, 3)))

    def mg_forward_index(self, coords, types, radii, T, natoms=None, centers=None, quats=None,
                         translations=None, out=None, workspace=None, dtype=torch.float32):
        """``dtype`` (or ``out.dtype``) torch.float64 calls ``mg_forward_index_f64``."""
        B, N, pc, pn, pce, pq, pt = self._common(coords, natoms, centers, quats, translations)
        D = self.D
        if out is None:
            out = torch.empty(self.grid_shape(B, T), dtype=dtype, device=coords.device)
        ws, wsb = self._workspace(B, N, T, coords.device, workspace)
        rshape = (T,) if self.radius_type_indexed else (B, N)
        fn = lib().mg_forward_index_f64 if out.dtype == torch.float64 else lib().mg_forward_index
        rc = fn(
            self._h, B, N, T, pc, _ptr(types, torch.int32, "types", (B, N)),
            _ptr(radii, torch.float32, "radii", rshape), pn, pce, pq, pt,
            _ptr(out, out.dtype, "out", self.grid_shape(B, T)), ctypes.c_void_p(ws.data_ptr()), wsb,
            _stream())
        if rc != MG_OK:
            raise MolgridError(rc, "mg_forward_index")
        return out

    def mg_forward_index_static(self, coords, types, radii, T, out, natoms=None, centers=None,
                                quats=None, translations=None):
        """``mg_forward_index`` with the workspace in the library's static device array: the
        call allocates nothing, so ``out`` is required."""
        B, N, pc, pn, pce, pq, pt = self._common(coords, natoms, centers, quats, translations)
        rshape = (T,) if self.radius_type_indexed else (B, N)
        rc = lib().mg_forward_index_static(
            self._h, B, N, T, pc, _ptr(types, torch.int32, "types", (B, N)),
            _ptr(radii, torch.float32, "radii", rshape), pn, pce, pq, pt,
            _ptr(out, torch.float32, "out", self.grid_shape(B, T)), _stream())
        if rc != MG_OK:
            raise MolgridError(rc, "mg_forward_index_static")
        return out

    def mg_forward_vector(self, coords, weights, radii, natoms=None, centers=None, quats=None,
                          translations=None, out=None, workspace=None, dtype=torch.float32):
        B, N, pc, pn, pce, pq, pt = self._common(coords, natoms, centers, quats, translations)
        T = weights.shape[2]
        D = self.D
        if out is None:
            out = torch.empty(self.grid_shape(B, T), dtype=dtype, device=coords.device)
        ws, wsb = self._workspace(B, N, T, coords.device, workspace)
        fn = lib().mg_forward_vector_f64 if out.dtype == torch.float64 else lib().mg_forward_vector
        rc = fn(
            self._h, B, N, T, pc, _ptr(weights, torch.float32, "weights", (B, N, T)),
            _ptr(radii, torch.float32, "radii", (T,)), pn, pce, pq, pt,
            _ptr(out, out.dtype, "out", self.grid_shape(B, T)), ctypes.c_void_p(ws.data_ptr()), wsb,
            _stream())
        if rc != MG_OK:
            raise MolgridError(rc, "mg_forward_vector")
        return out

    def mg_backward_index(self, coords, types, radii, T, grad_out, natoms=None, centers=None,
                          quats=None, translations=None, grad_coords=None, workspace=None):
        B, N, pc, pn, pce, pq, pt = self._common(coords, natoms, centers, quats, translations)
        D = self.D
        if grad_coords is None:
            grad_coords = torch.empty((B, N, 3), dtype=torch.float32, device=coords.device)
        ws, wsb = self._workspace(B, N, T, coords.device, workspace)
        rshape = (T,) if self.radius_type_indexed else (B, N)
        fn = (lib().mg_backward_index_f64 if grad_out.dtype == torch.float64
              else lib().mg_backward_index)
        rc = fn(
            self._h, B, N, T, pc, _ptr(types, torch.int32, "types", (B, N)),
            _ptr(radii, torch.float32, "radii", rshape), pn, pce, pq, pt,
            _ptr(grad_out, grad_out.dtype, "grad_out", self.grid_shape(B, T)),
            _ptr(grad_coords, torch.float32, "grad_coords", (B, N, 3)),
            ctypes.c_void_p(ws.data_ptr()), wsb, _stream())
        if rc != MG_OK:
            raise MolgridError(rc, "mg_backward_index")
        return grad_coords

    def mg_backward_vector(self, coords, weights, radii, grad_out, natoms=None, centers=None,
                           quats=None, translations=None, grad_coords=None, grad_weights=None,
                           want_coords=True, want_weights=True, workspace=None):
        B, N, pc, pn, pce, pq, pt = self._common(coords, natoms, centers, quats, translations)
        T = weights.shape[2]
        D = self.D
        if grad_coords is None and want_coords:
            grad_coords = torch.empty((B, N, 3), dtype=torch.float32, device=coords.device)
        if grad_weights is None and want_weights:
            grad_weights = torch.empty((B, N, T), dtype=torch.float32, device=coords.device)
        ws, wsb = self._workspace(B, N, T, coords.device, workspace)
        fn = (lib().mg_backward_vector_f64 if grad_out.dtype == torch.float64
              else lib().mg_backward_vector)
        rc = fn(
            self._h, B, N, T, pc, _ptr(weights, torch.float32, "weights", (B, N, T)),
            _ptr(radii, torch.float32, "radii", (T,)), pn, pce, pq, pt,
            _ptr(grad_out, grad_out.dtype, "grad_out", self.grid_shape(B, T)),
            _ptr(grad_coords, torch.float32, "grad_coords", (B, N, 3)),
            _ptr(grad_weights, torch.float32, "grad_weights", (B, N, T)),
            ctypes.c_void_p(ws.data_ptr()), wsb, _stream())
        if rc != MG_OK:
            raise MolgridError(rc, "mg_backward_vector")
        return grad_coords, grad_weights

    # ---- tables once, calls many (mg_prepare + the *_prepared calls) ----

    def mg_prepare(self, coords, types, radii, T, natoms=None, centers=None, quats=None,
                   translations=None, workspace=None):
        """Build the workspace's tables for these atoms and poses (``types=None``: the tables
        of vector types) and return the workspace tensor the ``*_prepared`` calls then take."""
        B, N, pc, pn, pce, pq, pt = self._common(coords, natoms, centers, quats, translations)
        if workspace is None:
            workspace = torch.empty(self.workspace_bytes(B, N, T), dtype=torch.uint8,
                                    device=coords.device)
        rshape = (T,) if (self.radius_type_indexed or types is None) else (B, N)
        rc = lib().mg_prepare(
            self._h, B, N, T, pc, _ptr(types, torch.int32, "types", (B, N)),
            _ptr(radii, torch.float32, "radii", rshape), pn, pce, pq, pt,
            ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
            _stream())
        if rc != MG_OK:
            raise MolgridError(rc, "mg_prepare")
        return workspace

    def mg_forward_index_prepared(self, B, N, T, workspace, out=None):
        if out is None:
            out = torch.empty(self.grid_shape(B, T), dtype=torch.float32, device=workspace.device)
        rc = lib().mg_forward_index_prepared(
            self._h, B, N, T, _ptr(out, torch.float32, "out", self.grid_shape(B, T)),
            ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
            _stream())
        if rc != MG_OK:
            raise MolgridError(rc, "mg_forward_index_prepared")
        return out

    def mg_forward_vector_prepared(self, weights, radii, workspace, out=None):
        B, N, T = weights.shape
        if out is None:
            out = torch.empty(self.grid_shape(B, T), dtype=torch.float32, device=weights.device)
        rc = lib().mg_forward_vector_prepared(
            self._h, B, N, T, _ptr(weights, torch.float32, "weights", (B, N, T)),
            _ptr(radii, torch.float32, "radii", (T,)),
            _ptr(out, torch.float32, "out", self.grid_shape(B, T)),
            ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
            _stream())
        if rc != MG_OK:
            raise MolgridError(rc, "mg_forward_vector_prepared")
        return out

    def mg_backward_index_prepared(self, B, N, T, grad_out, workspace, grad_coords=None):
        if grad_coords is None:
            grad_coords = torch.empty((B, N, 3), dtype=torch.float32, device=grad_out.device)
        rc = lib().mg_backward_index_prepared(
            self._h, B, N, T,
            _ptr(grad_out, torch.float32, "grad_out", self.grid_shape(B, T)),
            _ptr(grad_coords, torch.float32, "grad_coords", (B, N, 3)),
            ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
            _stream())
        if rc != MG_OK:
            raise MolgridError(rc, "mg_backward_index_prepared")
        return grad_coords

    def mg_backward_vector_prepared(self, weights, radii, grad_out, workspace, grad_coords=None,
                                    grad_weights=None, want_coords=True, want_weights=True):
        B, N, T = weights.shape
        if grad_coords is None and want_coords:
            grad_coords = torch.empty((B, N, 3), dtype=torch.float32, device=weights.device)
        if grad_weights is None and want_weights:
            grad_weights = torch.empty((B, N, T), dtype=torch.float32, device=weights.device)
        rc = lib().mg_backward_vector_prepared(
            self._h, B, N, T, _ptr(weights, torch.float32, "weights", (B, N, T)),
            _ptr(radii, torch.float32, "radii", (T,)),
            _ptr(grad_out, torch.float32, "grad_out", self.grid_shape(B, T)),
            _ptr(grad_coords, torch.float32, "grad_coords", (B, N, 3)),
            _ptr(grad_weights, torch.float32, "grad_weights", (B, N, T)),
            ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
            _stream())
        if rc != MG_OK:
            raise MolgridError(rc, "mg_backward_vector_prepared")
        return grad_coords, grad_weights
