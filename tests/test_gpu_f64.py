"""Grids of doubles (the paper's grids come in float and double flavours): the f64 entry points
against the oracle's double output, forward (index, vector, binary) and backward."""
import numpy as np
import pytest

import oracle
from paper_1912_04822_amd import workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from test_gpu_parity import GRID_TOL, GRAD_RTOL, dev, mg  # noqa: E402,F401


def poses(w):
    return dict(centers=w.centers, quats=w.quats, translations=w.translations)


def dposes(w):
    return dict(centers=dev(w.centers), quats=dev(w.quats), translations=dev(w.translations))


@pytest.mark.parametrize("make", ["protein", "ragged", "tiny"])
def test_forward_into_a_grid_of_doubles(mg, make):
    """Aligned (D = 48, 24) and unaligned (D = 13) stores; the double grid holds exactly the
    float path's values, so it also equals the float grid widened."""
    w = {"protein": lambda: workloads.protein_ligand(B=2, seed=41, with_weights=True),
         "ragged": workloads.ragged_small, "tiny": workloads.tiny}[make]()
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    args = (dev(w.coords), dev(w.types), dev(w.radii), w.T)
    out64 = gm.mg_forward_index(*args, dtype=torch.float64, **dposes(w))
    assert out64.dtype == torch.float64
    ref = oracle.forward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension,
                               out_dtype=np.float64, **poses(w))
    assert ref.dtype == np.float64
    got = out64.cpu().numpy()
    assert np.abs(got - ref).max() <= GRID_TOL
    out32 = gm.mg_forward_index(*args, **dposes(w)).cpu().numpy()
    assert np.abs(got - out32.astype(np.float64)).max() <= 2e-7 * max(1.0, out32.max())
    # binary: the same 0/1 pattern
    gmb = mg.GridMaker(w.resolution, w.dimension, binary=True, radius_type_indexed=True)
    b64 = gmb.mg_forward_index(*args, dtype=torch.float64, **dposes(w)).cpu().numpy()
    refb = oracle.forward_binary(w.coords, w.radii, w.T, w.resolution, w.dimension, types=w.types,
                                 **poses(w))
    assert np.array_equal(b64, refb.astype(np.float64))
    if w.weights is not None:
        v64 = gm.mg_forward_vector(dev(w.coords), dev(w.weights), dev(w.radii),
                                   dtype=torch.float64, **dposes(w)).cpu().numpy()
        refv = oracle.forward_vector(w.coords, w.weights, w.radii, w.resolution, w.dimension,
                                     **poses(w))
        assert np.abs(v64 - refv).max() <= GRID_TOL


@pytest.mark.parametrize("make", ["protein", "ragged"])
def test_backward_from_a_gradient_grid_of_doubles(mg, make):
    w = {"protein": lambda: workloads.protein_ligand(B=2, seed=42, with_weights=True),
         "ragged": workloads.ragged_small}[make]()
    rng = np.random.default_rng(14)
    G = rng.standard_normal(w.out_shape)                    # float64
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    g = gm.mg_backward_index(dev(w.coords), dev(w.types), dev(w.radii), w.T, dev(G),
                             **dposes(w)).cpu().numpy()
    ref = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension, G,
                                **poses(w))
    for b in range(w.B):
        scale = np.abs(ref[b]).max()
        assert scale == 0 or np.abs(g[b] - ref[b]).max() <= GRAD_RTOL * scale
    gc, gw = gm.mg_backward_vector(dev(w.coords), dev(w.weights), dev(w.radii), dev(G), **dposes(w))
    rc, rw = oracle.backward_vector(w.coords, w.weights, w.radii, w.resolution, w.dimension, G,
                                    **poses(w))
    gc, gw = gc.cpu().numpy(), gw.cpu().numpy()
    for b in range(w.B):
        if np.abs(rc[b]).max() > 0:
            assert np.abs(gc[b] - rc[b]).max() <= GRAD_RTOL * np.abs(rc[b]).max()
            assert np.abs(gw[b] - rw[b]).max() <= GRAD_RTOL * np.abs(rw[b]).max()


def test_double_grid_must_be_8_byte_aligned(mg):
    w = workloads.tiny()
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    import ctypes
    # a float-aligned but not double-aligned address, handed over as raw storage
    buf = torch.empty(int(np.prod(w.out_shape)) * 2 + 1, dtype=torch.float32, device="cuda")
    L = mg.lib()
    ws = torch.empty(gm.workspace_bytes(w.B, w.N, w.T), dtype=torch.uint8, device="cuda")
    rc = L.mg_forward_index_f64(gm._h, w.B, w.N, w.T, ctypes.c_void_p(dev(w.coords).data_ptr()),
                                ctypes.c_void_p(dev(w.types).data_ptr()),
                                ctypes.c_void_p(dev(w.radii).data_ptr()), None, None, None, None,
                                ctypes.c_void_p(buf.data_ptr() + 4), ctypes.c_void_p(ws.data_ptr()),
                                ws.numel(), None)
    assert rc == -7
