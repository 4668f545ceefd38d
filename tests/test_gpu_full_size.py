"""Parity at the full benchmark sizes, in the launch configuration bench.py times.

The oracle's cutoff-box variant finishes each of these in seconds, so every output
element is compared (not a sample): protein-ligand forward (B=50), its binary mode, its
backward, the vector-typed forward, and two 16-example chunks of the high-resolution case.
"""
import numpy as np
import pytest

import oracle
from paper_1912_04822_amd import workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

GRID_TOL = 1e-5
GRAD_RTOL = 1e-4


@pytest.fixture(scope="module")
def mg():
    from paper_1912_04822_amd import molgrid
    molgrid.lib()
    return molgrid


@pytest.fixture(scope="module")
def c1():
    return workloads.protein_ligand(B=50, with_grad=True, with_weights=True)


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def okw(w):
    return dict(centers=w.centers, quats=w.quats, translations=w.translations)


def dkw(w):
    return dict(centers=dev(w.centers), quats=dev(w.quats), translations=dev(w.translations))


def test_protein_ligand_forward_full(mg, c1):
    w = c1
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    out = gm.mg_forward_index(dev(w.coords), dev(w.types), dev(w.radii), w.T, **dkw(w))
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    del out
    ref = oracle.forward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension, **okw(w))
    assert got.shape == (50, 28, 48, 48, 48)
    err = float(np.abs(got - ref).max())
    assert err <= GRID_TOL, err
    # what is zero in the oracle is exactly zero here (and nothing was left unwritten)
    assert np.isfinite(got).all()
    assert (got[ref == 0] == 0).all()
    frac = float((got != 0).mean())
    assert 0.05 < frac < 0.3


def test_protein_ligand_binary_full_bit_exact(mg, c1):
    w = c1
    gm = mg.GridMaker(w.resolution, w.dimension, binary=True, radius_type_indexed=True)
    out = gm.mg_forward_index(dev(w.coords), dev(w.types), dev(w.radii), w.T, **dkw(w))
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    del out
    ref = oracle.forward_binary(w.coords, w.radii, w.T, w.resolution, w.dimension, types=w.types,
                                **okw(w))
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    # voxels where the double-precision distance is within 1e-5 of r^2 ("knife edges"): count them
    assert got.sum() > 1e5


def test_protein_ligand_backward_full(mg, c1):
    w = c1
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    g = gm.mg_backward_index(dev(w.coords), dev(w.types), dev(w.radii), w.T, dev(w.grad_out),
                             **dkw(w))
    torch.cuda.synchronize()
    got = g.cpu().numpy()
    ref = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension,
                                w.grad_out, **okw(w))
    assert got.shape == (50, 2040, 3)
    for b in range(w.B):
        scale = np.abs(ref[b]).max()
        assert np.abs(got[b] - ref[b]).max() <= GRAD_RTOL * scale
    assert ((ref == 0) == (got == 0)).all()


def test_protein_ligand_vector_forward_full(mg, c1):
    w = c1
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    out = gm.mg_forward_vector(dev(w.coords), dev(w.weights), dev(w.radii), **dkw(w))
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    del out
    ref = oracle.forward_vector(w.coords, w.weights, w.radii, w.resolution, w.dimension, **okw(w))
    err = float(np.abs(got - ref).max())
    assert err <= GRID_TOL, err
    assert got.min() >= 0.0


@pytest.mark.parametrize("chunk", [0, 5])
def test_high_resolution_chunk(mg, chunk):
    """B=128 is produced in chunks of 16 examples; each chunk is one call."""
    w = workloads.large_chunk(chunk)
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    assert gm.D == 96
    out = gm.mg_forward_index(dev(w.coords), dev(w.types), dev(w.radii), w.T, **dkw(w))
    torch.cuda.synchronize()
    ref = oracle.forward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension, **okw(w))
    worst = 0.0
    for b in range(w.B):                    # compare example by example: bounded host memory
        got = out[b].cpu().numpy()
        worst = max(worst, float(np.abs(got - ref[b]).max()))
        assert (got[ref[b] == 0] == 0).all()
    assert worst <= GRID_TOL, worst
