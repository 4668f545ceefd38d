"""Parity of a GridMaker with a subgrid decomposition with the oracle: forward (index, vector,
binary: bit-exact) and backward (coordinates, type weights), through the C ABI."""
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


@pytest.mark.parametrize("S", [2, 3])
def test_forward_index_subgrids_small_ragged(mg, S):
    w = workloads.ragged_small()
    nat = w.extra["natoms"]
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True, subgrids_per_side=S)
    assert gm.S == S
    out = gm.mg_forward_index(dev(w.coords), dev(w.types), dev(w.radii), w.T, natoms=dev(nat),
                              **dposes(w)).cpu().numpy()
    ref = oracle.forward_subgrids(w.coords, w.radii, S, w.resolution, w.dimension, T=w.T,
                                  types=w.types, natoms=nat, **poses(w))
    assert out.shape == ref.shape == (w.B, S, S, S, w.T, w.D, w.D, w.D)
    assert np.abs(out - ref).max() <= GRID_TOL
    assert ref.max() > 0.5


def test_sixteen_subgrids_per_side(mg):
    """The largest decomposition the ABI takes: 16^3 = 4096 subgrids per example (3 points per
    side each, a 48^3 lattice in all), forward and backward."""
    S, D, res = 16, 3, 0.5
    w = workloads.ragged_small(seed=17, B=2, N=300, T=3, D=D, resolution=res)
    rng = np.random.default_rng(18)
    w.coords[:] = (w.centers[:, None, :] + rng.uniform(-12.5, 12.5, w.coords.shape)).astype(np.float32)
    gm = mg.GridMaker(res, w.dimension, radius_type_indexed=True, subgrids_per_side=S)
    out = gm.mg_forward_index(dev(w.coords), dev(w.types), dev(w.radii), w.T, **dposes(w)).cpu().numpy()
    ref = oracle.forward_subgrids(w.coords, w.radii, S, res, w.dimension, T=w.T, types=w.types,
                                  **poses(w))
    assert out.shape == ref.shape == (2, S, S, S, w.T, D, D, D)
    assert np.abs(out - ref).max() <= GRID_TOL
    assert (ref.reshape(2, S ** 3, -1).max(axis=2) > 0).mean() > 0.5       # most subgrids hold density
    G = rng.standard_normal(ref.shape).astype(np.float32)
    g = gm.mg_backward_index(dev(w.coords), dev(w.types), dev(w.radii), w.T, dev(G),
                             **dposes(w)).cpu().numpy()
    rg = oracle.backward_subgrids(w.coords, w.radii, S, res, w.dimension, G, T=w.T, types=w.types,
                                  **poses(w))
    for b in range(2):
        assert np.abs(g[b] - rg[b]).max() <= GRAD_RTOL * np.abs(rg[b]).max()


def test_forward_subgrids_protein_ligand_real_binary_vector(mg):
    """Two examples of the protein-ligand recipe in 2^3 subgrids of 24^3 points each (the 48^3
    region of the plain GridMaker cut in eight)."""
    w = workloads.protein_ligand(B=2, seed=91, with_weights=True)
    S, dim = 2, 11.5
    args = (dev(w.coords), dev(w.types), dev(w.radii), w.T)
    gm = mg.GridMaker(w.resolution, dim, radius_type_indexed=True, subgrids_per_side=S)
    out = gm.mg_forward_index(*args, **dposes(w)).cpu().numpy()
    ref = oracle.forward_subgrids(w.coords, w.radii, S, w.resolution, dim, T=w.T, types=w.types,
                                  **poses(w))
    assert out.shape == (2, 2, 2, 2, w.T, 24, 24, 24)
    assert np.abs(out - ref).max() <= GRID_TOL
    # the same region from the plain GridMaker, cut into blocks
    plain = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    big = plain.mg_forward_index(*args, **dposes(w)).cpu().numpy()
    blocks = big.reshape(2, w.T, 2, 24, 2, 24, 2, 24).transpose(0, 2, 4, 6, 1, 3, 5, 7)
    assert np.abs(blocks - out).max() <= 2 * GRID_TOL
    # binary: bit-exact
    gmb = mg.GridMaker(w.resolution, dim, binary=True, radius_type_indexed=True,
                       subgrids_per_side=S)
    outb = gmb.mg_forward_index(*args, **dposes(w)).cpu().numpy()
    refb = oracle.forward_subgrids(w.coords, w.radii, S, w.resolution, dim, T=w.T, types=w.types,
                                   binary=True, **poses(w))
    assert np.array_equal(outb.view(np.uint32), refb.view(np.uint32))
    assert refb.sum() > 1000
    # vector types
    outv = gm.mg_forward_vector(dev(w.coords), dev(w.weights), dev(w.radii),
                                **dposes(w)).cpu().numpy()
    refv = oracle.forward_subgrids(w.coords, w.radii, S, w.resolution, dim, weights=w.weights,
                                   **poses(w))
    assert np.abs(outv - refv).max() <= GRID_TOL


def test_backward_subgrids_index_and_vector(mg):
    w = workloads.protein_ligand(B=2, seed=92, with_weights=True)
    S, dim = 2, 11.5
    rng = np.random.default_rng(13)
    G = rng.standard_normal((2, S, S, S, w.T, 24, 24, 24)).astype(np.float32)
    gm = mg.GridMaker(w.resolution, dim, radius_type_indexed=True, subgrids_per_side=S)
    g = gm.mg_backward_index(dev(w.coords), dev(w.types), dev(w.radii), w.T, dev(G),
                             **dposes(w)).cpu().numpy()
    ref = oracle.backward_subgrids(w.coords, w.radii, S, w.resolution, dim, G, T=w.T,
                                   types=w.types, **poses(w))
    for b in range(w.B):
        assert np.abs(g[b] - ref[b]).max() <= GRAD_RTOL * np.abs(ref[b]).max()
    # a second call into the same (dirty) workspace gives the same bits
    g2 = gm.mg_backward_index(dev(w.coords), dev(w.types), dev(w.radii), w.T, dev(G),
                              **dposes(w)).cpu().numpy()
    assert np.array_equal(g, g2)
    gc, gw = gm.mg_backward_vector(dev(w.coords), dev(w.weights), dev(w.radii), dev(G), **dposes(w))
    rc, rw = oracle.backward_subgrids(w.coords, w.radii, S, w.resolution, dim, G,
                                      weights=w.weights, **poses(w))
    gc, gw = gc.cpu().numpy(), gw.cpu().numpy()
    for b in range(w.B):
        assert np.abs(gc[b] - rc[b]).max() <= GRAD_RTOL * np.abs(rc[b]).max()
        assert np.abs(gw[b] - rw[b]).max() <= GRAD_RTOL * np.abs(rw[b]).max()
    # only the weights
    _, gw2 = gm.mg_backward_vector(dev(w.coords), dev(w.weights), dev(w.radii), dev(G),
                                   want_coords=False, **dposes(w))
    assert np.array_equal(gw2.cpu().numpy(), gw)


def test_subgrid_gridmaker_rejects_bad_counts(mg):
    for S in (0, -1, 17):
        with pytest.raises(mg.MolgridError):
            mg.GridMaker(0.5, 11.5, subgrids_per_side=S)
    gm = mg.GridMaker(0.5, 11.5, radius_type_indexed=True, subgrids_per_side=16)
    with pytest.raises(mg.MolgridError):
        gm.workspace_bytes(16, 10, 4)          # 16 * 4096 virtual examples > 65535


@pytest.mark.parametrize("N,single_type", [(9000, False), (9000, True)])
def test_subgrids_with_the_per_group_prep_kernel_and_per_atom_radii(mg, N, single_type):
    """N = 9000 takes the slower prep kernel (one wavefront per example and type; with a single
    type the group is not binned at all); radii given per atom; natoms ragged."""
    w = workloads.ragged_small(seed=12, B=2, N=N, T=3, D=8, resolution=0.5)
    if single_type:
        w.types[:] = 2
    S = 2
    nat = np.array([N, N - 411], np.int32)
    per_atom = w.radii[np.clip(w.types, 0, w.T - 1)]
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=False, subgrids_per_side=S)
    out = gm.mg_forward_index(dev(w.coords), dev(w.types), dev(per_atom), w.T, natoms=dev(nat),
                              **dposes(w)).cpu().numpy()
    ref = oracle.forward_subgrids(w.coords, per_atom, S, w.resolution, w.dimension, T=w.T,
                                  types=w.types, natoms=nat, radius_type_indexed=False, **poses(w))
    assert np.abs(out - ref).max() <= GRID_TOL + 2e-6 * ref.max()
    gmb = mg.GridMaker(w.resolution, w.dimension, binary=True, radius_type_indexed=False,
                       subgrids_per_side=S)
    outb = gmb.mg_forward_index(dev(w.coords), dev(w.types), dev(per_atom), w.T, natoms=dev(nat),
                                **dposes(w)).cpu().numpy()
    refb = oracle.forward_subgrids(w.coords, per_atom, S, w.resolution, w.dimension, T=w.T,
                                   types=w.types, natoms=nat, binary=True,
                                   radius_type_indexed=False, **poses(w))
    assert np.array_equal(outb.view(np.uint32), refb.view(np.uint32))
    rng = np.random.default_rng(3)
    G = rng.standard_normal(ref.shape).astype(np.float32)
    g = gm.mg_backward_index(dev(w.coords), dev(w.types), dev(per_atom), w.T, dev(G),
                             natoms=dev(nat), **dposes(w)).cpu().numpy()
    rg = oracle.backward_subgrids(w.coords, per_atom, S, w.resolution, w.dimension, G, T=w.T,
                                  types=w.types, natoms=nat, radius_type_indexed=False, **poses(w))
    for b in range(w.B):
        assert np.abs(g[b] - rg[b]).max() <= GRAD_RTOL * np.abs(rg[b]).max()
