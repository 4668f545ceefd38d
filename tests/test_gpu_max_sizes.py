"""The largest shapes the ABI accepts: 1024 points per side (2^30 voxels per channel, byte
offsets beyond 4 GiB), 65535 examples, 65535 channels.  The oracle computes what it can in
seconds: sub-boxes of the big grid around the atoms (a grid whose centre is a lattice point of
the big one has the same lattice points, exactly, for the binary fractions used here), and the
rest of the big grid must be zero."""
import numpy as np
import pytest

import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from test_gpu_parity import GRID_TOL, GRAD_RTOL, dev, mg  # noqa: E402,F401


def test_1024_points_per_side(mg):
    D, res, T, Dsub = 1024, 0.125, 2, 33
    dim = (D - 1) * res                     # 127.875: lattice points are multiples of 1/16
    half_sub = (Dsub - 1) // 2
    rng = np.random.default_rng(41)
    corners = [(16, 16, 16), (1007, 1007, 1007), (512, 300, 1007), (1007, 16, 700)]
    coords, types = [], []
    for c in corners:                       # atoms well inside a 33^3 sub-box about lattice point c
        centre = -dim / 2 + res * np.array(c)
        coords.append(centre + rng.uniform(-1.0, 1.0, (12, 3)))
        types.append(rng.integers(0, T, 12))
    coords = np.concatenate(coords)[None].astype(np.float32)
    types = np.concatenate(types)[None].astype(np.int32)
    radii = np.array([0.45, 0.6], np.float32)           # cutoff <= 0.9 A: spheres stay in the boxes
    gm = mg.GridMaker(res, dim, radius_type_indexed=True)
    assert gm.D == D
    out = gm.mg_forward_index(dev(coords), dev(types), dev(radii), T)
    torch.cuda.synchronize()
    assert tuple(out.shape) == (1, T, D, D, D)
    inside = 0
    G = torch.zeros_like(out)
    gen = torch.Generator(device="cuda").manual_seed(5)
    ref_grad = np.zeros((1, coords.shape[1], 3))
    for n, c in enumerate(corners):
        lo = [v - half_sub for v in c]
        sl = (0, slice(None), slice(lo[0], lo[0] + Dsub), slice(lo[1], lo[1] + Dsub),
              slice(lo[2], lo[2] + Dsub))
        centre = (-dim / 2 + res * np.array(c)).astype(np.float32)[None]
        ref = oracle.forward_index(coords, types, radii, T, res, (Dsub - 1) * res, centers=centre)
        got = out[sl].cpu().numpy()
        assert np.abs(got - ref[0]).max() <= GRID_TOL, (n, np.abs(got - ref[0]).max())
        assert ref.max() > 0.5
        inside += int((got != 0).sum())
        # upstream gradient: random inside the boxes, zero elsewhere
        g = torch.randn((T, Dsub, Dsub, Dsub), generator=gen, device="cuda")
        G[sl] = g
        ref_grad += oracle.backward_index(coords, types, radii, T, res, (Dsub - 1) * res,
                                          g.cpu().numpy()[None], centers=centre)
    # nothing was written anywhere else: every nonzero lies in one of the four boxes
    assert int(torch.count_nonzero(out)) == inside
    assert bool(torch.isfinite(out).all())
    grad = gm.mg_backward_index(dev(coords), dev(types), dev(radii), T, G).cpu().numpy()
    assert np.abs(grad - ref_grad).max() <= GRAD_RTOL * np.abs(ref_grad).max()


def test_65535_examples(mg):
    B, N, T, D, res = 65535, 2, 1, 2, 1.0
    rng = np.random.default_rng(42)
    coords = rng.uniform(-1.5, 1.5, (B, N, 3)).astype(np.float32)
    types = rng.integers(-1, T, (B, N)).astype(np.int32)
    radii = np.array([0.9], np.float32)
    q = rng.standard_normal((B, 4)).astype(np.float32)
    gm = mg.GridMaker(res, (D - 1) * res, radius_type_indexed=True)
    out = gm.mg_forward_index(dev(coords), dev(types), dev(radii), T, quats=dev(q)).cpu().numpy()
    ref = oracle.forward_index(coords, types, radii, T, res, (D - 1) * res, quats=q)
    assert np.abs(out - ref).max() <= GRID_TOL
    assert (out[-1] == ref[-1]).all() or np.abs(out[-1] - ref[-1]).max() <= GRID_TOL
    G = rng.standard_normal(ref.shape).astype(np.float32)
    g = gm.mg_backward_index(dev(coords), dev(types), dev(radii), T, dev(G), quats=dev(q)).cpu().numpy()
    rg = oracle.backward_index(coords, types, radii, T, res, (D - 1) * res, G, quats=q)
    assert np.abs(g - rg).max() <= GRAD_RTOL * np.abs(rg).max()
    with pytest.raises(mg.MolgridError):
        gm.workspace_bytes(B + 1, N, T)


def test_65535_channels(mg):
    B, N, T, D, res = 1, 500, 65535, 3, 0.5
    rng = np.random.default_rng(43)
    coords = rng.uniform(-1.5, 1.5, (B, N, 3)).astype(np.float32)
    types = rng.integers(0, T, (B, N)).astype(np.int32)
    types[0, :4] = [0, T - 1, T - 1, T]                 # first and last channel; one past the end
    radii = rng.uniform(0.5, 1.5, T).astype(np.float32)
    gm = mg.GridMaker(res, (D - 1) * res, radius_type_indexed=True)
    out = gm.mg_forward_index(dev(coords), dev(types), dev(radii), T).cpu().numpy()
    ref = oracle.forward_index(coords, types, radii, T, res, (D - 1) * res)
    assert np.abs(out - ref).max() <= GRID_TOL
    assert ref[0, T - 1].max() > 0
    G = rng.standard_normal(ref.shape).astype(np.float32)
    g = gm.mg_backward_index(dev(coords), dev(types), dev(radii), T, dev(G)).cpu().numpy()
    rg = oracle.backward_index(coords, types, radii, T, res, (D - 1) * res, G)
    assert np.abs(g - rg).max() <= GRAD_RTOL * np.abs(rg).max()
    with pytest.raises(mg.MolgridError):
        gm.workspace_bytes(B, N, T + 1)


def test_backward_boxes_of_hundreds_of_voxels_per_side(mg):
    """Radii so large that an atom's cutoff box spans the whole 256^3 grid: millions of 4-voxel
    slots per atom (more than a float counts exactly), the every-slot-of-the-box path of the
    backward kernel, index and vector types.  The oracle's box variant visits the same voxels."""
    D, res, T = 256, 0.25, 2
    dim = (D - 1) * res
    rng = np.random.default_rng(44)
    coords = rng.uniform(-20.0, 20.0, (1, 3, 3)).astype(np.float32)
    types = np.array([[0, 1, 1]], np.int32)
    radii = np.array([30.0, 22.0], np.float32)          # cutoff 45 A and 33 A: 180 / 132 voxels
    G = rng.standard_normal((1, T, D, D, D)).astype(np.float32)
    gm = mg.GridMaker(res, dim, radius_type_indexed=True)
    assert gm.D == D
    dG = dev(G)
    g = gm.mg_backward_index(dev(coords), dev(types), dev(radii), T, dG).cpu().numpy()
    rg = oracle.backward_index(coords, types, radii, T, res, dim, G)
    assert np.abs(g - rg).max() <= GRAD_RTOL * np.abs(rg).max()
    weights = rng.uniform(0.1, 1.0, (1, 3, T)).astype(np.float32)
    gc, gw = gm.mg_backward_vector(dev(coords), dev(weights), dev(radii), dG)
    rc, rw = oracle.backward_vector(coords, weights, radii, res, dim, G)
    assert np.abs(gc.cpu().numpy() - rc).max() <= GRAD_RTOL * np.abs(rc).max()
    assert np.abs(gw.cpu().numpy() - rw).max() <= GRAD_RTOL * np.abs(rw).max()
