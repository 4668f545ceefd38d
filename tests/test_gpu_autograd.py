"""The autograd wrapper: gradients that reach ``coords`` / ``weights`` through the grid equal the
oracle's backward for the same upstream gradient (GridMaker section: atomic gradients for
optimising coordinates and types)."""
import numpy as np
import pytest

import oracle
from paper_1912_04822_amd import workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from test_gpu_parity import GRID_TOL, GRAD_RTOL, dev, mg  # noqa: E402,F401


def test_index_types_gradient_of_a_squared_error_loss(mg):
    from paper_1912_04822_amd.autograd import GridLayer
    w = workloads.protein_ligand(B=2, seed=31)
    layer = GridLayer(w.resolution, w.dimension)
    coords = dev(w.coords).requires_grad_(True)
    rng = np.random.default_rng(8)
    target = rng.uniform(0, 1, w.out_shape).astype(np.float32)
    grid = layer(coords, dev(w.radii), types=dev(w.types), T=w.T, centers=dev(w.centers),
                 quats=dev(w.quats), translations=dev(w.translations))
    loss = ((grid - dev(target)) ** 2).sum()
    loss.backward()
    ref_grid = oracle.forward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension,
                                    centers=w.centers, quats=w.quats, translations=w.translations)
    assert np.abs(grid.detach().cpu().numpy() - ref_grid).max() <= GRID_TOL
    G = 2.0 * (ref_grid.astype(np.float64) - target)
    ref = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension, G,
                                centers=w.centers, quats=w.quats, translations=w.translations)
    got = coords.grad.cpu().numpy()
    for b in range(w.B):
        assert np.abs(got[b] - ref[b]).max() <= GRAD_RTOL * np.abs(ref[b]).max()


def test_vector_types_gradients_reach_coords_and_weights(mg):
    from paper_1912_04822_amd.autograd import GridLayer
    w = workloads.ragged_small()
    rng = np.random.default_rng(9)
    wts = rng.dirichlet(0.3 * np.ones(w.T), (w.B, w.N)).astype(np.float32)
    layer = GridLayer(w.resolution, w.dimension)
    coords = dev(w.coords).requires_grad_(True)
    weights = dev(wts).requires_grad_(True)
    G = rng.standard_normal((w.B, w.T, w.D, w.D, w.D)).astype(np.float32)
    grid = layer(coords, dev(w.radii), weights=weights, centers=dev(w.centers), quats=dev(w.quats),
                 translations=dev(w.translations))
    (grid * dev(G)).sum().backward()
    gc, gw = oracle.backward_vector(w.coords, wts, w.radii, w.resolution, w.dimension, G,
                                    centers=w.centers, quats=w.quats, translations=w.translations)
    got_c, got_w = coords.grad.cpu().numpy(), weights.grad.cpu().numpy()
    for b in range(w.B):
        assert np.abs(got_c[b] - gc[b]).max() <= GRAD_RTOL * max(np.abs(gc[b]).max(), 1e-30)
        assert np.abs(got_w[b] - gw[b]).max() <= GRAD_RTOL * max(np.abs(gw[b]).max(), 1e-30)
    # only the weights ask for a gradient
    weights2 = dev(wts).requires_grad_(True)
    grid = layer(dev(w.coords), dev(w.radii), weights=weights2, centers=dev(w.centers),
                 quats=dev(w.quats), translations=dev(w.translations))
    (grid * dev(G)).sum().backward()
    assert torch.equal(weights2.grad, weights.grad)


def test_gradient_descent_on_coordinates_lowers_the_loss(mg):
    """Coordinate optimisation through the grid: move displaced atoms back towards the grid of
    the undisplaced ones; a few plain gradient steps reduce the squared error."""
    from paper_1912_04822_amd.autograd import GridLayer
    w = workloads.tiny()
    layer = GridLayer(w.resolution, w.dimension)
    radii, types = dev(w.radii), dev(w.types)
    with torch.no_grad():
        target = layer(dev(w.coords), radii, types=types, T=w.T)
    rng = np.random.default_rng(10)
    x = dev(w.coords + rng.normal(0, 0.15, w.coords.shape).astype(np.float32)).requires_grad_(True)
    losses = []
    for _ in range(12):
        loss = ((layer(x, radii, types=types, T=w.T) - target) ** 2).sum()
        losses.append(float(loss.detach()))
        (g,) = torch.autograd.grad(loss, x)
        with torch.no_grad():
            x -= 0.02 * g
    assert losses[-1] < 0.5 * losses[0]
    assert losses[1] < losses[0]            # the first step goes downhill


def test_subgrid_layer_gradient(mg):
    """A 2x2x2 sequence of subgrids as a layer: the gradient of a weighted sum over all subgrids
    equals the oracle's subgrid backward (contributions of the subgrids added up per atom)."""
    from paper_1912_04822_amd.autograd import GridLayer
    w = workloads.ragged_small(seed=5, B=2, N=120, T=3, D=10, resolution=0.5)
    S = 2
    layer = GridLayer(w.resolution, w.dimension, subgrids_per_side=S)
    coords = dev(w.coords).requires_grad_(True)
    grid = layer(coords, dev(w.radii), types=dev(w.types), T=w.T, centers=dev(w.centers),
                 quats=dev(w.quats), translations=dev(w.translations))
    assert tuple(grid.shape) == (w.B, S, S, S, w.T, w.D, w.D, w.D)
    rng = np.random.default_rng(12)
    G = rng.standard_normal(tuple(grid.shape)).astype(np.float32)
    (grid * dev(G)).sum().backward()
    ref_grid = oracle.forward_subgrids(w.coords, w.radii, S, w.resolution, w.dimension, T=w.T,
                                       types=w.types, centers=w.centers, quats=w.quats,
                                       translations=w.translations)
    assert np.abs(grid.detach().cpu().numpy() - ref_grid).max() <= GRID_TOL
    ref = oracle.backward_subgrids(w.coords, w.radii, S, w.resolution, w.dimension, G, T=w.T,
                                   types=w.types, centers=w.centers, quats=w.quats,
                                   translations=w.translations)
    got = coords.grad.cpu().numpy()
    for b in range(w.B):
        assert np.abs(got[b] - ref[b]).max() <= GRAD_RTOL * np.abs(ref[b]).max()


def test_layer_with_random_augmentation_keeps_the_applied_transforms(mg):
    """Random rotation + translation drawn per call: the grid and the gradient equal the oracle's
    for the transforms the layer kept; the next call draws different ones; the same seed and call
    number draw the same."""
    from paper_1912_04822_amd.autograd import GridLayer
    w = workloads.ragged_small(seed=6, B=3, N=90, T=3, D=12, resolution=0.5)
    layer = GridLayer(w.resolution, w.dimension)
    layer.seed = 77
    coords = dev(w.coords).requires_grad_(True)
    rng = np.random.default_rng(13)
    G = rng.standard_normal(w.out_shape).astype(np.float32)
    grid = layer(coords, dev(w.radii), types=dev(w.types), T=w.T, centers=dev(w.centers),
                 random_rotation=True, random_translation=1.5)
    (grid * dev(G)).sum().backward()
    q, t = layer.last_quats.cpu().numpy(), layer.last_translations.cpu().numpy()
    rq, rt = oracle.draw_transforms(77, 0, w.B, True, 1.5)
    assert np.abs(q - rq).max() <= 1.2e-7 and np.abs(t - rt).max() <= 2.4e-7   # one float ulp
    assert np.abs(t).max() <= 1.5 and np.allclose((q.astype(np.float64) ** 2).sum(1), 1.0, atol=1e-6)
    ref_grid = oracle.forward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension,
                                    centers=w.centers, quats=q, translations=t)
    assert np.abs(grid.detach().cpu().numpy() - ref_grid).max() <= GRID_TOL
    ref = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension, G,
                                centers=w.centers, quats=q, translations=t)
    got = coords.grad.cpu().numpy()
    for b in range(w.B):
        assert np.abs(got[b] - ref[b]).max() <= GRAD_RTOL * np.abs(ref[b]).max()
    layer(dev(w.coords), dev(w.radii), types=dev(w.types), T=w.T, random_rotation=True)
    assert not np.array_equal(layer.last_quats.cpu().numpy(), q)
    assert float(layer.last_translations.abs().max()) == 0.0
    again = GridLayer(w.resolution, w.dimension)
    again.seed = 77
    again(dev(w.coords), dev(w.radii), types=dev(w.types), T=w.T, random_rotation=True,
          random_translation=1.5)
    assert np.array_equal(again.last_quats.cpu().numpy(), q)


def test_binary_grid_refuses_a_gradient(mg):
    from paper_1912_04822_amd.autograd import GridLayer
    w = workloads.tiny()
    layer = GridLayer(w.resolution, w.dimension, binary=True)
    x = dev(w.coords).requires_grad_(True)
    grid = layer(x, dev(w.radii), types=dev(w.types), T=w.T)
    with pytest.raises(RuntimeError):
        grid.sum().backward()
