"""Pins for the oracle's backward pass: finite differences of the double forward,
the translational-invariance identity, compact support, box == brute force."""
import numpy as np
import pytest

import oracle
from paper_1912_04822_amd import workloads


def loss_index(w, coords, G, **kw):
    out = oracle.forward_index(coords, w.types, w.radii, w.T, w.resolution, w.dimension,
                               out_dtype=np.float64, coords_as_float=False, **kw)
    return float((G * out).sum())


def fd_grad(f, x, h):
    g = np.zeros(x.shape, np.float64)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        xp = x.copy(); xp[i] += h
        xm = x.copy(); xm[i] -= h
        # coordinates are float32 at the boundary: use the steps actually taken
        g[i] = (f(xp) - f(xm)) / (float(xp[i]) - float(xm[i]))
    return g


def relerr(a, ref):
    return np.abs(a - ref).max() / np.abs(ref).max()


def test_backward_matches_central_differences_tiny():
    w = workloads.tiny()
    rng = np.random.default_rng(5)
    G = rng.standard_normal(w.out_shape)
    g = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension, G,
                              coords_as_float=False)
    sub = w.coords[:, :24]
    wsub = workloads.Workload(**{**w.__dict__, "coords": sub, "types": w.types[:, :24], "N": 24})
    gsub = oracle.backward_index(sub, wsub.types, w.radii, w.T, w.resolution, w.dimension, G,
                                 coords_as_float=False)
    # each atom's gradient does not depend on the other atoms
    assert np.array_equal(gsub, g[:, :24])
    fd = fd_grad(lambda c: loss_index(wsub, c, G), sub, 2.5e-4)
    assert relerr(gsub, fd) < 2e-5
    assert np.abs(g).max() > 1.0


def test_backward_with_rotation_center_translation_and_ragged_input():
    w = workloads.ragged_small()
    nat = w.extra["natoms"]
    G = w.grad_out.astype(np.float64)
    kw = dict(natoms=nat, centers=w.centers, quats=w.quats, translations=w.translations)
    g = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension, G,
                              coords_as_float=False, **kw)
    fd = fd_grad(lambda c: loss_index(w, c, G, **kw), w.coords, 2.5e-4)
    assert relerr(g, fd) < 2e-5
    # padded atoms, skipped types and atoms past natoms get exactly zero
    for b in range(w.B):
        dead = (np.arange(w.N) >= nat[b]) | (w.types[b] < 0) | (w.types[b] >= w.T)
        assert (g[b][dead] == 0).all()
    assert (g[2] == 0).all()
    # box == brute force, bitwise
    g2 = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension, G,
                               coords_as_float=False, box=False, **kw)
    assert np.array_equal(g, g2)
    # grm other than 1
    g3 = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension, G,
                               coords_as_float=False, grm=0.6, radius_scale=1.1, **kw)
    fd3 = fd_grad(lambda c: loss_index(w, c, G, grm=0.6, radius_scale=1.1, **kw), w.coords, 2.5e-4)
    assert relerr(g3, fd3) < 2e-5


def test_sum_of_atom_gradients_is_minus_the_center_gradient():
    """Moving every atom and the grid center together changes nothing, so
    sum_a dL/dx_a = - dL/dcenter (holds with rotation: the center is the rotation origin)."""
    w = workloads.ragged_small()
    G = w.grad_out.astype(np.float64)
    kw = dict(quats=w.quats, translations=w.translations)
    g = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension, G,
                              coords_as_float=False, centers=w.centers, **kw)
    fdc = fd_grad(lambda c: loss_index(w, w.coords, G, centers=c, **kw), w.centers, 2.5e-4)
    assert np.allclose(g.sum(axis=1), -fdc, rtol=1e-4, atol=1e-4 * np.abs(fdc).max())


def test_far_atom_has_zero_gradient_and_support_is_compact():
    res, D = 0.5, 24
    dim = (D - 1) * res
    r = 1.6
    coords = np.array([[[0.1, 0.2, -0.3], [dim / 2 + 1.5 * r + 0.01, 0, 0]]], np.float32)
    types = np.zeros((1, 2), np.int32)
    G = np.random.default_rng(3).standard_normal((1, 1, D, D, D))
    g = oracle.backward_index(coords, types, np.array([r], np.float32), 1, res, dim, G,
                              box=False)
    assert (g[0, 1] == 0).all() and np.abs(g[0, 0]).max() > 0
    # zeroing G outside the atom's cutoff sphere does not change its gradient
    ax = np.arange(D) * res - dim / 2
    d = np.sqrt((ax[:, None, None] - coords[0, 0, 0]) ** 2 + (ax[None, :, None] - coords[0, 0, 1]) ** 2
                + (ax[None, None, :] - coords[0, 0, 2]) ** 2)
    G2 = G * (d < 1.5 * float(np.float32(r)))
    g2 = oracle.backward_index(coords, types, np.array([r], np.float32), 1, res, dim, G2,
                               box=False)
    assert np.array_equal(g[0, 0], g2[0, 0])
    # an atom exactly on a grid point with G a delta there: d = 0 contributes nothing
    G3 = np.zeros_like(G); G3[0, 0, 12, 12, 12] = 1.0
    p = np.array([[[ax[12], ax[12], ax[12]]]], np.float32)
    g3 = oracle.backward_index(p, np.zeros((1, 1), np.int32), np.array([r], np.float32), 1, res,
                               dim, G3)
    assert (g3 == 0).all()


def test_float_and_double_upstream_gradients_agree():
    w = workloads.tiny()
    G32 = np.random.default_rng(9).standard_normal(w.out_shape).astype(np.float32)
    a = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension, G32)
    b = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension,
                              G32.astype(np.float64))
    assert np.array_equal(a, b)


def test_vector_backward_matches_finite_differences_and_index_case():
    w = workloads.ragged_small(B=2, N=9, T=3, D=11)
    G = w.grad_out.astype(np.float64)
    kw = dict(centers=w.centers, quats=w.quats, translations=w.translations)

    def loss(coords, weights):
        out = oracle.forward_vector(coords, weights, w.radii, w.resolution, w.dimension,
                                    out_dtype=np.float64, coords_as_float=False, **kw)
        return float((G * out).sum())

    gc, gw = oracle.backward_vector(w.coords, w.weights, w.radii, w.resolution, w.dimension, G,
                                    coords_as_float=False, **kw)
    fdc = fd_grad(lambda c: loss(c, w.weights), w.coords, 2.5e-4)
    assert relerr(gc, fdc) < 2e-5
    fdw = fd_grad(lambda ww: loss(w.coords, ww), w.weights, 1e-2)
    assert relerr(gw, fdw) < 1e-6
    # one-hot weights reproduce the index-typed coordinate gradient
    types = np.clip(w.types, 0, w.T - 1)
    onehot = np.eye(w.T, dtype=np.float32)[types]
    gi = oracle.backward_index(w.coords, types, w.radii, w.T, w.resolution, w.dimension, G,
                               coords_as_float=False, **kw)
    gv, _ = oracle.backward_vector(w.coords, onehot, w.radii, w.resolution, w.dimension, G,
                                   coords_as_float=False, **kw)
    assert np.allclose(gi, gv, rtol=1e-13, atol=1e-15)
