"""Pins for the oracle's real-valued forward pass (index and vector types)."""
import numpy as np
import pytest

import oracle
from paper_1912_04822_amd import workloads


def fwd(w, **kw):
    kw.setdefault("centers", w.centers)
    kw.setdefault("quats", w.quats)
    kw.setdefault("translations", w.translations)
    return oracle.forward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension, **kw)


def test_layout_and_axis_order():
    """An atom on grid point (i,j,k)=(3,5,7) puts exactly 1.0 at out[0,t,3,5,7] (x slowest)."""
    res, D = 0.5, 12
    dim = (D - 1) * res
    center = np.array([[1.0, -2.0, 0.5]], np.float32)
    p = center[0] - dim / 2 + res * np.array([3, 5, 7])
    coords = p.reshape(1, 1, 3).astype(np.float32)
    out = oracle.forward_index(coords, np.array([[2]], np.int32),
                               np.array([1.0, 1.0, 1.5], np.float32), 3, res, dim,
                               centers=center)
    assert out.shape == (1, 3, D, D, D) and out.dtype == np.float32
    assert out[0, 2, 3, 5, 7] == 1.0
    assert np.unravel_index(np.argmax(out), out.shape) == (0, 2, 3, 5, 7)
    assert out[0, :2].max() == 0.0
    # neighbours along each axis are at distance res: value rho(res / r)
    v = np.float32(oracle.density(res / 1.5, 1.0))
    assert out[0, 2, 4, 5, 7] == v and out[0, 2, 3, 6, 7] == v and out[0, 2, 3, 5, 8] == v


@pytest.mark.parametrize("make", [workloads.tiny, workloads.ragged_small])
def test_box_variant_equals_brute_force_bitwise(make):
    w = make()
    kw = dict(natoms=w.extra.get("natoms"), out_dtype=np.float64)
    a = fwd(w, box=True, **kw)
    b = fwd(w, box=False, **kw)
    assert np.array_equal(a, b)
    assert a.max() > 0.5


def test_box_variant_with_atoms_on_faces_and_outside():
    res, D = 0.5, 9
    dim = (D - 1) * res
    r = 1.0
    cut = 1.5 * r
    xs = [-dim / 2 - cut, -dim / 2 - cut + 1e-4, -dim / 2 - cut - 1e-4, -dim / 2, dim / 2,
          dim / 2 + cut - 1e-4, 0.0, 50.0]
    coords = np.array([[[x, 0.25, -0.25] for x in xs]], np.float32)
    types = np.zeros((1, len(xs)), np.int32)
    kw = dict(out_dtype=np.float64)
    a = oracle.forward_index(coords, types, np.array([r], np.float32), 1, res, dim, box=True, **kw)
    b = oracle.forward_index(coords, types, np.array([r], np.float32), 1, res, dim, box=False, **kw)
    assert np.array_equal(a, b)


def test_against_numpy_broadcast_on_tiny():
    """Brute force by a different route: dense numpy distance tensor, no loops over voxels."""
    w = workloads.ragged_small()
    nat = w.extra["natoms"]
    out = fwd(w, natoms=nat, out_dtype=np.float64)
    pos = oracle.transform(w.coords, w.centers, w.quats, w.translations).astype(np.float64)
    rho = np.vectorize(lambda x: oracle.density(x, 1.0))
    ax = np.arange(w.D) * w.resolution - 0.5 * (w.D - 1) * w.resolution
    for b in range(w.B):
        gx = w.centers[b, 0] + ax
        gy = w.centers[b, 1] + ax
        gz = w.centers[b, 2] + ax
        ref = np.zeros((w.T, w.D, w.D, w.D))
        for a in range(int(nat[b])):
            t = int(w.types[b, a])
            if t < 0 or t >= w.T:
                continue
            d = np.sqrt((gx[:, None, None] - pos[b, a, 0]) ** 2
                        + (gy[None, :, None] - pos[b, a, 1]) ** 2
                        + (gz[None, None, :] - pos[b, a, 2]) ** 2)
            ref[t] += rho(d / float(w.radii[t]))
        assert np.allclose(out[b], ref, atol=1e-13)
    assert out[2].max() == 0.0              # natoms = 0: an empty example is all zeros


def test_quarter_turn_equals_axis_permutation():
    w = workloads.tiny()
    base = fwd(w, out_dtype=np.float64)
    q = np.array([[1, 0, 0, 1]], np.float32)        # exact quarter turn about z
    rot = fwd(w, quats=q, out_dtype=np.float64)
    # rotated atom (-y, x, z): rot[i, j, k] == base[j, D-1-i, k]
    assert np.array_equal(rot, np.flip(base.swapaxes(2, 3), axis=2))
    q = np.array([[1, 1, 0, 0]], np.float32)        # about x: (x, -z, y)
    rot = fwd(w, quats=q, out_dtype=np.float64)
    # (the sum dx^2 + dy^2 + dz^2 is taken in another order here: equal to rounding)
    assert np.allclose(rot, np.flip(base.swapaxes(3, 4), axis=3), rtol=1e-13, atol=1e-15)


def test_translation_equivariance():
    w = workloads.tiny()
    base = fwd(w, out_dtype=np.float64)
    shift = np.array([3.0, -1.5, 8.0], np.float32)      # exactly representable shifts
    moved = oracle.forward_index(w.coords + shift, w.types, w.radii, w.T, w.resolution,
                                 w.dimension, centers=w.centers + shift, out_dtype=np.float64)
    assert np.allclose(moved, base, atol=1e-6)
    # a translation argument moves atoms relative to the grid by the same amount
    t = np.array([[0.5, 0.0, -1.0]], np.float32)
    a = fwd(w, translations=t, out_dtype=np.float64)
    b = oracle.forward_index(w.coords + t[0], w.types, w.radii, w.T, w.resolution, w.dimension,
                             out_dtype=np.float64)
    assert np.allclose(a, b, atol=1e-6)
    # one grid step along x is a shift of the array by one plane
    t = np.array([[w.resolution, 0, 0]], np.float32)
    c = fwd(w, translations=t, out_dtype=np.float64)
    assert np.allclose(c[:, :, 1:], base[:, :, :-1], atol=1e-6)


def test_radius_scale_and_per_atom_radii():
    w = workloads.tiny()
    a = fwd(w, radius_scale=1.25, out_dtype=np.float64)
    b = oracle.forward_index(w.coords, w.types, (w.radii.astype(np.float64) * 1.25), w.T,
                             w.resolution, w.dimension, out_dtype=np.float64)
    assert np.allclose(a, b, atol=1e-6)         # radii rounded to float on one side only
    per_atom = w.radii[w.types]
    c = oracle.forward_index(w.coords, w.types, per_atom, w.T, w.resolution, w.dimension,
                             radius_type_indexed=False, out_dtype=np.float64)
    assert np.array_equal(c, fwd(w, out_dtype=np.float64))


def test_gaussian_radius_multiple_changes_the_support():
    w = workloads.tiny()
    for grm in (0.5, 1.0, 2.0):
        out = fwd(w, grm=grm, out_dtype=np.float64)
        one = oracle.forward_index(np.zeros((1, 1, 3), np.float32), np.zeros((1, 1), np.int32),
                                   np.array([1.6], np.float32), 1, 0.5, 11.5, grm=grm,
                                   out_dtype=np.float64)
        reach = oracle.cutoff(grm) * float(np.float32(1.6))
        ax = np.arange(24) * 0.5 - 5.75
        d = np.sqrt(ax[:, None, None] ** 2 + ax[None, :, None] ** 2 + ax[None, None, :] ** 2)
        assert np.array_equal(one[0, 0] != 0, d < reach)
        assert out.max() > 0


def test_skipped_atoms_and_natoms():
    w = workloads.tiny()
    types = w.types.copy()
    types[0, ::3] = -1
    types[0, 1::7] = w.T            # out of range: skipped
    a = oracle.forward_index(w.coords, types, w.radii, w.T, w.resolution, w.dimension,
                             out_dtype=np.float64)
    keep = (types[0] >= 0) & (types[0] < w.T)
    b = oracle.forward_index(w.coords[:, keep], types[:, keep], w.radii, w.T, w.resolution,
                             w.dimension, out_dtype=np.float64)
    assert np.array_equal(a, b)
    c = oracle.forward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension,
                             natoms=np.array([40], np.int32), out_dtype=np.float64)
    d = oracle.forward_index(w.coords[:, :40], w.types[:, :40], w.radii, w.T, w.resolution,
                             w.dimension, out_dtype=np.float64)
    assert np.array_equal(c, d)
    coords = w.coords.copy()
    coords[0, 5] = np.nan
    e = oracle.forward_index(coords, w.types, w.radii, w.T, w.resolution, w.dimension,
                             out_dtype=np.float64)
    assert np.isfinite(e).all()


def test_vector_types_one_hot_equal_index_types_and_are_linear():
    w = workloads.ragged_small()
    types = np.clip(w.types, 0, w.T - 1)
    onehot = np.eye(w.T, dtype=np.float32)[types]
    kw = dict(centers=w.centers, quats=w.quats, translations=w.translations,
              out_dtype=np.float64)
    a = oracle.forward_index(w.coords, types, w.radii, w.T, w.resolution, w.dimension, **kw)
    b = oracle.forward_vector(w.coords, onehot, w.radii, w.resolution, w.dimension, **kw)
    assert np.array_equal(a, b)
    c = oracle.forward_vector(w.coords, w.weights, w.radii, w.resolution, w.dimension, **kw)
    d = oracle.forward_vector(w.coords, 2 * w.weights, w.radii, w.resolution, w.dimension, **kw)
    assert np.allclose(d, 2 * c, rtol=1e-15)
    e = oracle.forward_vector(w.coords, w.weights, w.radii, w.resolution, w.dimension, box=False,
                              **kw)
    assert np.array_equal(c, e)
    # channel t only sees column t of the weights
    w2 = w.weights.copy()
    w2[:, :, 1] = 0
    f = oracle.forward_vector(w.coords, w2, w.radii, w.resolution, w.dimension, **kw)
    assert f[:, 1].max() == 0 and np.array_equal(f[:, 0], c[:, 0])


def test_float_output_is_the_rounded_double_output():
    w = workloads.tiny()
    assert np.array_equal(fwd(w), fwd(w, out_dtype=np.float64).astype(np.float32))
    # using the un-rounded transformed coordinate moves the grid by far less than 1e-5
    wr = workloads.ragged_small()
    a = fwd(wr, out_dtype=np.float64, coords_as_float=True)
    b = fwd(wr, out_dtype=np.float64, coords_as_float=False)
    assert 0 < np.abs(a - b).max() < 2e-6
