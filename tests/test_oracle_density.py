"""Pins for the oracle's density function and its volume integral.

None of these re-type the oracle's formula: they use what the paper fixes (a
unit-peak Gaussian to grm, a quadratic that decays to zero at the printed
cutoff), smoothness at the two special points, a closed form built from erf,
and numerical quadrature.
"""
import math
import os

import numpy as np
import pytest
from scipy import integrate

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")
GRMS = [0.25, 0.5, 0.75, 1.0, 1.5, 2.0]


def read_golden():
    vals = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split("=")
            vals[k.strip()] = v.strip()
    return vals


def test_cutoff_matches_paper_values():
    g = read_golden()
    for key, val in g.items():
        if key.startswith("cutoff_at_grm_"):
            grm = float(key[len("cutoff_at_grm_"):])
            assert oracle.cutoff(grm) == pytest.approx(float(val), abs=1e-15)


def test_default_grid_has_48_points():
    g = read_golden()
    assert oracle.points_per_side(float(g["resolution"]), float(g["dimension"])) == 48
    assert oracle.points_per_side(0.5, 11.5) == 24
    assert oracle.points_per_side(0.25, 23.75) == 96


@pytest.mark.parametrize("grm", GRMS)
def test_peak_is_one_and_gaussian_core(grm):
    assert oracle.density(0.0, grm) == 1.0
    # a Gaussian: log(rho) is proportional to x^2 inside the core
    xs = np.linspace(0.05, grm, 7)
    k = [math.log(oracle.density(x, grm)) / (x * x) for x in xs]
    assert np.allclose(k, k[0], rtol=1e-12)
    assert k[0] < 0


@pytest.mark.parametrize("grm", GRMS)
def test_join_is_c1_and_cutoff_is_a_smooth_zero(grm):
    c = oracle.cutoff(grm)
    eps = 1e-9
    # value continuity at the join and at the cutoff
    assert oracle.density(grm - eps, grm) == pytest.approx(oracle.density(grm + eps, grm), abs=1e-8)
    assert oracle.density(c, grm) == 0.0
    assert oracle.density(c - eps, grm) == pytest.approx(0.0, abs=1e-15)
    assert oracle.density(c + 1.0, grm) == 0.0
    # slope continuity at the join, zero slope at the cutoff
    assert oracle.density_deriv(grm - eps, grm) == pytest.approx(
        oracle.density_deriv(grm + eps, grm), abs=1e-7)
    assert oracle.density_deriv(c - eps, grm) == pytest.approx(0.0, abs=1e-7)
    assert oracle.density_deriv(c, grm) == 0.0
    # the tail is a quadratic: its third finite difference vanishes
    xs = np.linspace(grm + 1e-3, c - 1e-3, 9)
    v = np.array([oracle.density(x, grm) for x in xs])
    assert np.allclose(np.diff(v, 3), 0.0, atol=1e-13)
    # ... and it is the quadratic with a double root at c: rho/(x-c)^2 constant
    assert np.allclose(v / (xs - c) ** 2, v[0] / (xs[0] - c) ** 2, rtol=1e-10)


@pytest.mark.parametrize("grm", GRMS)
def test_monotone_nonnegative(grm):
    c = oracle.cutoff(grm)
    xs = np.linspace(0, c * 1.2, 2001)
    v = np.array([oracle.density(x, grm) for x in xs])
    assert (v >= 0).all()
    assert (np.diff(v) <= 1e-16).all()


@pytest.mark.parametrize("grm", GRMS)
def test_derivative_matches_finite_difference(grm):
    c = oracle.cutoff(grm)
    h = 1e-6
    for x in np.linspace(0.01, c * 1.1, 57):
        if abs(x - grm) < 2 * h or abs(x - c) < 2 * h:
            continue
        fd = (oracle.density(x + h, grm) - oracle.density(x - h, grm)) / (2 * h)
        assert oracle.density_deriv(x, grm) == pytest.approx(fd, abs=2e-9)


def test_known_values_at_grm_1():
    # exp(-2) at the join, and the slope there; independent constants
    assert oracle.density(1.0, 1.0) == pytest.approx(math.exp(-2.0), rel=1e-15)
    assert oracle.density(1.0, 1.0) == pytest.approx(0.1353352832366127, rel=1e-15)
    assert oracle.density_deriv(1.0, 1.0) == pytest.approx(-0.5413411329464508, rel=1e-14)
    # mid-tail: a parabola through (1, e^-2) with slope -4e^-2, double root at 1.5
    # is e^-2 (2x-3)^2, so rho(1.25) = e^-2 / 4
    assert oracle.density(1.25, 1.0) == pytest.approx(math.exp(-2.0) / 4.0, rel=1e-14)


def closed_form_volume(grm):
    """Integral of rho(|x|) over R^3 in units of r^3: erf part + polynomial part."""
    c = (1 + 2 * grm * grm) / (2 * grm)
    gauss = (math.sqrt(math.pi) / (4 * 2 ** 1.5)) * math.erf(math.sqrt(2) * grm) \
        - grm * math.exp(-2 * grm * grm) / 4
    # slope continuity: A (c-g)^2 = exp(-2 g^2)
    A = math.exp(-2 * grm * grm) / (c - grm) ** 2

    def F(x):
        return x ** 5 / 5 - c * x ** 4 / 2 + c * c * x ** 3 / 3
    return 4 * math.pi * (gauss + A * (F(c) - F(grm)))


@pytest.mark.parametrize("grm", GRMS)
def test_quadrature_matches_closed_form(grm):
    c = oracle.cutoff(grm)
    num, _ = integrate.quad(lambda x: 4 * math.pi * x * x * oracle.density(x, grm), 0, c,
                            points=[grm], epsabs=1e-13, epsrel=1e-13)
    assert num == pytest.approx(closed_form_volume(grm), rel=1e-11)


def test_closed_form_value_at_grm_1():
    assert closed_form_volume(1.0) == pytest.approx(1.8153495674, rel=1e-9)


@pytest.mark.parametrize("r,res,tol", [(1.6, 0.5, 2e-3), (1.6, 0.25, 1e-4), (2.0, 0.5, 2e-3),
                                       (1.2, 0.5, 2e-3)])
def test_single_atom_lattice_sum_matches_volume_integral(r, res, tol):
    """One isolated atom on a grid point: res^3 * sum(grid) ~ r^3 * I(grm)."""
    D = 2 * int(math.ceil(1.5 * r / res)) + 5
    dim = (D - 1) * res
    coords = np.zeros((1, 1, 3), np.float32)
    out = oracle.forward_index(coords, np.zeros((1, 1), np.int32), np.array([r], np.float32), 1,
                               res, dim, out_dtype=np.float64, box=False)
    assert out.shape == (1, 1, D, D, D)
    lattice = out.sum() * res ** 3
    assert lattice == pytest.approx(r ** 3 * closed_form_volume(1.0), rel=tol)
    # and the atom sits exactly on the middle grid point: the value there is 1
    m = D // 2
    assert out[0, 0, m, m, m] == 1.0


@pytest.mark.parametrize("r,res", [(1.6, 0.5), (1.6, 0.25), (2.0, 0.5), (1.2, 0.5)])
def test_support_size_matches_lattice_count(r, res):
    """Non-zero voxels of one on-lattice atom = lattice points with d < 1.5 r (grm = 1)."""
    reach = int(math.ceil(1.5 * r / res)) + 1
    D = 2 * reach + 1
    out = oracle.forward_index(np.zeros((1, 1, 3), np.float32), np.zeros((1, 1), np.int32),
                               np.array([r], np.float32), 1, res, (D - 1) * res,
                               out_dtype=np.float64)
    r32 = float(np.float32(r))
    n = 0
    for i in range(-reach, reach + 1):
        for j in range(-reach, reach + 1):
            for k in range(-reach, reach + 1):
                if math.sqrt((i * i + j * j + k * k)) * res < 1.5 * r32:
                    n += 1
    assert int((out != 0).sum()) == n
    expected = {(1.6, 0.5): 461, (1.6, 0.25): 3743, (2.0, 0.5): 895, (1.2, 0.5): 179}
    assert n == expected[(r, res)]
