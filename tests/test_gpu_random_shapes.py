"""Seeded random small problems (grid size, atom count, channel count, radii, density
parameters, ragged natoms, poses) through every mode of the HIP path, against the oracle."""
import numpy as np
import pytest

import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from test_gpu_parity import GRAD_RTOL, dev, grid_tol, mg  # noqa: E402,F401


def draw_case(rng):
    D = int(rng.choice([1, 2, 3, 5, 8, 11, 12, 16, 19, 24, 31, 40]))
    res = float(rng.choice([0.25, 0.375, 0.5, 0.75, 1.0]))
    B = int(rng.integers(1, 5))
    N = int(rng.choice([1, 2, 7, 33, 64, 65, 130, 300]))
    T = int(rng.choice([1, 2, 3, 5, 9]))
    dim = (D - 1) * res
    centers = rng.uniform(-4, 4, (B, 3)).astype(np.float32)
    span = dim / 2 + 3.0
    coords = (centers[:, None, :] + rng.uniform(-span, span, (B, N, 3))).astype(np.float32)
    types = rng.integers(-1, T + 1, (B, N)).astype(np.int32)
    radii = rng.uniform(0.5, 2.5, T).astype(np.float32)
    if rng.random() < 0.3:
        radii[rng.integers(0, T)] = 0.0                      # a channel that takes no atoms
    q = rng.standard_normal((B, 4)).astype(np.float32)
    t = rng.uniform(-1.5, 1.5, (B, 3)).astype(np.float32)
    natoms = rng.integers(0, N + 1, B).astype(np.int32) if rng.random() < 0.5 else None
    weights = rng.dirichlet(np.full(T, 0.4), size=(B, N)).astype(np.float32)
    weights[rng.random((B, N, T)) < 0.2] = 0.0
    return dict(D=D, res=res, dim=dim, B=B, N=N, T=T, centers=centers, coords=coords, types=types,
                radii=radii, quats=q, translations=t, natoms=natoms, weights=weights,
                grm=float(rng.choice([0.5, 1.0, 1.5])), scale=float(rng.choice([0.8, 1.0, 1.25])))


@pytest.mark.parametrize("seed", range(24))
def test_random_small_problem(mg, seed):
    rng = np.random.default_rng(1000 + seed)
    c = draw_case(rng)
    pose = dict(centers=c["centers"], quats=c["quats"], translations=c["translations"])
    dpose = {k: dev(v) for k, v in pose.items()}
    nat = c["natoms"]
    common = dict(grm=c["grm"], radius_scale=c["scale"], natoms=nat, **pose)
    gm = mg.GridMaker(c["res"], c["dim"], radius_type_indexed=True, radius_scale=c["scale"],
                      gaussian_radius_multiple=c["grm"])
    assert gm.D == c["D"]
    co, ty, ra, we = dev(c["coords"]), dev(c["types"]), dev(c["radii"]), dev(c["weights"])
    # forward, index types
    out = gm.mg_forward_index(co, ty, ra, c["T"], natoms=dev(nat), **dpose).cpu().numpy()
    ref = oracle.forward_index(c["coords"], c["types"], c["radii"], c["T"], c["res"], c["dim"],
                               **common)
    assert np.abs(out - ref).max() <= grid_tol(ref), ("index", seed)
    # forward, vector types
    outv = gm.mg_forward_vector(co, we, ra, natoms=dev(nat), **dpose).cpu().numpy()
    refv = oracle.forward_vector(c["coords"], c["weights"], c["radii"], c["res"], c["dim"], **common)
    assert np.abs(outv - refv).max() <= grid_tol(refv), ("vector", seed)
    # binary, bit-exact
    gmb = mg.GridMaker(c["res"], c["dim"], binary=True, radius_type_indexed=True,
                       radius_scale=c["scale"])
    outb = gmb.mg_forward_index(co, ty, ra, c["T"], natoms=dev(nat), **dpose).cpu().numpy()
    refb = oracle.forward_binary(c["coords"], c["radii"], c["T"], c["res"], c["dim"],
                                 types=c["types"], radius_scale=c["scale"], natoms=nat, **pose)
    assert np.array_equal(outb.view(np.uint32), refb.view(np.uint32)), ("binary", seed)
    # backward, both kinds of types
    G = rng.standard_normal(ref.shape).astype(np.float32)
    g = gm.mg_backward_index(co, ty, ra, c["T"], dev(G), natoms=dev(nat), **dpose).cpu().numpy()
    rg = oracle.backward_index(c["coords"], c["types"], c["radii"], c["T"], c["res"], c["dim"], G,
                               **common)
    gc, gw = gm.mg_backward_vector(co, we, ra, dev(G), natoms=dev(nat), **dpose)
    rc, rw = oracle.backward_vector(c["coords"], c["weights"], c["radii"], c["res"], c["dim"], G,
                                    **common)
    for b in range(c["B"]):
        for got, want, what in ((g[b], rg[b], "gi"), (gc[b].cpu().numpy(), rc[b], "gc"),
                                (gw[b].cpu().numpy(), rw[b], "gw")):
            scale = np.abs(want).max()
            assert np.abs(got - want).max() <= GRAD_RTOL * scale + 1e-30, (what, seed, b)


def draw_wide_case(rng):
    """Larger and odder problems than draw_case: grids around the 4 KB tile sizes, thousands of
    atoms, tens of channels, weights of either sign and of size 30-300, crowded atoms (tiles that
    fall back to float accumulation); bounded so that the oracle takes a second or two."""
    while True:
        D = int(rng.choice([5, 16, 19, 31, 47, 48, 49, 63, 64, 65]))
        res = float(rng.choice([0.25, 0.375, 0.5, 0.75, 1.0]))
        B = int(rng.integers(1, 4))
        N = int(rng.choice([7, 65, 300, 1000, 2040, 4097]))
        T = int(rng.choice([1, 3, 9, 28, 64, 70]))
        vox = min(D, 2 * 3.75 / res + 1) ** 3
        if B * N * vox * T <= 1.5e8 and B * T * D ** 3 <= 2e7:
            break
    c = dict(D=D, res=res, B=B, N=N, T=T, dim=(D - 1) * res)
    c["centers"] = rng.uniform(-4, 4, (B, 3)).astype(np.float32)
    span = c["dim"] / 2 + 3.0
    c["coords"] = (c["centers"][:, None, :] + rng.uniform(-span, span, (B, N, 3))).astype(np.float32)
    if rng.random() < 0.25:     # crowded
        c["coords"][:, : N // 2] = c["centers"][:, None, :] + rng.normal(0, 0.3, (B, N // 2, 3)).astype(np.float32)
    c["types"] = rng.integers(-1, T + 1, (B, N)).astype(np.int32)
    c["radii"] = rng.uniform(0.5, 2.5, T).astype(np.float32)
    c["quats"] = rng.standard_normal((B, 4)).astype(np.float32)
    c["translations"] = rng.uniform(-1.5, 1.5, (B, 3)).astype(np.float32)
    c["natoms"] = rng.integers(0, N + 1, B).astype(np.int32) if rng.random() < 0.5 else None
    w = rng.dirichlet(np.full(T, 0.4), size=(B, N)).astype(np.float32)
    w[rng.random((B, N, T)) < 0.2] = 0.0
    if rng.random() < 0.5:
        w *= rng.choice([-1.0, 1.0], size=w.shape).astype(np.float32)
    if rng.random() < 0.25:
        w *= np.float32(rng.choice([30.0, 300.0]))
    c["weights"] = w
    c["grm"] = float(rng.choice([0.5, 1.0, 1.5]))
    c["scale"] = float(rng.choice([0.8, 1.0, 1.25]))
    c["f64"] = bool(rng.random() < 0.3)
    return c


@pytest.mark.parametrize("seed", range(16))
def test_random_wider_problem(mg, seed):
    rng = np.random.default_rng(7000 + seed)
    c = draw_wide_case(rng)
    pose = dict(centers=c["centers"], quats=c["quats"], translations=c["translations"])
    dpose = {k: dev(v) for k, v in pose.items()}
    nat = c["natoms"]
    common = dict(grm=c["grm"], radius_scale=c["scale"], natoms=nat, **pose)
    gm = mg.GridMaker(c["res"], c["dim"], radius_type_indexed=True, radius_scale=c["scale"],
                      gaussian_radius_multiple=c["grm"])
    assert gm.D == c["D"]
    co, ty, ra, we = dev(c["coords"]), dev(c["types"]), dev(c["radii"]), dev(c["weights"])
    odt = torch.float64 if c["f64"] else torch.float32
    shape = (c["B"], c["T"]) + (c["D"],) * 3
    # index types (into a grid of floats or doubles)
    out = torch.empty(shape, dtype=odt, device="cuda")
    gm.mg_forward_index(co, ty, ra, c["T"], natoms=dev(nat), out=out, **dpose)
    ref = oracle.forward_index(c["coords"], c["types"], c["radii"], c["T"], c["res"], c["dim"],
                               **common)
    assert np.abs(out.cpu().numpy() - ref).max() <= grid_tol(ref), ("index", seed)
    # vector types, weights of either sign: the error goes with what was added up, sum |w| rho
    outv = torch.empty(shape, dtype=odt, device="cuda")
    gm.mg_forward_vector(co, we, ra, natoms=dev(nat), out=outv, **dpose)
    refv = oracle.forward_vector(c["coords"], c["weights"], c["radii"], c["res"], c["dim"], **common)
    refa = oracle.forward_vector(c["coords"], np.abs(c["weights"]), c["radii"], c["res"], c["dim"],
                                 **common)
    assert np.abs(outv.cpu().numpy() - refv).max() <= grid_tol(refa), ("vector", seed)
    # binary occupancy, index and vector types, bit-exact
    gmb = mg.GridMaker(c["res"], c["dim"], binary=True, radius_type_indexed=True,
                       radius_scale=c["scale"])
    outb = gmb.mg_forward_index(co, ty, ra, c["T"], natoms=dev(nat), **dpose).cpu().numpy()
    refb = oracle.forward_binary(c["coords"], c["radii"], c["T"], c["res"], c["dim"],
                                 types=c["types"], radius_scale=c["scale"], natoms=nat, **pose)
    assert np.array_equal(outb.view(np.uint32), refb.view(np.uint32)), ("binary", seed)
    outbv = gmb.mg_forward_vector(co, we, ra, natoms=dev(nat), **dpose).cpu().numpy()
    refbv = oracle.forward_binary(c["coords"], c["radii"], c["T"], c["res"], c["dim"],
                                  weights=c["weights"], radius_scale=c["scale"], natoms=nat, **pose)
    assert np.array_equal(outbv.view(np.uint32), refbv.view(np.uint32)), ("binary vector", seed)
    # backward; the vector-typed sums are scaled by what |w| would give (signed weights cancel)
    G = rng.standard_normal(ref.shape).astype(np.float64 if c["f64"] else np.float32)
    g = gm.mg_backward_index(co, ty, ra, c["T"], dev(G), natoms=dev(nat), **dpose).cpu().numpy()
    rg = oracle.backward_index(c["coords"], c["types"], c["radii"], c["T"], c["res"], c["dim"], G,
                               **common)
    gc, gw = gm.mg_backward_vector(co, we, ra, dev(G), natoms=dev(nat), **dpose)
    rc, rw = oracle.backward_vector(c["coords"], c["weights"], c["radii"], c["res"], c["dim"], G,
                                    **common)
    ra_c, _ = oracle.backward_vector(c["coords"], np.abs(c["weights"]), c["radii"], c["res"],
                                     c["dim"], np.abs(G), **common)
    for b in range(c["B"]):
        for got, want, scale, what in ((g[b], rg[b], np.abs(rg[b]).max(), "gi"),
                                       (gc[b].cpu().numpy(), rc[b], max(np.abs(rc[b]).max(), np.abs(ra_c[b]).max() * 0.1), "gc"),
                                       (gw[b].cpu().numpy(), rw[b], np.abs(rw[b]).max(), "gw")):
            assert np.abs(got - want).max() <= GRAD_RTOL * scale + 1e-30, (what, seed, b)
