"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element.

Tolerances (the benchmark spec): real-valued grid max-abs 1e-5; binary bit-exact; gradients
relative 1e-4, taken as max_a |delta_a|_inf <= 1e-4 * max_a |g_ref,a|_inf per example.
"""
import numpy as np
import pytest

import oracle
from paper_1912_04822_amd import workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

GRID_TOL = 1e-5
GRAD_RTOL = 1e-4


def grid_tol(ref):
    """1e-5 as long as no voxel sum passes 8 (every workload of the paper's shape: their sums stay
    below 3); where thousands of atoms pile up on a voxel the bound follows the largest sum, 2e-6
    of it (about 17 float spacings of that value), and is never below 1e-5."""
    return max(GRID_TOL, 2e-6 * float(np.max(ref)))


@pytest.fixture(scope="module")
def mg():
    from paper_1912_04822_amd import molgrid
    molgrid.lib()           # raises if the HIP library is not built: no fallback
    return molgrid


@pytest.fixture(autouse=True, params=[1, 0], ids=["single_launch", "prep_tables"])
def both_small_problem_paths(request, mg):
    """Small problems (at most 256 atoms per example, 2048 in all) run as one kernel launch by
    default; every test of this file also runs with that path switched off, so that the small
    and awkward cases keep exercising the prep kernel and its tables as well."""
    mg.set_option("single_launch", request.param)
    yield
    mg.set_option("single_launch", 1)


def dev(a, dtype=None):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def run_forward_index(mg, w, *, binary=False, grm=1.0, radius_scale=1.0, natoms=None,
                      per_atom_radii=False):
    gm = mg.GridMaker(w.resolution, w.dimension, binary=binary,
                      radius_type_indexed=not per_atom_radii, radius_scale=radius_scale,
                      gaussian_radius_multiple=grm)
    assert gm.D == w.D
    radii = w.radii[np.clip(w.types, 0, w.T - 1)] if per_atom_radii else w.radii
    out = gm.mg_forward_index(dev(w.coords), dev(w.types), dev(radii), w.T, natoms=dev(natoms),
                              centers=dev(w.centers), quats=dev(w.quats),
                              translations=dev(w.translations))
    torch.cuda.synchronize()
    return out.cpu().numpy()


def oracle_forward_index(w, *, binary=False, grm=1.0, radius_scale=1.0, natoms=None,
                         per_atom_radii=False, **kw):
    radii = w.radii[np.clip(w.types, 0, w.T - 1)] if per_atom_radii else w.radii
    common = dict(natoms=natoms, centers=w.centers, quats=w.quats, translations=w.translations,
                  radius_scale=radius_scale, radius_type_indexed=not per_atom_radii)
    if binary:
        return oracle.forward_binary(w.coords, radii, w.T, w.resolution, w.dimension,
                                     types=w.types, **common)
    return oracle.forward_index(w.coords, w.types, radii, w.T, w.resolution, w.dimension, grm=grm,
                                **common, **kw)


# ---------------------------------------------------------------------------
# step 1: transform
# ---------------------------------------------------------------------------

def test_transform_is_bit_identical_to_the_oracle(mg):
    rng = np.random.default_rng(11)
    B, N = 37, 1111
    x = rng.uniform(-40, 40, (B, N, 3)).astype(np.float32)
    c = rng.uniform(-10, 10, (B, 3)).astype(np.float32)
    t = rng.uniform(-2, 2, (B, 3)).astype(np.float32)
    q = (rng.standard_normal((B, 4)) * rng.uniform(0.1, 10, (B, 1))).astype(np.float32)
    q[3] = 0                    # no rotation given
    q[4] = [1, 0, 0, 1]         # exact quarter turn
    got = mg.mg_transform_forward(dev(x), dev(c), dev(q), dev(t)).cpu().numpy()
    ref = oracle.transform(x, c, q, t)
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    got = mg.mg_transform_forward(dev(x)).cpu().numpy()
    assert np.array_equal(got, x)


# ---------------------------------------------------------------------------
# steps 2-3: forward, index types
# ---------------------------------------------------------------------------

def test_forward_tiny(mg):
    w = workloads.tiny()
    got = run_forward_index(mg, w)
    ref = oracle_forward_index(w)
    assert got.shape == (1, 4, 24, 24, 24)
    assert np.abs(got - ref).max() <= GRID_TOL
    # also against the all-double reading (transformed coordinate not rounded to float)
    ref64 = oracle_forward_index(w, coords_as_float=False, box=False)
    assert np.abs(got - ref64).max() <= GRID_TOL


@pytest.mark.parametrize("grm,scale", [(1.0, 1.0), (0.5, 1.3), (2.0, 0.8)])
def test_forward_ragged_small_unaligned_grid(mg, grm, scale):
    """D = 13 (rows not 16-byte aligned), off-origin centers, padded / out-of-range types,
    natoms = [N, N/2, 0], un-normalised quaternions."""
    w = workloads.ragged_small()
    nat = w.extra["natoms"]
    got = run_forward_index(mg, w, grm=grm, radius_scale=scale, natoms=nat)
    ref = oracle_forward_index(w, grm=grm, radius_scale=scale, natoms=nat)
    assert np.abs(got - ref).max() <= GRID_TOL
    assert got[2].max() == 0.0


@pytest.mark.parametrize("N,single_type", [(5000, False), (9000, False), (9000, True)])
def test_forward_backward_many_atoms_per_example(mg, N, single_type):
    """N = 5000: eight atoms per thread in the one-workgroup-per-example prep kernel.  N = 9000 is
    past what that kernel takes (the per-group kernel runs instead); with every atom of one type
    the group is also too long for that kernel to bin by x-plane (records stay in atom order)."""
    w = workloads.ragged_small(seed=11, B=2, N=N, T=3, D=16, resolution=0.5)
    if single_type:
        w.types[:] = 1
    nat = np.array([N, N - 679], np.int32)
    got = run_forward_index(mg, w, natoms=nat)
    ref = oracle_forward_index(w, natoms=nat)
    # dozens of atoms overlap in every voxel: float accumulation, error relative to the sums
    assert np.abs(got - ref).max() <= GRID_TOL + 2e-6 * ref.max()
    gotb = run_forward_index(mg, w, natoms=nat, binary=True)
    refb = oracle_forward_index(w, natoms=nat, binary=True)
    assert np.array_equal(gotb.view(np.uint32), refb.astype(np.float32).view(np.uint32))
    gb = run_backward_index(mg, w, natoms=nat)
    rb = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension,
                               w.grad_out, natoms=nat, centers=w.centers, quats=w.quats,
                               translations=w.translations)
    assert grad_err(gb, rb) <= GRAD_RTOL


def test_forward_backward_many_channels(mg):
    """T * (D + 3) = 300 * 27 (type, x-bin) pairs are more than the one-workgroup-per-example prep
    kernel keeps in LDS: the per-group kernel runs instead."""
    w = workloads.ragged_small(seed=23, B=2, N=400, T=300, D=24, resolution=0.5)
    got = run_forward_index(mg, w)
    ref = oracle_forward_index(w)
    assert np.abs(got - ref).max() <= GRID_TOL
    assert (ref.reshape(2, 300, -1).max(axis=2) > 0).sum() > 100     # many channels hold atoms
    gotb = run_forward_index(mg, w, binary=True)
    refb = oracle_forward_index(w, binary=True)
    assert np.array_equal(gotb.view(np.uint32), refb.astype(np.float32).view(np.uint32))
    gb = run_backward_index(mg, w)
    rb = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension,
                               w.grad_out, centers=w.centers, quats=w.quats,
                               translations=w.translations)
    assert grad_err(gb, rb) <= GRAD_RTOL


@pytest.mark.parametrize("D,res", [(1, 1.0), (4, 0.5), (7, 0.3), (50, 0.5), (130, 0.125)])
def test_forward_odd_grid_sizes(mg, D, res):
    w = workloads.ragged_small(seed=D, B=2, N=50, T=3, D=D, resolution=res)
    got = run_forward_index(mg, w)
    ref = oracle_forward_index(w)
    assert got.shape == ref.shape
    assert np.abs(got - ref).max() <= GRID_TOL


def test_forward_per_atom_radii(mg):
    w = workloads.ragged_small()
    got = run_forward_index(mg, w, per_atom_radii=True)
    ref = oracle_forward_index(w, per_atom_radii=True)
    assert np.abs(got - ref).max() <= GRID_TOL


def test_forward_protein_ligand_subset_and_determinism(mg):
    w = workloads.protein_ligand(B=6)
    got = run_forward_index(mg, w)
    ref = oracle_forward_index(w)
    err = np.abs(got - ref).max()
    assert err <= GRID_TOL, err
    assert got.max() > 1.0
    again = run_forward_index(mg, w)
    assert np.array_equal(got.view(np.uint32), again.view(np.uint32))
    for tile_floats, waves in ((1024, 1), (1024, 2), (2048, 2), (2048, 4), (4096, 1), (4096, 2),
                               (4096, 4)):
        mg.set_option("tile_floats", tile_floats)
        mg.set_option("waves_per_tile", waves)
        try:
            other = run_forward_index(mg, w)
        finally:
            mg.set_option("tile_floats", 0)
            mg.set_option("waves_per_tile", 0)
        # the knob changes the order in which overlapping atoms are summed: equal to rounding
        assert np.abs(got - other).max() <= 2e-6
        assert np.abs(other - ref).max() <= GRID_TOL


@pytest.mark.parametrize("key,value", [("keep_alive", 0), ("keep_alive", 64), ("keep_alive", 1024),
                                       ("keep_alive_stride", 4), ("tile_order", 1), ("xcd_run", 8),
                                       ("lds_floor", 0), ("lds_floor", 16384)])
def test_launch_knobs_do_not_change_a_bit(mg, key, value):
    """Launch order, residency and the keep-alive reads only change when things run: the grid is
    the same to the bit (index types, binary, and an unaligned grid)."""
    cases = [workloads.protein_ligand(B=3, seed=17), workloads.ragged_small()]
    base = [(run_forward_index(mg, w), run_forward_index(mg, w, binary=True)) for w in cases]
    default = {"keep_alive": 1, "keep_alive_stride": 1, "tile_order": 0, "xcd_run": 0, "lds_floor": -1}[key]
    mg.set_option(key, value)
    try:
        for w, (real, binary) in zip(cases, base):
            assert np.array_equal(run_forward_index(mg, w).view(np.uint32), real.view(np.uint32))
            assert np.array_equal(run_forward_index(mg, w, binary=True).view(np.uint32),
                                  binary.view(np.uint32))
    finally:
        mg.set_option(key, default)


def test_forward_single_type_many_atoms(mg):
    """All atoms in one channel: the record list of that channel is longer than one LDS round."""
    w = workloads.protein_ligand(B=2)
    w.types[:] = 3
    got = run_forward_index(mg, w)
    ref = oracle_forward_index(w)
    assert ref.max() > 5                                # 2040 atoms of one type pile up
    err = np.abs(got - ref).max()
    assert err <= grid_tol(ref), (err, ref.max())
    assert got[:, :3].max() == 0 and got[:, 4:].max() == 0


def test_single_launch_path_equals_the_prep_path_bit_for_bit(mg):
    """Fixed-point sums do not depend on the order of the atoms, and both paths transform and
    cull with the same arithmetic: the grids are identical, real and binary."""
    cases = [(workloads.tiny(), None), (workloads.ragged_small(), workloads.ragged_small().extra["natoms"]),
             (workloads.protein_ligand(B=8, n_receptor=216, n_ligand=40, seed=9), None)]
    for w, nat in cases:
        assert w.N <= 256 and w.B * w.N <= 2048
        for binary in (False, True):
            for per_atom in (False, True):
                grids = []
                for single in (1, 0):
                    mg.set_option("single_launch", single)
                    grids.append(run_forward_index(mg, w, binary=binary, natoms=nat,
                                                   per_atom_radii=per_atom))
                assert np.array_equal(grids[0].view(np.uint32), grids[1].view(np.uint32))
                ref = oracle_forward_index(w, binary=binary, natoms=nat, per_atom_radii=per_atom)
                if binary:
                    assert np.array_equal(grids[0].view(np.uint32), ref.view(np.uint32))
                else:
                    assert np.abs(grids[0] - ref).max() <= GRID_TOL


def test_forward_overwrites_output_and_empty_batch(mg):
    w = workloads.tiny()
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    out = torch.full((1, 4, 24, 24, 24), 7.0, device="cuda")
    far = w.coords + 1000.0
    gm.mg_forward_index(dev(far), dev(w.types), dev(w.radii), w.T, out=out)
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0


# ---------------------------------------------------------------------------
# step 5: binary occupancy (bit-exact)
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("make", ["tiny", "ragged", "protein"])
def test_binary_is_bit_exact(mg, make):
    if make == "tiny":
        w, nat = workloads.tiny(), None
    elif make == "ragged":
        w = workloads.ragged_small()
        nat = w.extra["natoms"]
    else:
        w, nat = workloads.protein_ligand(B=6), None
    got = run_forward_index(mg, w, binary=True, natoms=nat)
    ref = oracle_forward_index(w, binary=True, natoms=nat)
    assert set(np.unique(got)) <= {0.0, 1.0}
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    assert got.sum() > 0 or make == "ragged"
    got2 = run_forward_index(mg, w, binary=True, natoms=nat, radius_scale=1.37)
    ref2 = oracle_forward_index(w, binary=True, natoms=nat, radius_scale=1.37)
    assert np.array_equal(got2.view(np.uint32), ref2.view(np.uint32))


def test_binary_knife_edges_on_lattice(mg):
    """Atoms exactly on grid points with radii that put grid points exactly at distance r."""
    res, D = 0.5, 16
    dim = (D - 1) * res
    ax = np.arange(D) * res - dim / 2
    coords = np.array([[[ax[3], ax[4], ax[5]], [ax[10], ax[10], ax[10]], [ax[0], ax[15], ax[7]]]],
                      np.float32)
    types = np.array([[0, 1, 2]], np.int32)
    radii = np.array([1.5, 2.0, 2.5], np.float32)        # multiples of res
    w = workloads.Workload("edges", 1, 3, 3, res, dim, D, coords, types, radii,
                           np.zeros((1, 3), np.float32))
    got = run_forward_index(mg, w, binary=True)
    ref = oracle_forward_index(w, binary=True)
    assert np.array_equal(got, ref)
    assert got[0, 0, 3, 4, 8] == 1.0 and got[0, 0, 3, 4, 9] == 0.0   # d = 1.5 inside, 2.0 outside


# ---------------------------------------------------------------------------
# step 4: vector types
# ---------------------------------------------------------------------------

def run_forward_vector(mg, w, binary=False, natoms=None):
    gm = mg.GridMaker(w.resolution, w.dimension, binary=binary, radius_type_indexed=True)
    out = gm.mg_forward_vector(dev(w.coords), dev(w.weights), dev(w.radii), natoms=dev(natoms),
                               centers=dev(w.centers), quats=dev(w.quats),
                               translations=dev(w.translations))
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_forward_vector_small_and_subset(mg):
    w = workloads.ragged_small()
    nat = w.extra["natoms"]
    got = run_forward_vector(mg, w, natoms=nat)
    ref = oracle.forward_vector(w.coords, w.weights, w.radii, w.resolution, w.dimension,
                                natoms=nat, centers=w.centers, quats=w.quats,
                                translations=w.translations)
    assert np.abs(got - ref).max() <= GRID_TOL
    w = workloads.protein_ligand(B=2, with_weights=True)
    got = run_forward_vector(mg, w)
    ref = oracle.forward_vector(w.coords, w.weights, w.radii, w.resolution, w.dimension,
                                centers=w.centers, quats=w.quats, translations=w.translations)
    assert np.abs(got - ref).max() <= GRID_TOL
    assert got.min() >= 0 and got.max() > 0.1


def test_forward_vector_negative_weights_large_weights_and_ragged_channel_groups(mg):
    """Weights of both signs (the signed path of the kernel that takes four channels at a time),
    weights so large that a tile's sums cannot stay in fixed point (it starts over in floats),
    and channel counts that leave the last group of four partly empty."""
    for T, scale, seed in ((5, 1.0, 1), (6, 1.0, 2), (7, 60.0, 3), (28, 200.0, 4), (1, 1.0, 5)):
        rng = np.random.default_rng(100 + seed)
        w = workloads.protein_ligand(B=2, seed=50 + seed)
        w.T = T
        w.radii = rng.uniform(1.0, 2.2, T).astype(np.float32)
        w.weights = (rng.standard_normal((w.B, w.N, T)) * scale).astype(np.float32)
        w.weights[rng.random((w.B, w.N, T)) < 0.3] = 0.0
        got = run_forward_vector(mg, w)
        ref = oracle.forward_vector(w.coords, w.weights, w.radii, w.resolution, w.dimension,
                                    centers=w.centers, quats=w.quats, translations=w.translations)
        scale_ref = float(np.abs(ref).max())
        assert scale_ref > 1.0
        err = float(np.abs(got - ref).max())
        assert err <= max(GRID_TOL, 2e-6 * scale_ref), (T, scale, err, scale_ref)
        again = run_forward_vector(mg, w)           # float tiles too repeat bit for bit
        assert np.array_equal(got.view(np.uint32), again.view(np.uint32))


def test_forward_and_backward_vector_with_more_channels_than_are_ranked(mg):
    """Beyond 256 channels the channels are taken as they come instead of in order of radius."""
    rng = np.random.default_rng(77)
    w = workloads.ragged_small(B=2, N=40, T=300, D=12)
    got = run_forward_vector(mg, w)
    ref = oracle.forward_vector(w.coords, w.weights, w.radii, w.resolution, w.dimension,
                                centers=w.centers, quats=w.quats, translations=w.translations)
    assert ref.max() > 0.05
    assert np.abs(got - ref).max() <= GRID_TOL
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    G = rng.standard_normal(ref.shape).astype(np.float32)
    gc, gw = gm.mg_backward_vector(dev(w.coords), dev(w.weights), dev(w.radii), dev(G),
                                   centers=dev(w.centers), quats=dev(w.quats),
                                   translations=dev(w.translations))
    rc, rw = oracle.backward_vector(w.coords, w.weights, w.radii, w.resolution, w.dimension, G,
                                    centers=w.centers, quats=w.quats, translations=w.translations)
    assert np.abs(gc.cpu().numpy() - rc).max() <= GRAD_RTOL * np.abs(rc).max()
    assert np.abs(gw.cpu().numpy() - rw).max() <= GRAD_RTOL * np.abs(rw).max()


def test_forward_vector_binary_is_bit_exact(mg):
    w = workloads.ragged_small()
    wt = w.weights.copy()
    wt[wt < 0.02] = 0.0                 # exact zeros: those atoms do not mark the channel
    w.weights = wt
    got = run_forward_vector(mg, w, binary=True)
    ref = oracle.forward_binary(w.coords, w.radii, w.T, w.resolution, w.dimension, weights=wt,
                                centers=w.centers, quats=w.quats, translations=w.translations)
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


@pytest.mark.parametrize("tile_floats,waves", [(512, 1), (1024, 1), (1024, 2), (2048, 1), (2048, 2),
                                               (2048, 4), (4096, 4)])
def test_tile_shapes_binary_and_vector(mg, tile_floats, waves):
    """The other tile sizes and workgroup shapes of the forward kernel, in binary and vector mode
    (several wavefronts per tile, several rounds of atoms, more than one pair of planes)."""
    mg.set_option("tile_floats", tile_floats)
    mg.set_option("waves_per_tile", waves)
    try:
        w = workloads.protein_ligand(B=2, with_weights=True)
        got = run_forward_index(mg, w, binary=True)
        ref = oracle_forward_index(w, binary=True)
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
        got = run_forward_vector(mg, w)
        ref = oracle.forward_vector(w.coords, w.weights, w.radii, w.resolution, w.dimension,
                                    centers=w.centers, quats=w.quats, translations=w.translations)
        assert np.abs(got - ref).max() <= GRID_TOL
        w = workloads.ragged_small()
        nat = w.extra["natoms"]
        got = run_forward_index(mg, w, natoms=nat)
        ref = oracle_forward_index(w, natoms=nat)
        assert np.abs(got - ref).max() <= GRID_TOL
    finally:
        mg.set_option("tile_floats", 0)
        mg.set_option("waves_per_tile", 0)


# ---------------------------------------------------------------------------
# step 6: backward
# ---------------------------------------------------------------------------

def grad_err(got, ref):
    worst = 0.0
    for b in range(ref.shape[0]):
        scale = np.abs(ref[b]).max()
        if scale == 0:
            assert np.abs(got[b]).max() == 0
            continue
        worst = max(worst, np.abs(got[b] - ref[b]).max() / scale)
    return worst


def run_backward_index(mg, w, natoms=None, grm=1.0):
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True,
                      gaussian_radius_multiple=grm)
    g = gm.mg_backward_index(dev(w.coords), dev(w.types), dev(w.radii), w.T, dev(w.grad_out),
                             natoms=dev(natoms), centers=dev(w.centers), quats=dev(w.quats),
                             translations=dev(w.translations))
    torch.cuda.synchronize()
    return g.cpu().numpy()


@pytest.mark.parametrize("grm", [1.0, 0.6])
def test_backward_ragged_small(mg, grm):
    w = workloads.ragged_small()
    nat = w.extra["natoms"]
    got = run_backward_index(mg, w, natoms=nat, grm=grm)
    ref = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension,
                                w.grad_out, grm=grm, natoms=nat, centers=w.centers, quats=w.quats,
                                translations=w.translations)
    assert grad_err(got, ref) <= GRAD_RTOL
    for b in range(w.B):
        dead = (np.arange(w.N) >= nat[b]) | (w.types[b] < 0) | (w.types[b] >= w.T)
        assert (got[b][dead] == 0).all()


def test_backward_protein_ligand_subset_and_finite_differences(mg):
    w = workloads.protein_ligand(B=3, with_grad=True)
    got = run_backward_index(mg, w)
    ref = oracle.backward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension,
                                w.grad_out, centers=w.centers, quats=w.quats,
                                translations=w.translations)
    assert got.shape == (3, 2040, 3)
    assert grad_err(got, ref) <= GRAD_RTOL
    # atoms whose cutoff misses the grid get exactly zero
    assert ((ref == 0) == (got == 0)).all()
    # central finite differences of the double forward on a few atoms
    G = w.grad_out.astype(np.float64)
    rng = np.random.default_rng(3)
    live = np.argwhere(np.abs(ref[0]).max(axis=1) > 1.0)[:, 0]
    for a in rng.choice(live, 4, replace=False):
        for k in range(3):
            vals = []
            for s in (+1, -1):
                c = w.coords[:1].copy()
                c[0, a, k] += s * 2.5e-4
                out = oracle.forward_index(c, w.types[:1], w.radii, w.T, w.resolution, w.dimension,
                                           centers=w.centers[:1], quats=w.quats[:1],
                                           translations=w.translations[:1], out_dtype=np.float64,
                                           coords_as_float=False)
                vals.append(((G[:1] * out).sum(), float(c[0, a, k])))
            fd = (vals[0][0] - vals[1][0]) / (vals[0][1] - vals[1][1])
            assert abs(got[0, a, k] - fd) <= 2e-4 * np.abs(ref[0]).max()
    again = run_backward_index(mg, w)
    assert np.array_equal(got.view(np.uint32), again.view(np.uint32))


def test_backward_vector(mg):
    w = workloads.ragged_small()
    nat = w.extra["natoms"]
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    gc, gw = gm.mg_backward_vector(dev(w.coords), dev(w.weights), dev(w.radii), dev(w.grad_out),
                                   natoms=dev(nat), centers=dev(w.centers), quats=dev(w.quats),
                                   translations=dev(w.translations))
    torch.cuda.synchronize()
    rc, rw = oracle.backward_vector(w.coords, w.weights, w.radii, w.resolution, w.dimension,
                                    w.grad_out, natoms=nat, centers=w.centers, quats=w.quats,
                                    translations=w.translations)
    assert grad_err(gc.cpu().numpy(), rc) <= GRAD_RTOL
    assert grad_err(gw.cpu().numpy(), rw) <= GRAD_RTOL
    # coordinates only / weights only
    gc2, none = gm.mg_backward_vector(dev(w.coords), dev(w.weights), dev(w.radii), dev(w.grad_out),
                                      natoms=dev(nat), centers=dev(w.centers), quats=dev(w.quats),
                                      translations=dev(w.translations), want_weights=False)
    assert none is None and torch.equal(gc2, gc)


@pytest.mark.parametrize("T", [6, 64, 70])
def test_backward_vector_channel_groups(mg, T):
    """Vector-typed backward takes an atom's channels four at a time, in order of radius when
    there are at most 64 of them: a last group that is not full (T = 6, 70), equal radii, a
    channel without radius, exactly 64 channels, and more than 64 (taken as they come)."""
    w = workloads.ragged_small(seed=40 + T, B=2, N=60, T=T, D=12, resolution=0.5)
    rng = np.random.default_rng(T)
    radii = rng.uniform(0.6, 2.2, T).astype(np.float32)
    radii[1] = radii[4]                     # a tie
    radii[2] = 0.0                          # takes no atoms: zero gradient
    wts = rng.dirichlet(0.4 * np.ones(T), (w.B, w.N)).astype(np.float32)
    wts[rng.random(wts.shape) < 0.2] = 0.0
    G = rng.standard_normal((w.B, T, w.D, w.D, w.D)).astype(np.float32)
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    gc, gw = gm.mg_backward_vector(dev(w.coords), dev(wts), dev(radii), dev(G),
                                   centers=dev(w.centers), quats=dev(w.quats),
                                   translations=dev(w.translations))
    rc, rw = oracle.backward_vector(w.coords, wts, radii, w.resolution, w.dimension, G,
                                    centers=w.centers, quats=w.quats, translations=w.translations)
    gc, gw = gc.cpu().numpy(), gw.cpu().numpy()
    for b in range(w.B):
        assert np.abs(gc[b] - rc[b]).max() <= GRAD_RTOL * np.abs(rc[b]).max()
        assert np.abs(gw[b] - rw[b]).max() <= GRAD_RTOL * np.abs(rw[b]).max()
    assert (gw[:, :, 2] == 0).all() and np.abs(rw[:, :, 2]).max() == 0


def test_backward_rejects_binary_mode(mg):
    w = workloads.tiny()
    gm = mg.GridMaker(w.resolution, w.dimension, binary=True, radius_type_indexed=True)
    with pytest.raises(mg.MolgridError) as e:
        gm.mg_backward_index(dev(w.coords), dev(w.types), dev(w.radii), w.T,
                             torch.zeros(w.out_shape, device="cuda"))
    assert e.value.code == -6


def _poisoned():
    """ragged_small with data errors planted: non-finite and huge coordinates, a NaN and a
    negative radius, types outside [0,T), natoms outside [0,N], a NaN quaternion, an infinite
    translation (the documented rule: such atoms contribute nothing and get zero gradient)."""
    w = workloads.ragged_small(seed=77, B=4, N=80, T=4, D=12, resolution=0.5)
    w.coords[0, 3, 1] = np.nan
    w.coords[0, 4, 0] = np.inf
    w.coords[0, 5, 2] = -np.inf
    w.coords[1, 6] = [1e30, -1e30, 3e38]
    w.types[0, 7] = w.T
    w.types[1, 8] = -5
    w.types[2, 9] = 2 ** 31 - 1
    radii = w.radii.copy()
    radii[1] = np.nan
    radii[2] = -1.0
    quats = w.quats.copy()
    quats[2] = [np.nan, 0.0, 1.0, 0.0]          # not a rotation: taken as the identity
    trans = w.translations.copy()
    trans[3, 1] = np.inf                         # every atom of example 3 becomes non-finite
    nat = np.array([w.N + 50, -3, w.N, w.N], np.int32)
    return w, radii, quats, trans, nat


def test_data_errors_are_skipped_not_reported(mg):
    w, radii, quats, trans, nat = _poisoned()
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    kw = dict(natoms=dev(nat), centers=dev(w.centers), quats=dev(quats), translations=dev(trans))
    okw = dict(natoms=nat, centers=w.centers, quats=quats, translations=trans)
    out = gm.mg_forward_index(dev(w.coords), dev(w.types), dev(radii), w.T, **kw).cpu().numpy()
    ref = oracle.forward_index(w.coords, w.types, radii, w.T, w.resolution, w.dimension, **okw)
    assert np.isfinite(out).all() and np.isfinite(ref).all()
    assert np.abs(out - ref).max() <= GRID_TOL
    assert out[0].max() > 0.5 and out[1].max() == 0 and out[3].max() == 0    # natoms -3; all atoms non-finite
    assert out[:, 1].max() == 0 and out[:, 2].max() == 0                     # NaN and negative radius
    gmb = mg.GridMaker(w.resolution, w.dimension, binary=True, radius_type_indexed=True)
    outb = gmb.mg_forward_index(dev(w.coords), dev(w.types), dev(radii), w.T, **kw).cpu().numpy()
    refb = oracle.forward_binary(w.coords, radii, w.T, w.resolution, w.dimension, types=w.types, **okw)
    assert np.array_equal(outb.view(np.uint32), refb.view(np.uint32))
    G = np.random.default_rng(3).standard_normal(ref.shape).astype(np.float32)
    g = gm.mg_backward_index(dev(w.coords), dev(w.types), dev(radii), w.T, dev(G), **kw).cpu().numpy()
    rg = oracle.backward_index(w.coords, w.types, radii, w.T, w.resolution, w.dimension, G, **okw)
    assert np.isfinite(g).all()
    assert grad_err(g[:1], rg[:1]) <= GRAD_RTOL and grad_err(g[2:3], rg[2:3]) <= GRAD_RTOL
    assert (g[1] == 0).all() and (g[3] == 0).all() and (g[0, 3:8] == 0).all()
    # vector types: the same atoms, weights instead of types
    rng = np.random.default_rng(4)
    wts = rng.dirichlet(0.5 * np.ones(w.T), (w.B, w.N)).astype(np.float32)
    outv = gm.mg_forward_vector(dev(w.coords), dev(wts), dev(radii), **kw).cpu().numpy()
    refv = oracle.forward_vector(w.coords, wts, radii, w.resolution, w.dimension, **okw)
    assert np.isfinite(outv).all() and np.abs(outv - refv).max() <= GRID_TOL
    gc, gw = gm.mg_backward_vector(dev(w.coords), dev(wts), dev(radii), dev(G), **kw)
    rc, rw = oracle.backward_vector(w.coords, wts, radii, w.resolution, w.dimension, G, **okw)
    gc, gw = gc.cpu().numpy(), gw.cpu().numpy()
    assert np.isfinite(gc).all() and np.isfinite(gw).all()
    for b in (0, 2):
        assert np.abs(gc[b] - rc[b]).max() <= GRAD_RTOL * np.abs(rc[b]).max()
        assert np.abs(gw[b] - rw[b]).max() <= GRAD_RTOL * np.abs(rw[b]).max()
    assert (gc[1] == 0).all() and (gw[3] == 0).all() and (gw[:, :, 1:3] == 0).all()
