"""The library's calls are kernel launches on the caller's stream and nothing else (no
allocation, no memset, no synchronisation), so a caller can capture them in a HIP graph: a
launch-bound loop (the tiny configuration: a few microseconds of GPU work per call) then costs
one graph launch per step.  Each replay is checked against the eager result and the oracle, with
eager work and synchronisations between the replays and new coordinates written into the
captured input buffer."""
import numpy as np
import pytest

import oracle
from paper_1912_04822_amd import workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from test_gpu_parity import GRID_TOL, GRAD_RTOL, dev, mg  # noqa: E402,F401


def test_forward_and_backward_replayed_from_a_graph(mg):
    w = workloads.tiny()
    gm = mg.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    rng = np.random.default_rng(21)
    coords, types, radii = dev(w.coords), dev(w.types), dev(w.radii)
    G = dev(rng.standard_normal(w.out_shape).astype(np.float32))
    out = torch.empty(w.out_shape, dtype=torch.float32, device="cuda")
    grad = torch.empty((w.B, w.N, 3), dtype=torch.float32, device="cuda")
    ws = torch.empty(gm.workspace_bytes(w.B, w.N, w.T), dtype=torch.uint8, device="cuda")

    def step():
        gm.mg_forward_index(coords, types, radii, w.T, out=out, workspace=ws)
        gm.mg_backward_index(coords, types, radii, w.T, G, grad_coords=grad, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for k in range(4):
        moved = (w.coords + rng.normal(0, 0.3, w.coords.shape)).astype(np.float32)
        coords.copy_(dev(moved))                # new input in the captured buffer
        out.fill_(-1.0)
        grad.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got, got_g = out.cpu().numpy(), grad.cpu().numpy()
        step()                                  # the same step, eagerly
        torch.cuda.synchronize()
        assert np.array_equal(got, out.cpu().numpy()), k
        assert np.array_equal(got_g, grad.cpu().numpy()), k
        ref = oracle.forward_index(moved, w.types, w.radii, w.T, w.resolution, w.dimension)
        assert np.abs(got - ref).max() <= GRID_TOL, k
        rg = oracle.backward_index(moved, w.types, w.radii, w.T, w.resolution, w.dimension,
                                   G.cpu().numpy())
        assert np.abs(got_g - rg).max() <= GRAD_RTOL * np.abs(rg).max(), k
