#!/usr/bin/env python3
"""Benchmark of the atom-to-grid hot path on one MI355X.

A step is one ``mg_forward_index`` call (transform + cull/bin + forward gather)
on the protein-ligand batch (B=50, N=2040, T=28, 48^3 points at 0.5 A, a random
rotation and translation per example), inputs resident in HBM.  The other rows
of the path (vector types, binary, backward) are timed on the same geometry and
reported under "rows".  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu] [--rows]
    python bench.py --copy-calibration   # plain copy kernel of known size, for counter scaling
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X published HBM3E peak
FP32_VECTOR_PEAK_TFLOPS = 157.3


def hip_runtime():
    for name in ("libamdhip64.so", "/opt/rocm/lib/libamdhip64.so"):
        try:
            return ctypes.CDLL(name)
        except OSError:
            continue
    raise RuntimeError("libamdhip64.so not found")


class Events:
    """hipEvent_t pairs for timing one kernel per step on the launch stream."""

    def __init__(self, n):
        self.hip = hip_runtime()
        self.hip.hipEventCreateWithFlags.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p,
                                                 ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.pairs = []
        for _ in range(n):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert self.hip.hipEventCreateWithFlags(ctypes.byref(a), EVENT_FLAGS) == 0
            assert self.hip.hipEventCreateWithFlags(ctypes.byref(b), EVENT_FLAGS) == 0
            self.pairs.append((a, b))

    def elapsed_ms(self):
        out = []
        for a, b in self.pairs:
            ms = ctypes.c_float()
            rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
            assert rc == 0, rc
            out.append(ms.value)
        return out

    def close(self):
        for a, b in self.pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(b)


def stored_traffic(kernel_tag):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, or None."""
    path = os.path.join(ROOT, "profiles", "%s_pmc.md" % kernel_tag)
    if not os.path.exists(path):
        return None
    m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read())
    return float(m.group(1)) if m else None


# hipEventDisableSystemFence: the events only time a kernel, so they need no system-scope fence
# (cache write-back and invalidation) when they complete; with the default flags that fence is
# charged to the timed kernel (+1.4 us) and to the step that carries the pair.
EVENT_FLAGS = 0x20000000
EVENT_EVERY = 5     # a step in five carries kernel timing events (a pair costs its step a few us)


def time_call(torch, molgrid, fn, steps, warmup):
    """Whole-call wall time over `steps` back-to-back calls and the main kernel's duration,
    sampled inside that same timed region: every EVENT_EVERY-th step hands the library a pair
    of HIP events that it attaches to the kernel's own dispatch on the launch stream."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = Events((steps + EVENT_EVERY - 1) // EVENT_EVERY)
    t0 = time.perf_counter()
    for i in range(steps):
        if i % EVENT_EVERY == 0:
            a, b = ev.pairs[i // EVENT_EVERY]
            molgrid.mg_time_next_kernel(a.value, b.value)
        fn()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kern = ev.elapsed_ms()
    ev.close()
    time_call.last = kern
    return (t1 - t0) * 1e3 / steps, float(np.mean(kern)), float(np.min(kern))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=150,
                    help="untimed steps first; the chip needs ~10 ms of work (~80 steps) to reach its steady clocks")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--rows", action="store_true", help="also time vector/binary/backward rows")
    ap.add_argument("--tile-floats", type=int, default=None, help="forward kernel tuning knob")
    ap.add_argument("--debug", type=int, default=None, help="forward kernel timing mode (wrong output)")
    ap.add_argument("--prep-stop", type=int, default=None, help="timing aid (wrong output)")
    ap.add_argument("--lds-floor", type=int, default=None, help="forward kernel tuning knob")
    ap.add_argument("--waves-per-tile", type=int, default=None, help="forward kernel tuning knob")
    ap.add_argument("--xcd-run", type=int, default=None, help="forward kernel tuning knob")
    ap.add_argument("--tile-order", type=int, default=None, help="forward kernel tuning knob")
    ap.add_argument("--keep-alive", type=int, default=None, help="forward kernel tuning knob")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain device copy of known size (for scaling rocprofv3 counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path shards by example with no "
              "collective); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)

    if args.copy_calibration:
        n = 619315200 // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": n * 4, "copy_bytes_written": n * 4, "launches": 10}))
        return

    from paper_1912_04822_amd import molgrid, workloads
    molgrid.lib()                       # raises if the HIP library is missing: no fallback
    if args.tile_floats is not None:
        molgrid.set_option("tile_floats", args.tile_floats)
    if args.debug is not None:
        molgrid.set_option("debug", args.debug)
    if args.xcd_run is not None:
        molgrid.set_option("xcd_run", args.xcd_run)
    if args.tile_order is not None:
        molgrid.set_option("tile_order", args.tile_order)
    if args.keep_alive is not None:
        molgrid.set_option("keep_alive", args.keep_alive)
    if args.lds_floor is not None:
        molgrid.set_option("lds_floor", args.lds_floor)
    if args.waves_per_tile is not None:
        molgrid.set_option("waves_per_tile", args.waves_per_tile)
    if args.prep_stop is not None:
        molgrid.set_option("prep_stop", args.prep_stop)

    w = workloads.protein_ligand(B=50, with_weights=args.rows, with_grad=args.rows)
    dev = lambda a, dt=None: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    coords, types, radii = dev(w.coords), dev(w.types), dev(w.radii)
    centers, quats, trans = dev(w.centers), dev(w.quats), dev(w.translations)
    gm = molgrid.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    out = torch.empty(w.out_shape, dtype=torch.float32, device="cuda")
    ws = torch.empty(gm.workspace_bytes(w.B, w.N, w.T), dtype=torch.uint8, device="cuda")

    def step():
        gm.mg_forward_index(coords, types, radii, w.T, centers=centers, quats=quats,
                            translations=trans, out=out, workspace=ws)

    ms_step, ms_kernel, ms_kernel_min = time_call(torch, molgrid, step, args.steps, args.warmup)
    grids_per_s = w.B / (ms_step * 1e-3)
    achieved = w.out_bytes / (ms_kernel * 1e-3) / 1e9
    result = {
        "metric": "voxel grids/sec (B=50, 28ch, 48^3 fp32)",
        "value": grids_per_s,
        "unit": "grids/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "protein-ligand forward (configs[1]): B=50, N=2040 atoms, T=28, "
                               "48^3 points @0.5A, random rotation + <=2A translation per example",
                   "out_bytes": w.out_bytes},
        "roofline": {"bound": "hbm", "kernel": "forward_kernel (index types, real density)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "kernel_ms_avg": ms_kernel, "kernel_ms_min": ms_kernel_min,
                     "kernel_samples": len(time_call.last),
                     "kernel_ms_pct": [float(x) for x in np.percentile(time_call.last, [10, 50, 90])],
                     "whole_call_GBs": w.out_bytes / (ms_step * 1e-3) / 1e9,
                     "traffic": stored_traffic("forward_index_protein_ligand")},
    }

    if args.rows:
        rows = {}
        weights, G = dev(w.weights), dev(w.grad_out)
        gmb = molgrid.GridMaker(w.resolution, w.dimension, binary=True, radius_type_indexed=True)
        gc = torch.empty((w.B, w.N, 3), dtype=torch.float32, device="cuda")
        k = max(5, args.steps // 10)

        def add(name, fn, nbytes, steps):
            ms, mk, mkmin = time_call(torch, molgrid, fn, steps, 3)
            rows[name] = {"ms_per_call": ms, "kernel_ms_avg": mk, "grids_per_s": w.B / (ms * 1e-3),
                          "algorithmic_GBs": nbytes / (mk * 1e-3) / 1e9}

        # for scale: the runtime's memset of the same output buffer (no atoms, no arithmetic)
        hip = hip_runtime()
        hip.hipMemsetAsync.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p]
        stream_h = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

        def memset_out():
            assert hip.hipMemsetAsync(ctypes.c_void_p(out.data_ptr()), 0, w.out_bytes, stream_h) == 0

        for _ in range(20):
            memset_out()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(200):
            memset_out()
        torch.cuda.synchronize()
        ms_memset = (time.perf_counter() - t0) * 1e3 / 200
        rows["memset_same_buffer"] = {"ms_per_call": ms_memset,
                                      "algorithmic_GBs": w.out_bytes / (ms_memset * 1e-3) / 1e9}
        add("forward_binary", lambda: gmb.mg_forward_index(
            coords, types, radii, w.T, centers=centers, quats=quats, translations=trans, out=out,
            workspace=ws), w.out_bytes, args.steps)
        qa = torch.empty((w.B, 4), dtype=torch.float32, device="cuda")
        ta = torch.empty((w.B, 3), dtype=torch.float32, device="cuda")
        counter = [0]

        def augmented():        # transforms drawn on the device, a new draw per call, then forward
            counter[0] += 1
            molgrid.mg_draw_transforms(2024, counter[0], w.B, True, 2.0, qa, ta)
            gm.mg_forward_index(coords, types, radii, w.T, centers=centers, quats=qa,
                                translations=ta, out=out, workspace=ws)

        add("forward_augmented", augmented, w.out_bytes, args.steps)
        out64 = torch.empty(w.out_shape, dtype=torch.float64, device="cuda")
        add("forward_index_f64", lambda: gm.mg_forward_index(
            coords, types, radii, w.T, centers=centers, quats=quats, translations=trans, out=out64,
            workspace=ws), 2 * w.out_bytes, max(20, args.steps // 4))
        del out64
        add("forward_vector", lambda: gm.mg_forward_vector(
            coords, weights, radii, centers=centers, quats=quats, translations=trans, out=out,
            workspace=ws), w.out_bytes, k)
        add("backward_index", lambda: gm.mg_backward_index(
            coords, types, radii, w.T, G, centers=centers, quats=quats, translations=trans,
            grad_coords=gc, workspace=ws), w.out_bytes, args.steps)
        gw = torch.empty((w.B, w.N, w.T), dtype=torch.float32, device="cuda")
        add("backward_vector", lambda: gm.mg_backward_vector(
            coords, weights, radii, G, centers=centers, quats=quats, translations=trans,
            grad_coords=gc, grad_weights=gw, workspace=ws), w.out_bytes, k)
        # one 16-example chunk of the large / high-resolution configuration (96^3 at 0.25 A,
        # 8000 atoms per example); freed first: the chunk's grid is 1.6 GB
        del out, ws, gw, G, weights
        torch.cuda.empty_cache()
        wc = workloads.large_chunk(0)
        gmc = molgrid.GridMaker(wc.resolution, wc.dimension, radius_type_indexed=True)
        outc = torch.empty(wc.out_shape, dtype=torch.float32, device="cuda")
        wsc = torch.empty(gmc.workspace_bytes(wc.B, wc.N, wc.T), dtype=torch.uint8, device="cuda")
        cc, tc, rc = dev(wc.coords), dev(wc.types), dev(wc.radii)
        cec, qc, trc = dev(wc.centers), dev(wc.quats), dev(wc.translations)
        ms, mk, _ = time_call(torch, molgrid, lambda: gmc.mg_forward_index(
            cc, tc, rc, wc.T, centers=cec, quats=qc, translations=trc, out=outc, workspace=wsc),
            max(20, args.steps // 4), 20)
        # the tiny configuration (configs[0]: one example, 100 atoms, 24^3): launch-bound, so a
        # latency in microseconds rather than a bandwidth -- called eagerly, and replayed from a
        # HIP graph that holds the call's two kernel launches
        wt = workloads.tiny()
        gmt = molgrid.GridMaker(wt.resolution, wt.dimension, radius_type_indexed=True)
        outt = torch.empty(wt.out_shape, dtype=torch.float32, device="cuda")
        wst = torch.empty(gmt.workspace_bytes(wt.B, wt.N, wt.T), dtype=torch.uint8, device="cuda")
        ct, tt, rt = dev(wt.coords), dev(wt.types), dev(wt.radii)

        def tiny_call():
            gmt.mg_forward_index(ct, tt, rt, wt.T, out=outt, workspace=wst)

        ms_eager, mk_tiny, _ = time_call(torch, molgrid, tiny_call, 2000, 200)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            tiny_call()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            tiny_call()
        for _ in range(200):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(2000):
            graph.replay()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - t0) * 1e3 / 2000
        rows["forward_tiny"] = {
            "latency_us_eager": ms_eager * 1e3, "latency_us_graph": ms_graph * 1e3,
            "kernel_us": mk_tiny * 1e3,
            "workload": "configs[0]: B=1, N=100, T=4, 24^3 @0.5A (221 KB out): calls back to back"}
        rows["forward_large_chunk"] = {
            "ms_per_call": ms, "kernel_ms_avg": mk, "grids_per_s": wc.B / (ms * 1e-3),
            "algorithmic_GBs": wc.out_bytes / (mk * 1e-3) / 1e9,
            "workload": "configs[4], one chunk: B=16, N=8000, T=28, 96^3 @0.25A"}
        result["rows"] = rows

    if not args.no_cpu:
        import oracle
        times, threads = [], 0
        for _ in range(10):         # about 13 s of CPU time on 16 threads
            t0 = time.perf_counter()
            _, threads = oracle.forward_index(w.coords, w.types, w.radii, w.T, w.resolution,
                                              w.dimension, centers=w.centers, quats=w.quats,
                                              translations=w.translations, return_threads=True)
            times.append(time.perf_counter() - t0)
        best = min(times)
        one = []
        for _ in range(2):          # the same batch on one thread, about 1.5 s each
            t0 = time.perf_counter()
            oracle.forward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension,
                                 centers=w.centers, quats=w.quats, translations=w.translations,
                                 threads=1)
            one.append(time.perf_counter() - t0)
        result["cpu_baseline"] = {
            "value": w.B / best, "unit": "grids/s", "cores": int(threads), "kind": "oracle",
            "one_core_value": w.B / min(one),
            "sample": "all 50 examples of the same batch, cutoff-box variant, OpenMP over "
                      "examples, best of 10 runs (%.2f s each, median %.2f s)"
                      % (best, float(np.median(times)))}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
