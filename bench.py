#!/usr/bin/env python3
"""Benchmark of the atom-to-grid hot path on one MI355X.

A step is one ``mg_forward_index`` call (transform + cull/bin + forward gather)
on the protein-ligand batch (B=50, N=2040, T=28, 48^3 points at 0.5 A, a random
rotation and translation per example), inputs resident in HBM.  Prints ONE JSON
line.

Order of a run:
  1. clock settling (disclosed as "settle"): the same call is repeated until at
     least 30 ms of GPU time has passed -- a chip that has just been idle runs its
     first ~10 ms of work at lower clocks, whatever the kernel;
  2. --warmup untimed steps, then exactly --steps timed steps between two
     synchronisations.  Every timed step (one in five beyond 100 steps) carries a
     pair of HIP events that the library attaches to the dispatch of the forward
     kernel itself, on the launch stream: the roofline figure is the algorithmic
     bytes of one launch over the mean of those durations;
  3. the other rows of the path on the same geometry ("rows": binary, vector types,
     backward, forward + backward of one training step, one 16-example chunk of the
     96^3 configuration, the tiny configuration's latency, a memset of the same
     buffer for scale), each with its own short settling phase and roofline;
  4. the CPU oracle on the same batch ("cpu_baseline").

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu] [--no-rows]
    python bench.py --copy-calibration   # plain copy kernel of known size, for counter scaling
    python bench.py --timing-aids --debug 3   # measurement build of the library (wrong grids)
"""
from __future__ import annotations

import argparse
import ctypes
import glob
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X published HBM3E peak
# 256 CUs x 4 SIMDs x 2.4 GHz, one 64-lane vector instruction per SIMD every 4 cycles, packed
# FP32 switched off: 1024 x 2.4e9 / 4 x 64 lanes = 39.3e12 lane-instructions per second (the data
# sheet's 157.3 TFLOP/s counts packed FMAs: two results per lane, two flops each)
VALU_PEAK_TLANE = 39.3
SETTLE_GPU_MS = 30.0


def hip_runtime():
    for name in ("libamdhip64.so", "/opt/rocm/lib/libamdhip64.so"):
        try:
            return ctypes.CDLL(name)
        except OSError:
            continue
    raise RuntimeError("libamdhip64.so not found")


# hipEventDisableSystemFence: the events only time a kernel, so they need no system-scope fence
# (cache write-back and invalidation) when they complete; with the default flags that fence is
# charged to the timed kernel and to the step that carries the pair.
EVENT_FLAGS = 0x20000000


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


def stored(key):
    """A figure kept in a committed rocprofv3 summary under profiles/ (a line ``key: value``),
    or None.  Counter values are NOT measured by this run; they are labelled as stored."""
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        m = re.search(r"^%s:\s*([0-9.eE+]+)\s*$" % re.escape(key), open(path).read(), re.M)
        if m:
            return float(m.group(1)), os.path.relpath(path, ROOT)
    return None, None


def settle(torch, fn, min_gpu_ms=SETTLE_GPU_MS, batch=20, max_gpu_ms=250.0):
    """Repeat fn until at least min_gpu_ms of GPU time (events on the launch stream) has passed
    AND two batches in a row took within 1 % of the batch before them (the clocks have stopped
    moving), or max_gpu_ms has passed."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    total, calls, prev, steady = 0.0, 0, None, 0
    while calls < 200000:
        e0.record()
        for _ in range(batch):
            fn()
        e1.record()
        e1.synchronize()
        t = e0.elapsed_time(e1)
        total += t
        calls += batch
        steady = steady + 1 if (prev is not None and abs(t - prev) <= 0.01 * prev) else 0
        prev = t
        if (total >= min_gpu_ms and steady >= 2) or total >= max(max_gpu_ms, min_gpu_ms):
            break
    return {"ms": total, "calls": calls, "last_batch_ms_per_call": prev / batch}


def time_call(torch, molgrid, fn, steps, warmup, timed_kernel=True):
    """Wall time per call over `steps` back-to-back calls, and the main kernel's duration sampled
    inside that same timed region (every step up to 100 steps, else one step in five)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    every = 1 if steps <= 100 else 5
    ev = Events((steps + every - 1) // every) if timed_kernel else None
    t0 = time.perf_counter()
    for i in range(steps):
        if ev is not None and i % every == 0:
            a, b = ev.pairs[i // every]
            molgrid.mg_time_next_kernel(a.value, b.value)
        fn()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    res = {"ms_per_call": (t1 - t0) * 1e3 / steps}
    if ev is not None:
        kern = ev.elapsed_ms()
        ev.close()
        res.update(kernel_ms_avg=float(np.mean(kern)), kernel_ms_min=float(np.min(kern)),
                   kernel_ms_median=float(np.median(kern)), kernel_samples=len(kern),
                   kernel_ms_pct=[float(x) for x in np.percentile(kern, [10, 50, 90])])
    return res


def hbm_roofline(nbytes, kernel_ms, what):
    gbs = nbytes / (kernel_ms * 1e-3) / 1e9
    return {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": gbs / HBM_PEAK_GBS, "algorithmic_bytes": int(nbytes), "bytes_are": what}


def alu_roofline(valu_key, kernel_ms):
    insts, src = stored(valu_key)
    if insts is None:
        return {"bound": "alu", "achieved": None, "peak": VALU_PEAK_TLANE,
                "unit": "T lane-instructions/s", "frac": None}
    rate = insts * 64 / (kernel_ms * 1e-3) / 1e12
    return {"bound": "alu", "achieved": rate, "peak": VALU_PEAK_TLANE,
            "unit": "T lane-instructions/s", "frac": rate / VALU_PEAK_TLANE,
            "valu_insts_per_launch": insts,
            "valu_insts_source": "%s (SQ_INSTS_VALU, stored from that profile, not measured in this run)" % src}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10,
                    help="untimed steps after the clock-settling phase")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-rows", action="store_true", help="only the headline forward call")
    ap.add_argument("--rows", action="store_true", help="(default now; kept for old command lines)")
    ap.add_argument("--settle-ms", type=float, default=SETTLE_GPU_MS,
                    help="GPU time of the clock-settling phase before the counted warm-up")
    ap.add_argument("--tile-floats", type=int, default=None, help="forward kernel launch knob")
    ap.add_argument("--lds-floor", type=int, default=None, help="forward kernel launch knob")
    ap.add_argument("--waves-per-tile", type=int, default=None, help="forward kernel launch knob")
    ap.add_argument("--xcd-run", type=int, default=None, help="forward kernel launch knob")
    ap.add_argument("--tile-order", type=int, default=None, help="forward kernel launch knob")
    ap.add_argument("--keep-alive", type=int, default=None, help="forward kernel launch knob")
    ap.add_argument("--keep-alive-stride", type=int, default=None, help="forward kernel launch knob")
    ap.add_argument("--timing-aids", action="store_true",
                    help="load the measurement build (python -m paper_1912_04822_amd.build --timing-aids)")
    ap.add_argument("--debug", type=int, default=None, help="timing aid (measurement build; wrong output)")
    ap.add_argument("--prep-stop", type=int, default=None, help="timing aid (measurement build; wrong output)")
    ap.add_argument("--lib", default=None, help="path of another build of libmolgrid_hip.so to load")
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

    from paper_1912_04822_amd import build as hip_build
    from paper_1912_04822_amd import molgrid, workloads
    aids = args.timing_aids or args.debug is not None or args.prep_stop is not None
    molgrid.lib(args.lib or (hip_build.LIB_TIMING if aids else None))   # raises if the library is missing: no fallback
    for key, val in (("tile_floats", args.tile_floats), ("xcd_run", args.xcd_run),
                     ("tile_order", args.tile_order), ("keep_alive", args.keep_alive),
                     ("lds_floor", args.lds_floor), ("keep_alive_stride", args.keep_alive_stride), ("waves_per_tile", args.waves_per_tile),
                     ("debug", args.debug), ("prep_stop", args.prep_stop)):
        if val is not None:
            molgrid.set_option(key, val)
    rows_on = not args.no_rows and not aids

    w = workloads.protein_ligand(B=50, with_weights=rows_on, with_grad=rows_on)
    dev = lambda a, dt=None: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    coords, types, radii = dev(w.coords), dev(w.types), dev(w.radii)
    centers, quats, trans = dev(w.centers), dev(w.quats), dev(w.translations)
    gm = molgrid.GridMaker(w.resolution, w.dimension, radius_type_indexed=True)
    out = torch.empty(w.out_shape, dtype=torch.float32, device="cuda")
    ws = torch.empty(gm.workspace_bytes(w.B, w.N, w.T), dtype=torch.uint8, device="cuda")

    def step():
        gm.mg_forward_index(coords, types, radii, w.T, centers=centers, quats=quats,
                            translations=trans, out=out, workspace=ws)

    settled = settle(torch, step, args.settle_ms)
    main_t = time_call(torch, molgrid, step, args.steps, args.warmup, timed_kernel=args.prep_stop is None)
    ms_step = main_t["ms_per_call"]
    ms_kernel = main_t.get("kernel_ms_avg", float("nan"))
    distinct_index = int(torch.count_nonzero(out))      # voxels within the cutoff of an atom of their channel
    traffic, traffic_src = stored("traffic_bytes_per_launch")
    roof = hbm_roofline(w.out_bytes, ms_kernel, "one 4-byte store per output element")
    roof.update({"kernel": "forward_kernel (index types, real density)",
                 "kernel_ms_avg": ms_kernel, "kernel_ms_min": main_t.get("kernel_ms_min"),
                 "kernel_ms_median": main_t.get("kernel_ms_median"),
                 "kernel_samples": main_t.get("kernel_samples"),
                 "kernel_ms_pct": main_t.get("kernel_ms_pct"),
                 "whole_call_GBs": w.out_bytes / (ms_step * 1e-3) / 1e9,
                 "whole_call_frac": w.out_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                 "traffic": traffic,
                 "traffic_source": None if traffic is None else
                 "%s (FETCH_SIZE + WRITE_SIZE per launch, stored from that profile, not measured in this run)"
                 % traffic_src})
    result = {
        "metric": "voxel grids/sec (B=50, 28ch, 48^3 fp32)",
        "value": w.B / (ms_step * 1e-3),
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
        "settle": dict(settled, what="the same forward call repeated, untimed, before the counted "
                                     "warm-up: at least %.0f ms of GPU time and until two batches of "
                                     "20 calls in a row took within 1 %% of the batch before them "
                                     "(at most 250 ms)" % args.settle_ms),
        "roofline": roof,
    }

    if rows_on:
        rows = {}
        weights, G = dev(w.weights), dev(w.grad_out)
        gmb = molgrid.GridMaker(w.resolution, w.dimension, binary=True, radius_type_indexed=True)
        gc = torch.empty((w.B, w.N, 3), dtype=torch.float32, device="cuda")
        n_fast = max(20, min(args.steps, 100))      # calls of ~0.1 ms
        n_slow = max(10, min(args.steps, 30))       # calls of ~1 ms

        def row(fn, steps, settle_ms=10.0, **kw):
            settle(torch, fn, settle_ms, batch=5, max_gpu_ms=60.0)
            return time_call(torch, molgrid, fn, steps, 3, **kw)

        # for scale: the runtime's memset of the same output buffer (no atoms, no arithmetic)
        hip = hip_runtime()
        hip.hipMemsetAsync.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p]
        stream_h = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

        def memset_out():
            assert hip.hipMemsetAsync(ctypes.c_void_p(out.data_ptr()), 0, w.out_bytes, stream_h) == 0

        r = row(memset_out, n_fast, timed_kernel=False)
        rows["memset_same_buffer"] = {"ms_per_call": r["ms_per_call"],
                                      "roofline": hbm_roofline(w.out_bytes, r["ms_per_call"],
                                                               "the buffer's size (wall time per call)")}

        def fwd_row(name, fn, steps, nbytes, B):
            r = row(fn, steps)
            r["grids_per_s"] = B / (r["ms_per_call"] * 1e-3)
            r["roofline"] = hbm_roofline(nbytes, r["kernel_ms_avg"], "one store per output element")
            rows[name] = r
            return r

        fwd_row("forward_binary", lambda: gmb.mg_forward_index(
            coords, types, radii, w.T, centers=centers, quats=quats, translations=trans, out=out,
            workspace=ws), n_fast, w.out_bytes, w.B)
        qa = torch.empty((w.B, 4), dtype=torch.float32, device="cuda")
        ta = torch.empty((w.B, 3), dtype=torch.float32, device="cuda")
        counter = [0]

        def augmented():        # transforms drawn on the device, a new draw per call, then forward
            counter[0] += 1
            molgrid.mg_draw_transforms(2024, counter[0], w.B, True, 2.0, qa, ta)
            gm.mg_forward_index(coords, types, radii, w.T, centers=centers, quats=qa,
                                translations=ta, out=out, workspace=ws)

        fwd_row("forward_augmented", augmented, n_fast, w.out_bytes, w.B)
        fwd_row("forward_index_static_workspace", lambda: gm.mg_forward_index_static(
            coords, types, radii, w.T, out, centers=centers, quats=quats, translations=trans),
            n_fast, w.out_bytes, w.B)
        out64 = torch.empty(w.out_shape, dtype=torch.float64, device="cuda")
        fwd_row("forward_index_f64", lambda: gm.mg_forward_index(
            coords, types, radii, w.T, centers=centers, quats=quats, translations=trans, out=out64,
            workspace=ws), n_slow, 2 * w.out_bytes, w.B)
        del out64

        # vector types: every atom feeds all 28 channels -- bound by vector arithmetic, so the
        # roofline is instruction issue (instruction count stored from the profile), with the HBM
        # fraction beside it
        r = row(lambda: gm.mg_forward_vector(
            coords, weights, radii, centers=centers, quats=quats, translations=trans, out=out,
            workspace=ws), n_slow)
        r["grids_per_s"] = w.B / (r["ms_per_call"] * 1e-3)
        r["roofline"] = alu_roofline("forward_vector_valu_insts_per_launch", r["kernel_ms_avg"])
        r["hbm_frac"] = w.out_bytes / (r["kernel_ms_avg"] * 1e-3) / 1e9 / HBM_PEAK_GBS
        rows["forward_vector"] = r
        distinct_vector = int(torch.count_nonzero(out))

        # backward: the algorithmic bytes are the distinct upstream-gradient voxels that lie within
        # the cutoff of an atom of their channel (counted above as the nonzeros of the forward
        # grid of the same inputs -- a density is positive exactly there), 4 bytes each; the bytes
        # the 128-byte lines of those voxels occupy (FETCH_SIZE of the profile) give the practical
        # bound, streaming the whole gradient grid once the trivial one
        def kernel_after_forward(fn, n):
            """The backward kernel's duration when a forward call (619 MB of stores) ran just
            before it, as in a training step: the gradient grid comes from HBM and the last part
            of the forward's stores still sits dirty in the 256 MB memory-side cache."""
            ev = Events(n)
            for i in range(3 + n):
                step()
                if i >= 3:
                    a, b = ev.pairs[i - 3]
                    molgrid.mg_time_next_kernel(a.value, b.value)
                fn()
            torch.cuda.synchronize()
            k = ev.elapsed_ms()
            ev.close()
            return float(np.mean(k)), float(np.min(k))

        def kernel_after_read(fn, n):
            """The backward kernel's duration when the caches were emptied WITHOUT leaving dirty
            lines behind: a read-only pass over another 619 MB buffer (the forward grid) runs
            before every timed call.  The gradient grid then comes from HBM and nothing else
            competes for it -- what a training step sees when the network's own kernels, not
            619 MB of fresh stores, ran since the forward pass."""
            ev = Events(n)
            for i in range(3 + n):
                torch.max(out)           # one reduction kernel: reads 619 MB, writes a few bytes
                if i >= 3:
                    a, b = ev.pairs[i - 3]
                    molgrid.mg_time_next_kernel(a.value, b.value)
                fn()
            torch.cuda.synchronize()
            k = ev.elapsed_ms()
            ev.close()
            return float(np.mean(k)), float(np.min(k))

        def bwd_row(name, fn, steps, distinct, fetch_key, valu_key):
            r = row(fn, steps)
            warm = r["kernel_ms_avg"]
            k, kmin = kernel_after_forward(fn, min(steps, 30))
            r["kernel_ms_after_forward"] = k
            r["kernel_ms_after_forward_min"] = kmin
            kc, kcmin = kernel_after_read(fn, min(steps, 30))
            r["kernel_ms_after_read_of_another_buffer"] = kc
            r["kernel_ms_after_read_of_another_buffer_min"] = kcmin
            r["kernel_ms_avg_is"] = "back-to-back backward calls"
            r["atoms_per_s"] = w.B * w.N / (r["ms_per_call"] * 1e-3)
            r["roofline"] = hbm_roofline(4 * distinct, kc, "distinct in-cutoff voxels of the upstream "
                                                           "gradient x 4 B (HBM read); kernel timed "
                                                           "after a read-only pass over another 619 MB "
                                                           "buffer: gradient grid from HBM, no dirty "
                                                           "lines of an earlier kernel being written "
                                                           "back meanwhile")
            r["roofline"]["back_to_back_frac"] = 4 * distinct / (warm * 1e-3) / 1e9 / HBM_PEAK_GBS
            r["roofline"]["after_forward_frac"] = 4 * distinct / (k * 1e-3) / 1e9 / HBM_PEAK_GBS
            r["roofline"]["after_forward_is"] = (
                "the kernel timed right after a forward call, whose last ~256 MB of stores are "
                "still dirty in the memory-side cache (a read-only probe of the same 270 MB of "
                "lines takes 45 us after a read pass and 90-97 us after a 619 MB fill; the "
                "index-type kernel's loads carry the non-temporal hint so that they do not push "
                "those lines out: 74 us, 100 us without the hint)")
            fetch, src = stored(fetch_key)
            lines, lsrc = stored(fetch_key.replace("fetch_bytes", "distinct_line_bytes"))
            if fetch is not None:
                r["roofline"]["traffic"] = fetch
                r["roofline"]["traffic_source"] = (
                    "%s (FETCH_SIZE x 2.00 per launch, stored from that profile, not measured in "
                    "this run)" % src)
            bound = lines if lines is not None else fetch
            if bound is not None:
                r["roofline"]["line_bound"] = {
                    "bytes": bound, "frac": bound / (kc * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "what": ("the distinct 128-byte lines those voxels lie in, counted on the host (%s)"
                             % lsrc) if lines is not None else
                            "the bytes the kernel fetches (see traffic): its distinct lines were not counted"}
            r["roofline"]["stream_whole_grid_frac"] = w.out_bytes / (kc * 1e-3) / 1e9 / HBM_PEAK_GBS
            r["alu"] = alu_roofline(valu_key, warm)
            rows[name] = r
            return r

        bwd_row("backward_index", lambda: gm.mg_backward_index(
            coords, types, radii, w.T, G, centers=centers, quats=quats, translations=trans,
            grad_coords=gc, workspace=ws), n_fast, distinct_index,
            "backward_index_fetch_bytes_per_launch", "backward_index_valu_insts_per_launch")
        gw = torch.empty((w.B, w.N, w.T), dtype=torch.float32, device="cuda")
        bwd_row("backward_vector", lambda: gm.mg_backward_vector(
            coords, weights, radii, G, centers=centers, quats=quats, translations=trans,
            grad_coords=gc, grad_weights=gw, workspace=ws), n_slow, distinct_vector,
            "backward_vector_fetch_bytes_per_launch", "backward_vector_valu_insts_per_launch")

        # forward + backward of one training step on the same inputs
        def train_step():
            gm.mg_forward_index(coords, types, radii, w.T, centers=centers, quats=quats,
                                translations=trans, out=out, workspace=ws)
            gm.mg_backward_index(coords, types, radii, w.T, G, centers=centers, quats=quats,
                                 translations=trans, grad_coords=gc, workspace=ws)

        r = row(train_step, n_fast, timed_kernel=False)

        def train_step_prepared():      # the tables built once, both passes on them
            gm.mg_prepare(coords, types, radii, w.T, centers=centers, quats=quats,
                          translations=trans, workspace=ws)
            gm.mg_forward_index_prepared(w.B, w.N, w.T, ws, out=out)
            gm.mg_backward_index_prepared(w.B, w.N, w.T, G, ws, grad_coords=gc)

        r2 = row(train_step_prepared, n_fast, timed_kernel=False)
        rows["forward_plus_backward_index"] = {
            "ms_per_step": r["ms_per_call"],
            "ms_per_step_prepared": r2["ms_per_call"],
            "what": "mg_forward_index then mg_backward_index on the same inputs and workspace; "
                    "prepared: mg_prepare once, then mg_forward_index_prepared and "
                    "mg_backward_index_prepared on its tables"}

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
        r = fwd_row("forward_large_chunk", lambda: gmc.mg_forward_index(
            cc, tc, rc, wc.T, centers=cec, quats=qc, translations=trc, out=outc, workspace=wsc),
            n_slow, wc.out_bytes, wc.B)
        r["workload"] = "configs[4], one chunk: B=16, N=8000, T=28, 96^3 @0.25A"
        del outc

        # the tiny configuration (configs[0]: one example, 100 atoms, 24^3): launch-bound, so a
        # latency in microseconds and no roofline fraction (221 KB would take 0.03 us at the HBM
        # peak) -- called eagerly, and replayed from a HIP graph that holds the call's launches
        wt = workloads.tiny()
        gmt = molgrid.GridMaker(wt.resolution, wt.dimension, radius_type_indexed=True)
        outt = torch.empty(wt.out_shape, dtype=torch.float32, device="cuda")
        wst = torch.empty(gmt.workspace_bytes(wt.B, wt.N, wt.T), dtype=torch.uint8, device="cuda")
        ct, tt, rt = dev(wt.coords), dev(wt.types), dev(wt.radii)

        def tiny_call():
            gmt.mg_forward_index(ct, tt, rt, wt.T, out=outt, workspace=wst)

        r = row(tiny_call, 1000, settle_ms=5.0, timed_kernel=False)
        # the same call straight through the C ABI with its arguments marshalled once: what the
        # library and the HIP runtime cost per call, without the Python binding's checks
        L = molgrid.lib()
        vp = ctypes.c_void_p
        raw_args = (gmt._h, wt.B, wt.N, wt.T, vp(ct.data_ptr()), vp(tt.data_ptr()), vp(rt.data_ptr()),
                    None, None, None, None, vp(outt.data_ptr()), vp(wst.data_ptr()), wst.numel(),
                    vp(torch.cuda.current_stream().cuda_stream))

        def tiny_raw():
            L.mg_forward_index(*raw_args)

        r_raw = row(tiny_raw, 2000, settle_ms=2.0, timed_kernel=False)
        molgrid.set_option("single_launch", 0)      # for comparison: prep kernel + forward kernel
        r2 = row(tiny_call, 1000, settle_ms=2.0, timed_kernel=False)
        molgrid.set_option("single_launch", 1)
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
        for _ in range(1000):
            graph.replay()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - t0) * 1e3 / 1000
        rows["forward_tiny"] = {
            "latency_us_eager": r["ms_per_call"] * 1e3, "latency_us_graph": ms_graph * 1e3,
            "latency_us_eager_two_launches": r2["ms_per_call"] * 1e3,
            "latency_us_c_abi": r_raw["ms_per_call"] * 1e3,
            "roofline": None,
            "workload": "configs[0]: B=1, N=100, T=4, 24^3 @0.5A (221 KB out): calls back to back, "
                        "one kernel launch per call (every tile looks at the 100 atoms itself); "
                        "launch-bound, so a latency and no roofline fraction"}
        result["rows"] = rows
        result["distinct_in_cutoff_voxels"] = {"index_types": distinct_index,
                                               "vector_types": distinct_vector,
                                               "counted": "nonzeros of the forward grid of the same inputs"}

    if not args.no_cpu:
        import oracle
        times, threads = [], 0
        t_leg = time.perf_counter()
        while time.perf_counter() - t_leg < 10.0 or len(times) < 3:     # about 10 s of wall time
            t0 = time.perf_counter()
            ref, threads = oracle.forward_index(w.coords, w.types, w.radii, w.T, w.resolution,
                                                w.dimension, centers=w.centers, quats=w.quats,
                                                translations=w.translations, return_threads=True)
            times.append(time.perf_counter() - t0)
        best = min(times)
        distinct_oracle = int(np.count_nonzero(ref))
        del ref
        one = []
        for _ in range(2):          # the same batch on one thread
            t0 = time.perf_counter()
            oracle.forward_index(w.coords, w.types, w.radii, w.T, w.resolution, w.dimension,
                                 centers=w.centers, quats=w.quats, translations=w.translations,
                                 threads=1)
            one.append(time.perf_counter() - t0)
        result["cpu_baseline"] = {
            "value": w.B / best, "unit": "grids/s", "cores": int(threads), "kind": "oracle",
            "one_core_value": w.B / min(one),
            "sample": "all 50 examples of the same batch, cutoff-box variant, OpenMP over "
                      "examples, best of %d runs in %.0f s (%.3f s each, median %.3f s)"
                      % (len(times), sum(times), best, float(np.median(times))),
            # (the GPU grid has slightly fewer nonzeros: it accumulates in steps of 2^-24, so a
            # density below 3e-8 at the very edge of a cutoff sphere is stored as zero)
            "distinct_in_cutoff_voxels": distinct_oracle}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
