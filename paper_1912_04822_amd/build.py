"""Compile the HIP library in-tree for gfx950 (``python -m paper_1912_04822_amd.build``)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmolgrid_hip.so")
# measurement build: the same sources with -DMG_TIMING_AIDS (kernel phases can be switched off
# to time the rest; such runs write wrong grids, so the release library has none of it)
LIB_TIMING = os.path.join(HERE, "libmolgrid_hip_timing.so")

# -ffp-contract=off: nothing is fused behind the code's back (the binary-mode
# predicate and the double-precision transform are specified operation by
# operation); fused multiply-adds are written as fmaf where wanted.
# packed FP32 instructions are switched off for the device code.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_library(verbose: bool = False, timing_aids: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = LIB_TIMING if timing_aids else LIB
    cmd = [hipcc] + HIPCC_FLAGS + (["-DMG_TIMING_AIDS"] if timing_aids else []) + ["-o", out] + sources()
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                     if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + msgs)
    if verbose and msgs.strip():
        print(msgs)
    return out


if __name__ == "__main__":
    print(build_library(verbose=True, timing_aids="--timing-aids" in sys.argv[1:]))
    sys.exit(0)
