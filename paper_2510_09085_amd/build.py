"""Compile the HIP decoder into an in-tree shared library for gfx950 (hipcc cross-compiles)."""
from __future__ import annotations

import glob
import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
LIB_PATH = os.path.join(_PKG, "libfltop_ctc.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",  # keep fp64 score arithmetic as written (no fused multiply-add)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # atomics are aggregated per wavefront by hand where that pays; the compiler's own pass turns
    # every single-lane LDS atomic into a loop over the active lanes (measured: 1-2% per decode)
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = False, out: str = LIB_PATH, defines=()) -> str:
    """Always recompiles; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = sorted(glob.glob(os.path.join(_PKG, "csrc", "*.hip")))
    cmd = [hipcc, *HIPCC_FLAGS, *[f"-D{d}" for d in defines],
           "-I", os.path.join(_ROOT, "include"),
           "-I", os.path.join(_PKG, "csrc"), *srcs, "-o", out]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--define", action="append", default=[],
                    help="preprocessor define, e.g. FLTOP_PHASE_CLOCKS for the profiling build")
    ap.add_argument("--out", default=LIB_PATH, help="path of the shared library to write")
    cli = ap.parse_args()
    print(build(verbose=True, out=cli.out, defines=cli.define))
