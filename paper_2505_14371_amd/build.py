"""Compile the HIP sources under csrc/ for gfx950 into libqoda.so next to this file."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = [os.path.join(_HERE, "csrc", f) for f in ("qoda_kernels.hip", "qoda_api.hip")]
LIB = os.path.join(_HERE, "libqoda.so")
PROBE_SRC = os.path.join(_HERE, "harness", "qoda_probe.hip")
PROBE = os.path.join(_HERE, "harness", "qoda_probe")

# -ffp-contract=off: every fp32/fp64 operation that feeds a packed bit stays a single IEEE operation.
# packed-fp32 instructions are switched off for the whole library.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall"]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *SOURCES, "-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    # the torch-free measurement driver (links the library through its C ABI only)
    cmd = [hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", PROBE_SRC, "-o", PROBE, "-L" + _HERE, "-lqoda",
           "-Wl,-rpath,$ORIGIN/.."]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
