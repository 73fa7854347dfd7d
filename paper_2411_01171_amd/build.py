"""Builds the HIP library (libsi.so) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libsi.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instruction forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the fused kernels rely on full unrolling so that every register array keeps constant indices
    "-mllvm", "-pragma-unroll-threshold=262144",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
]


def build_library(verbose: bool = False) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    src = os.path.join(CSRC, "si_api.hip")
    cmd = [hipcc, *HIPCC_FLAGS, src, "-o", LIB_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    lines = [l for l in (res.stdout + res.stderr).splitlines()
             if "is not a recognized feature for this target" not in l]
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(lines))
    if verbose and lines:
        print("\n".join(lines))
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
