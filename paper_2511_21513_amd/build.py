"""Builds libintattn.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libintattn.so")
SOURCES = ["api.cpp", "fwd_kernel.hip", "sweep_ab.hip", "sweep_c.hip", "quantonly_kernel.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-fp32 instructions
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",  # MFMA accumulators in VGPRs: no accvgpr copies around the ALU stage
    "-fvisibility=hidden", "-Wall", "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False, extra=()) -> str:
    srcs = []
    for s in SOURCES:
        path = os.path.join(CSRC, s)
        srcs += (["-x", "hip", path] if s.endswith(".cpp") else ["-x", "hip", path])
    cmd = [HIPCC, *FLAGS, *extra, *srcs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
    print(LIB)
