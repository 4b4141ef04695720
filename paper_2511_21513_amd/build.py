"""Builds libintattn.so (the C-ABI library) in-tree with hipcc for gfx950.

Every source is compiled to an object of its own, a few at a time, and the objects are linked into
the shared library; the objects live in `_build/` next to this file (not tracked)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libintattn.so")
SOURCES = ["api.cpp", "fwd_kernel.hip", "fwd_single.hip", "fwd_split.hip", "fwd_splitk.hip", "sweep_c.hip",
           "quantize_kernel.hip", "derive_kernel.hip", "decode_kernel.hip", "softmax_kernel.hip", "quantonly_kernel.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-fp32 instructions
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",  # MFMA accumulators in VGPRs: no accvgpr copies around the ALU stage
    "-fvisibility=hidden", "-Wall", "-Wno-unused-command-line-argument",
]


def _compile(src: str, extra, verbose: bool) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, *extra, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return obj


def build(verbose: bool = False, extra=(), jobs: int | None = None) -> str:
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(len(SOURCES), max(1, min(8, os.cpu_count() or 1)))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(lambda s: _compile(s, list(extra), verbose), SOURCES))
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-fvisibility=hidden", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
    print(LIB)
