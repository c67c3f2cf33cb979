"""Compile the HIP library for gfx950 (in-tree: paper_1708_08917_amd/libcirc.so)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcirc.so")
SOURCES = [os.path.join(HERE, "csrc", "circ_api.hip")]
# measurement helpers of bench.py (launch and memory floors); no layer arithmetic
FLOOR_LIB_PATH = os.path.join(HERE, "libcirc_floor.so")
FLOOR_SOURCES = [os.path.join(HERE, "csrc", "circ_floor.hip")]
FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 VALU forms are not used on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-pass-failed",
    # the first 16 dwords of kernel arguments arrive in scalar registers with the wave instead of
    # being fetched by its first instructions (gfx950 supports this; it takes a dependent memory
    # round trip off the start of every kernel: 0.3 us on the fused FC kernel)
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
]


def _compile(out: str, sources, verbose: bool) -> None:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, "-o", out, *sources]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build_lib(verbose: bool = True) -> str:
    _compile(LIB_PATH, SOURCES, verbose)
    _compile(FLOOR_LIB_PATH, FLOOR_SOURCES, verbose)
    return LIB_PATH


if __name__ == "__main__":
    build_lib()
