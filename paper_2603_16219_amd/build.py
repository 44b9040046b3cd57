"""Compile the HIP library in-tree for gfx950 (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
SOURCES = [os.path.join(_PKG, "csrc", n) for n in ("specsteer.hip", "split.hip")]
INCLUDE = os.path.join(_ROOT, "include")
LIBRARY = os.path.join(_PKG, "libspecsteer.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950",
    # packed-fp32 instructions are switched off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # The logit loads are 16 bytes wide on vector types that promise only element alignment (rows of an odd
    # vocabulary start anywhere).  This states to the compiler what the code relies on -- wide global loads at
    # any element-aligned address are legal on this target (the hardware's unaligned access mode, which the
    # ROCm kernel driver enables) -- instead of leaving it to the toolchain's default for the target.
    "-Xclang", "-target-feature", "-Xclang", "+unaligned-access-mode",
    "-shared", "-fPIC", "-Wl,-rpath,/opt/rocm/lib",
]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", INCLUDE, "-o", LIBRARY, *SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{proc.stdout}\n{proc.stderr}")
    return LIBRARY


if __name__ == "__main__":
    print(build(verbose=True))
