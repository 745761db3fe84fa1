"""Build libhire.so (HIP, gfx950) in-tree with hipcc.

The library is cross-compiled: no GPU is needed to build it.  Packed-fp32
instruction selection is switched off and floating-point contraction is off,
so every fp32/fp64 operation in the kernels is the one written in the source.
"""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhire.so")
LIB_TS = os.path.join(HERE, "libhire_ts.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False, timestamps: bool = False) -> str:
    """Compile every HIP source into libhire.so; always recompiles.  timestamps=True builds the profiling
    variant libhire_ts.so instead (phase stamps inside the selecting kernels; load it with HIRE_LIB=<path>)."""
    out = LIB_TS if timestamps else LIB
    cmd = [HIPCC, *FLAGS, *(["-DHIRE_TIMESTAMPS"] if timestamps else []), "-o", out, *sources()]
    if verbose:
        print(" ".join(cmd))
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{err}")
    if verbose and err.strip():
        print(err)
    return out


if __name__ == "__main__":
    import sys
    print(build(verbose=True, timestamps="--timestamps" in sys.argv[1:]))
