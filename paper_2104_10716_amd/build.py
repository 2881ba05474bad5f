"""Compile the HIP library for gfx950 in-tree (paper_2104_10716_amd/libes_spmm.so)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
SRC = os.path.join(PKG, "csrc", "es_spmm.hip")
LIB = os.path.join(PKG, "libes_spmm.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # packed-fp32 instruction selection is switched off for every kernel
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra",
    "-I" + os.path.join(ROOT, "include"),
    "-I" + os.path.join(PKG, "csrc"),
]


def build(verbose: bool = False, out: str = LIB, extra_flags=()) -> str:
    """Compile the library to `out` (default: in-tree).  `extra_flags` are added
    to the hipcc line (host-side instrumentation for the sanitizer test)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + [SRC, "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
