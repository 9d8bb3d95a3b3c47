"""Builds libdart_hip.so (the C-ABI library of include/dart.h) for gfx950 with hipcc.

Run as `python -m paper_2502_11494_amd.build`.  hipcc cross-compiles, so no GPU
is needed to build.
"""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libdart_hip.so")  # the path binding.py loads

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC", "-fvisibility=hidden",
    "-Wall", "-Wno-unused-function",
    # the compiler must not form packed-fp32 VALU instructions (kept off as a precaution
    # against silently wrong results of some of their forms)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build_hip(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    src = os.path.join(CSRC, "dart_api.hip")
    cmd = [hipcc, *HIPCC_FLAGS, src, "-o", LIB]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build_hip(verbose=True))
