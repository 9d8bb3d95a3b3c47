"""Builds libdart_hip.so (the C-ABI library of include/dart.h) for gfx950 with hipcc.

Run as `python -m paper_2502_11494_amd.build`.  hipcc cross-compiles, so no GPU
is needed to build.  A stamp file beside the library records the hash of the
sources it was built from; `ensure_built()` (what the tests, the smoke check and
the benchmark call) loads an up-to-date library as it is and rebuilds a missing or
stale one, so a library older than its sources is never measured as if it were new.
"""
from __future__ import annotations

import glob
import hashlib
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(_HERE), "include")
LIB = os.path.join(_HERE, "libdart_hip.so")  # the path binding.py loads
STAMP = LIB + ".sha256"

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC", "-fvisibility=hidden",
    "-Wall", "-Wno-unused-function",
    # the compiler must not form packed-fp32 VALU instructions (kept off as a precaution
    # against silently wrong results of some of their forms)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def source_hash() -> str:
    """sha256 over the kernel sources, the public header and the compiler flags."""
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(CSRC, "*"))) + sorted(
            glob.glob(os.path.join(INCLUDE, "*.h"))):
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    h.update(" ".join(HIPCC_FLAGS).encode())
    return h.hexdigest()


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
    with open(STAMP, "w") as f:
        f.write(source_hash() + "\n")
    return LIB


def build_host_sanitized(outdir: str) -> str:
    """The same library with AddressSanitizer and UndefinedBehaviorSanitizer on its HOST code
    (argument checks, workspace arithmetic, launches), written to `outdir` as
    libdart_hip_san.so; rebuilt only when the sources changed.  For the CPU test that sweeps
    the ABI with invalid arguments; never loaded by the product."""
    os.makedirs(outdir, exist_ok=True)
    out = os.path.join(outdir, "libdart_hip_san.so")
    stamp = out + ".sha256"
    try:
        with open(stamp) as f:
            if os.path.exists(out) and f.read().strip() == source_hash():
                return out
    except OSError:
        pass
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f != "-O3"] + ["-O1", "-g"]
    for san in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"):
        flags += ["-Xarch_host", san]
    res = subprocess.run([hipcc, *flags, os.path.join(CSRC, "dart_api.hip"), "-o", out],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc (host sanitizers) failed ({res.returncode}):\n{res.stderr}")
    with open(stamp, "w") as f:
        f.write(source_hash() + "\n")
    return out


def is_current() -> bool:
    """True if the library exists and was built from the sources as they are now."""
    try:
        with open(STAMP) as f:
            return os.path.exists(LIB) and f.read().strip() == source_hash()
    except OSError:
        return False


def ensure_built(verbose: bool = False) -> str:
    """The library's path; compiles only if it is missing or older than its sources."""
    if not is_current():
        build_hip(verbose=verbose)
    return LIB


if __name__ == "__main__":
    print(build_hip(verbose=True))
