"""Host sanitizers on the CPU side: the oracle (what every parity claim rests on) and the
C-ABI library's host code (argument checks, workspace arithmetic) run under AddressSanitizer
and UndefinedBehaviorSanitizer.  No GPU is involved."""
import os
import subprocess

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan():
    exe = oracle.build_sanitized()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "sanitize ok" in r.stdout, r.stderr[-3000:]
    # the same build stops an oracle call that is handed too short a buffer
    r = subprocess.run([exe, "plant"], capture_output=True, text=True, timeout=300)
    assert r.returncode != 0 and "AddressSanitizer" in r.stderr
    assert "went unnoticed" not in r.stdout


def test_abi_host_code_is_clean_under_asan_and_ubsan():
    """60 000 descriptors (extremes of every integer field, and plausible shapes) through the
    library's host-side validation and workspace arithmetic, built with the host sanitizers.
    Every call returns before anything is enqueued, so this runs without a GPU."""
    from paper_2502_11494_amd import build
    outdir = os.path.join(ROOT, "_build")
    lib = build.build_host_sanitized(outdir)
    exe = os.path.join(outdir, "abi_host_sanitize")
    clang = "/opt/rocm/llvm/bin/clang"  # the compiler whose sanitizer runtime the library uses
    subprocess.run([clang, "-O1", "-g", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "abi_host_sanitize.c"), "-L", outdir,
                    "-ldart_hip_san", "-Wl,-rpath," + outdir, "-o", exe], check=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and "abi sanitize ok" in r.stdout, (r.returncode, r.stderr[-3000:])
