"""Builds ``libmarsit.so`` (HIP, gfx950) in-tree with hipcc.  ``python -m paper_2204_06787_amd.build``."""

from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
SOURCES = [os.path.join(PKG, "csrc", name) for name in (
    "marsit_fused.hip",          # fused one-bit pass (ring / torus / tree), full-precision round
    "marsit_worker_ops.hip",     # per-worker kernels, the chain, host utilities
    "marsit_diagnostics.hip",    # matching rate, majority vote, SSDM / cascading strawman
    "marsit_pipeline.hip",       # the ring as one stream per worker
)]
HEADERS = [os.path.join(PKG, "csrc", "marsit_device.hpp"), os.path.join(PKG, "csrc", "marsit_host.hpp"),
           os.path.join(ROOT, "include", "marsit.h")]
LIB = os.path.join(PKG, "libmarsit.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                      # every fp32 step is a single rounding
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 instructions
    "-Wall", "-Wextra",
]


def fused_sources_digest() -> str:
    """First 16 hex digits of the SHA-256 of the sources that define the fused kernels.  Counter
    summaries of those kernels record it, so a reader can tell whether they describe this tree."""
    import hashlib
    h = hashlib.sha256()
    for name in ("marsit_fused.hip", "marsit_device.hpp", "marsit_host.hpp"):
        with open(os.path.join(PKG, "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the HIP library cannot be built on this machine")
    return exe


def build_library(force: bool = True, extra_flags=(), out: str | None = None) -> str:
    """Compile the HIP library.  With ``force=False`` an up-to-date library is kept."""
    out = out or LIB
    if not force and os.path.exists(out):
        newest = max(os.path.getmtime(p) for p in SOURCES + HEADERS)
        if os.path.getmtime(out) >= newest:
            return out
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(PKG, "csrc"), "-o", out, *SOURCES]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        sys.stderr.write(proc.stdout + proc.stderr)
        raise RuntimeError("hipcc failed: " + " ".join(cmd))
    return out


C_CLIENT_SRC = os.path.join(ROOT, "tests", "helpers", "abi_c_client.c")
C_CLIENT = os.path.join(ROOT, "tests", "helpers", "abi_c_client")


def build_c_client(rocm: str = "/opt/rocm") -> str:
    """Compile the plain-C test client of the ABI with gcc and link it against the built library."""
    if not os.path.exists(LIB):
        raise RuntimeError("build the HIP library first")
    cmd = ["gcc", "-std=c11", "-O2", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(rocm, "include"), "-I", os.path.join(ROOT, "include"), C_CLIENT_SRC,
           "-o", C_CLIENT, "-L", PKG, "-lmarsit", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_2204_06787_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        sys.stderr.write(proc.stdout + proc.stderr)
        raise RuntimeError("gcc failed: " + " ".join(cmd))
    return C_CLIENT


if __name__ == "__main__":
    print(build_library(force=True))
    print(build_c_client())
