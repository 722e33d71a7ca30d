"""Builds libbsgd.so (the C-ABI library of HIP kernels) for gfx950, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
LIB_PATH = os.path.join(PKG_DIR, "libbsgd.so")
SOURCES = [os.path.join(PKG_DIR, "csrc", "bsgd.hip")]
HEADERS = [os.path.join(PKG_DIR, "csrc", "bsgd_kernels.hpp"), os.path.join(ROOT, "include", "bsgd.h"),
           os.path.join(ROOT, "include", "bsgd_debug.h")]

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-shared", "-fPIC", "-std=c++17",
    # packed-fp32 instruction forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # fused multiply-adds are written out by hand; none are formed behind our back
    "-ffp-contract=off",
    "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; libbsgd.so cannot be built")
    return exe


def build_library(verbose: bool = True) -> str:
    """Compile libbsgd.so (always recompiles) and return its path."""
    cmd = [hipcc()] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-o", LIB_PATH + ".tmp"] + SOURCES
    if verbose:
        print("+", " ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "is not a recognized feature for this target" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    return LIB_PATH


def library_is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(s) > t for s in SOURCES + HEADERS)


if __name__ == "__main__":
    build_library()
    print(LIB_PATH)
    sys.exit(0)
