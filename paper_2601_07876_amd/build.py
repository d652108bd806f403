"""Builds libnovak.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

Usage:  python -m paper_2601_07876_amd.build
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libnovak.so")
HOSTCOST_PATH = os.path.join(PKG_DIR, "novak_hostcost")     # plain C++ timing loop over novak_step (no Python in the way)

SOURCES = ["novak_host.cpp", "novak_device.hip"]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared",
    "--offload-arch=gfx950",
    # IEEE arithmetic: explicit FMAs only, no fast-math, correctly rounded sqrt/div (hipcc default)
    "-ffp-contract=off",
    # packed fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-unknown-warning-option",
]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def ensure_built(verbose: bool = False) -> str:
    """For drivers (tests, smoke, bench): builds only where nothing has been built yet; the library itself never does."""
    if not os.path.exists(LIB_PATH):
        build_library(verbose)
    return LIB_PATH


def build_library(verbose: bool = True) -> str:
    cmd = [hipcc_path()] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    # the host-only source is C++ without device code; -x hip compiles both uniformly
    cmd += ["-x", "hip"] + [os.path.join(CSRC, s) for s in SOURCES]
    tmp = LIB_PATH + ".tmp"
    cmd += ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed")
    if verbose and res.stderr.strip():
        # hipcc's host pass does not know the packed-fp32 feature and says so; harmless
        lines = [l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip()]
        if lines:
            print("\n".join(lines))
    os.replace(tmp, LIB_PATH)
    build_hostcost(verbose)
    return LIB_PATH


def build_hostcost(verbose: bool = True) -> str:
    """The host-cost timing tool: a host-only program against include/novak.h, linked to the library beside it."""
    cmd = [hipcc_path(), "-O2", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wextra", "-Wno-unknown-warning-option", "-I", os.path.join(ROOT, "include"),
           os.path.join(CSRC, "novak_hostcost.cpp"), "-L", PKG_DIR, "-lnovak", "-Wl,-rpath,$ORIGIN", "-o", HOSTCOST_PATH + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed (novak_hostcost)")
    os.replace(HOSTCOST_PATH + ".tmp", HOSTCOST_PATH)
    return HOSTCOST_PATH


if __name__ == "__main__":
    print(build_library())
