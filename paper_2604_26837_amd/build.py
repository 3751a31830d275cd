"""Builds the HIP library in-tree: ``paper_2604_26837_amd/libspin.so``.

``python -m paper_2604_26837_amd.build`` compiles every ``csrc/*.hip`` for
gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
# SPIN_LIB_PATH lets a developer load an experimental build instead of the in-tree one
LIB_PATH = os.environ.get("SPIN_LIB_PATH") or os.path.join(PKG_DIR, "libspin.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 VALU forms stay disabled on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(PKG_DIR, "csrc", "*.hip")))


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG_DIR, "csrc"),
           *sources(), "-o", LIB_PATH + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    return LIB_PATH


EXAMPLE_SRC = os.path.join(PKG_DIR, "examples", "one_step.cpp")
EXAMPLE_BIN = os.path.join(PKG_DIR, "examples", "one_step")


def build_example() -> str:
    """The C++ caller of the C ABI (no Python involved at run time), linked against libspin.so beside it."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", EXAMPLE_SRC, "-I", os.path.join(ROOT, "include"),
           "-L", PKG_DIR, "-lspin", "-Wl,-rpath,$ORIGIN/..", "-o", EXAMPLE_BIN + ".tmp"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    os.replace(EXAMPLE_BIN + ".tmp", EXAMPLE_BIN)
    return EXAMPLE_BIN


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_example())
