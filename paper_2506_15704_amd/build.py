"""Builds liblfps.so (the HIP kernels + C ABI) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import shutil
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(os.path.dirname(PKG_DIR), "include")
LIB_PATH = os.path.join(PKG_DIR, "liblfps.so")
SOURCES = ["lfps_api.hip", "candidates.hip", "score.hip", "select.hip", "attention.hip", "tables.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # never emit packed-fp32 ALU ops
    "-fvisibility=hidden", "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; liblfps cannot be built")
    return exe


def build_library(verbose: bool = False) -> str:
    """Compile every kernel source into paper_2506_15704_amd/liblfps.so and return its path."""
    cmd = [hipcc(), *HIPCC_FLAGS, "-I", INCLUDE, "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB_PATH + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    return LIB_PATH


def ensure_built() -> str:
    """For tests, the smoke run and the benchmark: compile only if no library is there yet (the binding itself
    never builds and never falls back: without the library it raises)."""
    return LIB_PATH if os.path.exists(LIB_PATH) else build_library()


if __name__ == "__main__":
    print(build_library(verbose=True))
