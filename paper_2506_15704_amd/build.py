"""Builds liblfps.so (the HIP kernels + C ABI) in-tree with hipcc for gfx950."""
from __future__ import annotations

import hashlib
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(os.path.dirname(PKG_DIR), "include")
LIB_PATH = os.path.join(PKG_DIR, "liblfps.so")
SOURCES = ["lfps_api.hip", "candidates.hip", "score.hip", "select.hip", "select_attend.hip", "attention.hip", "tables.hip", "exact_topk.hip"]

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


def source_digest() -> str:
    """sha256 over the kernel sources, the internal header and the public header: what a built library was made from."""
    h = hashlib.sha256()
    for path in [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC))] + \
                [os.path.join(INCLUDE, f) for f in sorted(os.listdir(INCLUDE))]:
        if path.endswith((".hip", ".h", ".inc")):
            h.update(os.path.basename(path).encode())
            h.update(open(path, "rb").read())
    h.update(" ".join(HIPCC_FLAGS).encode())
    return h.hexdigest()


def built_digest() -> str:
    """The digest recorded beside the library when it was built ('' if there is none)."""
    try:
        return open(LIB_PATH + ".srchash").read().strip()
    except OSError:
        return ""


def build_library(verbose: bool = False) -> str:
    """Compile every kernel source (one hipcc per source, in parallel) and link paper_2506_15704_amd/liblfps.so;
    returns its path.  The digest of the sources is written beside it (liblfps.so.srchash)."""
    objdir = os.path.join(PKG_DIR, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc(), *flags, "-I", INCLUDE, "-I", CSRC, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n" + res.stdout + res.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), 8)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc (link) failed:\n" + res.stdout + res.stderr)
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    with open(LIB_PATH + ".srchash", "w") as f:
        f.write(source_digest() + "\n")
    return LIB_PATH


def ensure_built() -> str:
    """For tests, the smoke run and the benchmark: compile only if no library is there yet (the binding itself
    never builds and never falls back: without the library it raises).  A library built from other sources
    than the ones in the tree is loaded as it is, with a warning: build again after changing a source."""
    if not os.path.exists(LIB_PATH):
        return build_library()
    if built_digest() != source_digest():
        import warnings
        warnings.warn(f"{LIB_PATH} was not built from the sources in the tree (run `python -m paper_2506_15704_amd.build`)",
                      RuntimeWarning)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
