"""Fills a whole synthetic KV cache on the device (fill.hip), bit-identical to Case.kv_rows."""
from __future__ import annotations

import ctypes
import os
import shutil
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_DIR, "libgenfill.so")
_lib = None


def build_library() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    cmd = [exe, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-fvisibility=hidden",
           os.path.join(_DIR, "fill.hip"), "-o", LIB_PATH + ".tmp"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    return LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            build_library()
        _lib = ctypes.CDLL(LIB_PATH)
        _lib.gen_fill_kv.restype = ctypes.c_int
        _lib.gen_fill_kv.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_int] + [ctypes.c_void_p] * 6
    return _lib


def fill_kv(case, device="cuda:0"):
    """Allocate K and V [B, Hkv, Lcap, D] on the device and fill them.  Returns (K, V) torch tensors
    (bfloat16 or float32)."""
    import torch

    spec = case.spec
    lib = _load()
    dt = torch.bfloat16 if spec.kv_dtype == "bf16" else torch.float32
    shape = (spec.B, spec.Hkv, case.Lcap, spec.D)
    K = torch.empty(shape, dtype=dt, device=device)
    V = torch.empty(shape, dtype=dt, device=device)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
    key_k = dev(case.key_k.view(np.int64))
    key_v = dev(case.key_v.view(np.int64))
    row_end = dev((case.seq_lens0 + spec.T).astype(np.int32))
    recent = dev((case.seq_lens0 - spec.recency).astype(np.int32))
    hot = dev(case.hot_pos.astype(np.int32))
    bias = dev(case.bias.astype(np.float32))
    st = torch.cuda.current_stream(device).cuda_stream
    n_hot = spec.n_hot
    rc = lib.gen_fill_kv(K.data_ptr(), int(spec.kv_dtype == "bf16"), spec.B, spec.Hkv, case.Lcap, n_hot,
                         key_k.data_ptr(), row_end.data_ptr(), recent.data_ptr(),
                         hot.data_ptr() if n_hot > 0 else None, bias.data_ptr(), st)
    if rc != 0:
        raise RuntimeError(f"gen_fill_kv(K) failed with hipError {rc}")
    rc = lib.gen_fill_kv(V.data_ptr(), int(spec.kv_dtype == "bf16"), spec.B, spec.Hkv, case.Lcap, 0,
                         key_v.data_ptr(), row_end.data_ptr(), None, None, None, st)
    if rc != 0:
        raise RuntimeError(f"gen_fill_kv(V) failed with hipError {rc}")
    torch.cuda.synchronize(device)
    return K, V
