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
    (bfloat16, float16 or float32; K is float8_e4m3fn when the spec asks for FP8 keys)."""
    import torch

    spec = case.spec
    lib = _load()
    dt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[spec.kv_dtype]
    shape = (spec.B, spec.Hkv, case.Lcap, spec.D)
    k_fp8 = spec.k_dtype == "fp8"
    K = torch.empty(shape, dtype=torch.float8_e4m3fn if k_fp8 else dt, device=device)
    v_fp8 = spec.v_dtype == "fp8"
    V = torch.empty(shape, dtype=torch.float8_e4m3fn if v_fp8 else dt, device=device)
    fmt = {"f32": 0, "bf16": 1, "f16": 3}[spec.kv_dtype]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
    key_k = dev(case.key_k.view(np.int64))
    key_v = dev(case.key_v.view(np.int64))
    row_end = dev((case.seq_lens0 + spec.T).astype(np.int32))
    recent = dev((case.seq_lens0 - spec.recency).astype(np.int32))
    hot = dev(case.hot_pos.astype(np.int32))
    bias = dev(case.bias.astype(np.float32))
    st = torch.cuda.current_stream(device).cuda_stream
    n_hot = spec.n_hot
    rc = lib.gen_fill_kv(K.data_ptr(), 2 if k_fp8 else fmt, spec.B, spec.Hkv, case.Lcap, n_hot,
                         key_k.data_ptr(), row_end.data_ptr(), recent.data_ptr(),
                         hot.data_ptr() if n_hot > 0 else None, bias.data_ptr(), st)
    if rc != 0:
        raise RuntimeError(f"gen_fill_kv(K) failed with hipError {rc}")
    rc = lib.gen_fill_kv(V.data_ptr(), 2 if v_fp8 else fmt, spec.B, spec.Hkv, case.Lcap, 0,
                         key_v.data_ptr(), row_end.data_ptr(), None, None, None, st)
    if rc != 0:
        raise RuntimeError(f"gen_fill_kv(V) failed with hipError {rc}")
    torch.cuda.synchronize(device)
    return K, V


def paginate(K, V, block_size: int, seed: int = 0, spare_blocks: int = 3, layout: str = "block_head_row",
             table_pad: int = 2):
    """The same cache as a paged pool (data movement only): the rows of every request are cut into
    blocks of `block_size` rows and scattered over a pool in a seeded random order, with
    `spare_blocks` unused blocks (filled with 1e4, so that a wrong lookup cannot go unnoticed) mixed in.

    K, V: [B, Hkv, Lcap, D] device tensors.  Returns (K_pool, V_pool, block_table):
      K_pool, V_pool  [n_blocks, Hkv, block_size, D] views; memory order [block, head, row, D]
                      (layout "block_head_row") or [block, row, head, D] ("block_row_head")
      block_table     [B, ceil(Lcap / block_size) + table_pad] int32; the padding columns hold -1.
    """
    import torch

    B, Hkv, Lcap, D = K.shape
    nb = (Lcap + block_size - 1) // block_size
    n_blocks = B * nb + spare_blocks
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed) + 977)
    perm = torch.randperm(n_blocks, generator=g)[: B * nb].to(torch.int64)
    table = torch.full((B, nb + table_pad), -1, dtype=torch.int32)
    table[:, :nb] = perm.view(B, nb).to(torch.int32)
    pools = []
    for X in (K, V):
        as_bytes = X.dtype == torch.float8_e4m3fn          # moved as bytes; filler = 448, the largest E4M3 value
        fill = 0x7E if as_bytes else 1e4
        if as_bytes:
            X = X.view(torch.uint8)
        if layout == "block_head_row":
            pool = torch.full((n_blocks, Hkv, block_size, D), fill, dtype=X.dtype, device=X.device)
            view = pool
        elif layout == "block_row_head":
            pool = torch.full((n_blocks, block_size, Hkv, D), fill, dtype=X.dtype, device=X.device)
            view = pool.permute(0, 2, 1, 3)
        else:
            raise ValueError(layout)
        for b in range(B):
            xb = X[b]
            if nb * block_size != Lcap:
                pad = torch.full((Hkv, nb * block_size - Lcap, D), fill, dtype=X.dtype, device=X.device)
                xb = torch.cat([xb, pad], dim=1)
            blocks = xb.view(Hkv, nb, block_size, D).permute(1, 0, 2, 3)     # [nb, Hkv, bs, D]
            view[perm[b * nb: (b + 1) * nb].to(X.device)] = blocks
        pools.append(view.view(torch.float8_e4m3fn) if as_bytes else view)
    return pools[0], pools[1], table.to(K.device)
