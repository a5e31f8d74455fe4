"""ctypes binding of liblfps.so: same names as the C ABI, argument marshalling only.

Every array argument is a torch tensor living on the GPU (PyTorch is used for device memory
and streams, nothing else); its dtype/shape/contiguity are checked here and its data pointer
is handed to the library.  There is no fallback: if the shared library is missing the import
of this module fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "liblfps.so")

LFPS_F32, LFPS_BF16, LFPS_F16 = 0, 1, 2
_KV_DTYPES = {"f32": (LFPS_F32, torch.float32), "bf16": (LFPS_BF16, torch.bfloat16), "f16": (LFPS_F16, torch.float16)}
LFPS_OK, LFPS_EINVAL, LFPS_ECAP, LFPS_EHIP, LFPS_ENOMEM = 0, -1, -2, -3, -4
LFPS_FLAG_CAND_OVERFLOW = 1
LFPS_FLAG_TABLE_FULL = 2
LFPS_FLAG_Q_RANGE = 4
N_KERNELS = 15
NOALLOC_MAX_SCORES = 2097152


class LfpsError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"liblfps error {code}: {msg}")
        self.code = code


class lfps_config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "batch", "n_q_heads", "n_kv_heads", "head_dim", "kv_dtype", "max_seq_len", "max_k",
        "radius", "n_recent", "n_sink", "cand_cap", "device", "table_mode")] + [
        ("table_decay", ctypes.c_float), ("table_a", ctypes.c_float), ("k_fp8", ctypes.c_int32),
        ("v_fp8", ctypes.c_int32)]


class lfps_kv(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64),
                ("seq_lens", ctypes.c_void_p), ("block_table", ctypes.c_void_p),
                ("block_size", ctypes.c_int32), ("block_table_stride", ctypes.c_int32),
                ("n_blocks", ctypes.c_int32)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2506_15704_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    P, I32, VP = ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p
    sig = {
        "lfps_create": (ctypes.c_int, [ctypes.POINTER(lfps_config), ctypes.POINTER(P)]),
        "lfps_destroy": (ctypes.c_int, [P]),
        "lfps_last_error": (ctypes.c_char_p, [P]),
        "lfps_workspace_bytes": (ctypes.c_int, [ctypes.POINTER(lfps_config), ctypes.POINTER(ctypes.c_int64)]),
        "lfps_host_device_pointer": (ctypes.c_int, [VP, ctypes.POINTER(VP)]),
        "lfps_cand_cap": (I32, [P]),
        "lfps_candidates": (ctypes.c_int, [P, VP, VP, VP, VP, VP, VP]),
        "lfps_score_topk": (ctypes.c_int, [P, VP, ctypes.POINTER(lfps_kv), VP, VP, VP, VP, VP, VP, VP]),
        "lfps_sparse_attn": (ctypes.c_int, [P, VP, ctypes.POINTER(lfps_kv), VP, VP, VP, VP, VP]),
        "lfps_step": (ctypes.c_int, [P, VP, ctypes.POINTER(lfps_kv), VP, VP, VP, VP, VP, VP]),
        "lfps_sparse_attn_noalloc": (ctypes.c_int, [ctypes.POINTER(lfps_config), VP, ctypes.POINTER(lfps_kv), VP, VP, VP, VP]),
        "lfps_full_attn_decode": (ctypes.c_int, [P, VP, ctypes.POINTER(lfps_kv), VP, VP]),
        "lfps_exact_topk": (ctypes.c_int, [P, VP, ctypes.POINTER(lfps_kv), VP, VP, VP, VP]),
        "lfps_poll_status": (ctypes.c_int, [P, ctypes.POINTER(I32), VP]),
        "lfps_poll_rescored": (ctypes.c_int, [P, ctypes.POINTER(I32), VP]),
        "lfps_timing_enable": (ctypes.c_int, [P, I32]),
        "lfps_timing_read": (ctypes.c_int, [P, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(I32), VP]),
        "lfps_kernel_name": (ctypes.c_char_p, [I32]),
        "lfps_calib_copy": (ctypes.c_int, [VP, VP, ctypes.c_int64, VP]),
        "lfps_set_filter": (ctypes.c_int, [P, I32]),
        "lfps_reset_history": (ctypes.c_int, [P, VP]),
        "lfps_copy_cand_count": (ctypes.c_int, [P, VP, VP]),
        "lfps_tables_init": (ctypes.c_int, [P, VP, I32, ctypes.POINTER(lfps_kv), VP]),
        "lfps_tables_import": (ctypes.c_int, [P, VP, VP, VP, VP]),
        "lfps_tables_export": (ctypes.c_int, [P, VP, VP, VP, VP]),
        "lfps_table_candidates": (ctypes.c_int, [P, VP, VP, VP, VP]),
        "lfps_table_update": (ctypes.c_int, [P, VP, VP, VP, VP, VP]),
        "lfps_table_step": (ctypes.c_int, [P, VP, ctypes.POINTER(lfps_kv), VP, VP, VP, VP, VP]),
        "lfps_priors": (ctypes.c_int, [P, VP, ctypes.POINTER(lfps_kv), VP, VP, VP, VP]),
        "lfps_head_sparsity": (ctypes.c_int, [P, VP, ctypes.POINTER(lfps_kv), VP, VP, I32, ctypes.c_float, VP, VP, VP]),
        "lfps_table_step_gated": (ctypes.c_int, [P, VP, ctypes.POINTER(lfps_kv), VP, VP, VP, VP, I32, ctypes.c_float,
                                                 VP, VP, VP, VP, VP]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


_lib = _load()


def kernel_names():
    return [_lib.lfps_kernel_name(i).decode() for i in range(N_KERNELS)]


def workspace_bytes(**cfg) -> int:
    c = lfps_config(**cfg)
    out = ctypes.c_int64(0)
    rc = _lib.lfps_workspace_bytes(ctypes.byref(c), ctypes.byref(out))
    if rc != LFPS_OK:
        raise LfpsError(rc, _lib.lfps_last_error(None).decode())
    return out.value


def _cache_ptr(t: torch.Tensor) -> int:
    """Address of a cache tensor for the kernels: a GPU tensor's own, or for a pinned host tensor (a host-resident
    cache) the address at which the device sees it."""
    if t.is_cuda:
        return t.data_ptr()
    if not t.is_pinned():
        raise TypeError("a cache tensor must live on the GPU or in pinned host memory")
    dev = ctypes.c_void_p(None)
    rc = _lib.lfps_host_device_pointer(t.data_ptr(), ctypes.byref(dev))
    if rc != LFPS_OK:
        raise LfpsError(rc, _lib.lfps_last_error(None).decode())
    return dev.value


def _ptr(t: Optional[torch.Tensor], dtype, shape, name: str, device) -> Optional[int]:
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.device != device:
        raise TypeError(f"{name}: expected a tensor on {device}")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected dtype {dtype}, got {t.dtype}")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    return t.data_ptr()


def lfps_calib_copy(dst: torch.Tensor, src: torch.Tensor):
    """Plain device copy with exactly known traffic (src.nbytes read, the same written)."""
    if not (dst.is_cuda and src.is_cuda and dst.is_contiguous() and src.is_contiguous()):
        raise TypeError("lfps_calib_copy: contiguous GPU tensors expected")
    nbytes = src.numel() * src.element_size()
    if nbytes != dst.numel() * dst.element_size():
        raise ValueError("lfps_calib_copy: size mismatch")
    rc = _lib.lfps_calib_copy(dst.data_ptr(), src.data_ptr(), nbytes, torch.cuda.current_stream(src.device).cuda_stream)
    if rc != LFPS_OK:
        raise LfpsError(rc, "lfps_calib_copy")


class Lfps:
    """A liblfps context.  Methods mirror the C entry points one to one."""

    def __init__(self, batch: int, n_q_heads: int = 32, n_kv_heads: int = 8, head_dim: int = 128,
                 kv_dtype: str = "bf16", max_seq_len: int = 0, max_k: int = 0, radius: int = 0,
                 n_recent: int = 1, n_sink: int = 0, cand_cap: int = 0, device: int = 0,
                 table_mode: bool = False, table_decay: float = 0.95, table_a: float = 0.2, k_fp8: bool = False,
                 v_fp8: bool = False):
        if kv_dtype not in _KV_DTYPES:
            raise ValueError(f"kv_dtype must be one of {sorted(_KV_DTYPES)} (got {kv_dtype!r})")
        self.cfg = lfps_config(batch, n_q_heads, n_kv_heads, head_dim,
                               _KV_DTYPES[kv_dtype][0], max_seq_len, max_k,
                               radius, n_recent, n_sink, cand_cap, device, int(bool(table_mode)),
                               float(table_decay), float(table_a), int(bool(k_fp8)), int(bool(v_fp8)))
        self.kv_torch_dtype = _KV_DTYPES[kv_dtype][1]
        self.k_torch_dtype = torch.float8_e4m3fn if k_fp8 else self.kv_torch_dtype
        self.v_torch_dtype = torch.float8_e4m3fn if v_fp8 else self.kv_torch_dtype
        self.device = torch.device("cuda", device)
        self._ctx = ctypes.c_void_p(None)
        rc = _lib.lfps_create(ctypes.byref(self.cfg), ctypes.byref(self._ctx))
        if rc != LFPS_OK:
            raise LfpsError(rc, _lib.lfps_last_error(None).decode())
        self.B, self.Hq, self.Hkv, self.D = batch, n_q_heads, n_kv_heads, head_dim
        self.kmax, self.Lcap = max_k, max_seq_len
        self.cand_cap = int(_lib.lfps_cand_cap(self._ctx))

    # ------------------------------------------------------------------ plumbing
    def close(self):
        if self._ctx:
            _lib.lfps_destroy(self._ctx)
            self._ctx = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != LFPS_OK:
            raise LfpsError(rc, _lib.lfps_last_error(self._ctx).decode())

    def _stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def kv_view(self, K: torch.Tensor, V: Optional[torch.Tensor], seq_lens: torch.Tensor) -> lfps_kv:
        """View of a [B, Hkv, Lcap', D] cache (any strides with a contiguous last dim); K and V on the GPU, or in
        pinned host memory for a host-resident cache (rows are then fetched over the host link)."""
        for name, t in (("K", K), ("V", V)):
            if t is None:
                continue
            want = self.k_torch_dtype if name == "K" else self.v_torch_dtype
            if not (t.is_cuda or t.is_pinned()) or t.dtype != want or t.dim() != 4:
                raise TypeError(f"{name}: expected a 4-d {want} tensor on the GPU (or in pinned host memory)")
            if t.shape[0] != self.B or t.shape[1] != self.Hkv or t.shape[3] != self.D or t.stride(3) != 1:
                raise ValueError(f"{name}: expected [B={self.B}, Hkv={self.Hkv}, rows, D={self.D}] with unit channel stride")
            if t.shape[2] < self.Lcap:
                raise ValueError(f"{name}: holds {t.shape[2]} rows per head, fewer than max_seq_len={self.Lcap}")
        if V is not None and V.stride() != K.stride():
            raise ValueError("K and V must share strides")
        sl = _ptr(seq_lens, torch.int32, (self.B,), "seq_lens", self.device)
        view = lfps_kv(_cache_ptr(K), _cache_ptr(V) if V is not None else None,
                       K.stride(0), K.stride(1), K.stride(2), sl, None, 0, 0, 0)
        view._keep = (K, V, seq_lens)   # the struct holds raw pointers: keep their tensors alive with it
        return view

    def paged_kv_view(self, K: torch.Tensor, V: Optional[torch.Tensor], block_table: torch.Tensor,
                      seq_lens: torch.Tensor) -> lfps_kv:
        """View of a paged cache: K, V are pools [n_blocks, Hkv, block_size, D] (any strides with a
        contiguous last dim, e.g. a permuted [n_blocks, block_size, Hkv, D]); block_table [B, max_blocks]
        int32 names the pool block of every logical block of a request."""
        for name, t in (("K", K), ("V", V)):
            if t is None:
                continue
            want = self.k_torch_dtype if name == "K" else self.v_torch_dtype
            if not t.is_cuda or t.dtype != want or t.dim() != 4:
                raise TypeError(f"{name}: expected a 4-d {want} tensor on the GPU")
            if t.shape[1] != self.Hkv or t.shape[3] != self.D or t.stride(3) != 1:
                raise ValueError(f"{name}: expected [n_blocks, Hkv={self.Hkv}, block_size, D={self.D}] with unit channel stride")
        if V is not None and (V.stride() != K.stride() or V.shape != K.shape):
            raise ValueError("K and V pools must share shape and strides")
        if (not block_table.is_cuda or block_table.dtype != torch.int32 or block_table.dim() != 2
                or block_table.shape[0] != self.B or block_table.stride(1) != 1):
            raise ValueError(f"block_table: expected an int32 [B={self.B}, max_blocks] tensor on the GPU with unit column stride")
        sl = _ptr(seq_lens, torch.int32, (self.B,), "seq_lens", self.device)
        view = lfps_kv(K.data_ptr(), V.data_ptr() if V is not None else None,
                       K.stride(0), K.stride(1), K.stride(2), sl, block_table.data_ptr(),
                       int(K.shape[2]), int(block_table.stride(0)), int(K.shape[0]))
        view._keep = (K, V, seq_lens, block_table)
        return view

    # ------------------------------------------------------------------ entry points
    def lfps_candidates(self, prev_topk, k, seq_lens, cand, cand_count):
        d = self.device
        self._check(_lib.lfps_candidates(
            self._ctx, _ptr(prev_topk, torch.int32, (self.B, self.Hq, self.kmax), "prev_topk", d),
            _ptr(k, torch.int32, (self.B,), "k", d), _ptr(seq_lens, torch.int32, (self.B,), "seq_lens", d),
            _ptr(cand, torch.int32, (self.B, self.Hkv, self.cand_cap), "cand", d),
            _ptr(cand_count, torch.int32, (self.B, self.Hkv), "cand_count", d), self._stream()))

    def lfps_score_topk(self, q, kv: lfps_kv, cand, cand_count, k, topk_idx, topk_score=None, cand_score=None):
        d = self.device
        self._check(_lib.lfps_score_topk(
            self._ctx, _ptr(q, torch.float32, (self.B, self.Hq, self.D), "q", d), ctypes.byref(kv),
            _ptr(cand, torch.int32, (self.B, self.Hkv, self.cand_cap), "cand", d),
            _ptr(cand_count, torch.int32, (self.B, self.Hkv), "cand_count", d),
            _ptr(k, torch.int32, (self.B,), "k", d),
            _ptr(topk_idx, torch.int32, (self.B, self.Hq, self.kmax), "topk_idx", d),
            _ptr(topk_score, torch.float32, (self.B, self.Hq, self.kmax), "topk_score", d),
            _ptr(cand_score, torch.float32, (self.B, self.Hq, self.cand_cap), "cand_score", d), self._stream()))

    def lfps_sparse_attn(self, q, kv: lfps_kv, idx, idx_score, k, out):
        d = self.device
        self._check(_lib.lfps_sparse_attn(
            self._ctx, _ptr(q, torch.float32, (self.B, self.Hq, self.D), "q", d), ctypes.byref(kv),
            _ptr(idx, torch.int32, (self.B, self.Hq, self.kmax), "idx", d),
            _ptr(idx_score, torch.float32, (self.B, self.Hq, self.kmax), "idx_score", d),
            _ptr(k, torch.int32, (self.B,), "k", d),
            _ptr(out, torch.float32, (self.B, self.Hq, self.D), "out", d), self._stream()))

    def lfps_sparse_attn_noalloc(self, q, kv: lfps_kv, idx, k, out):
        """The context-free, allocation-free S4 (scores recomputed into the library's static array), called with
        this context's configuration."""
        d = self.device
        rc = _lib.lfps_sparse_attn_noalloc(
            ctypes.byref(self.cfg), _ptr(q, torch.float32, (self.B, self.Hq, self.D), "q", d), ctypes.byref(kv),
            _ptr(idx, torch.int32, (self.B, self.Hq, self.kmax), "idx", d), _ptr(k, torch.int32, (self.B,), "k", d),
            _ptr(out, torch.float32, (self.B, self.Hq, self.D), "out", d), self._stream())
        if rc != LFPS_OK:
            raise LfpsError(rc, _lib.lfps_last_error(None).decode())

    def lfps_step(self, q, kv: lfps_kv, prev_topk, k, topk_idx, out, topk_score=None):
        d = self.device
        self._check(_lib.lfps_step(
            self._ctx, _ptr(q, torch.float32, (self.B, self.Hq, self.D), "q", d), ctypes.byref(kv),
            _ptr(prev_topk, torch.int32, (self.B, self.Hq, self.kmax), "prev_topk", d),
            _ptr(k, torch.int32, (self.B,), "k", d),
            _ptr(topk_idx, torch.int32, (self.B, self.Hq, self.kmax), "topk_idx", d),
            _ptr(topk_score, torch.float32, (self.B, self.Hq, self.kmax), "topk_score", d),
            _ptr(out, torch.float32, (self.B, self.Hq, self.D), "out", d), self._stream()))

    def lfps_full_attn_decode(self, q, kv: lfps_kv, out):
        d = self.device
        self._check(_lib.lfps_full_attn_decode(
            self._ctx, _ptr(q, torch.float32, (self.B, self.Hq, self.D), "q", d), ctypes.byref(kv),
            _ptr(out, torch.float32, (self.B, self.Hq, self.D), "out", d), self._stream()))

    def lfps_exact_topk(self, q, kv: lfps_kv, k, topk_idx, topk_score=None):
        d = self.device
        self._check(_lib.lfps_exact_topk(
            self._ctx, _ptr(q, torch.float32, (self.B, self.Hq, self.D), "q", d), ctypes.byref(kv),
            _ptr(k, torch.int32, (self.B,), "k", d),
            _ptr(topk_idx, torch.int32, (self.B, self.Hq, self.kmax), "topk_idx", d),
            _ptr(topk_score, torch.float32, (self.B, self.Hq, self.kmax), "topk_score", d), self._stream()))

    # ------------------------------------------------------------------ score tables
    def lfps_tables_init(self, q_hist, kv: lfps_kv):
        """q_hist: [s, B, Hq, D] (or [B, Hq, D] for one query), most recent query first."""
        if q_hist.dim() == 3:
            q_hist = q_hist.unsqueeze(0)
        s = int(q_hist.shape[0])
        self._check(_lib.lfps_tables_init(
            self._ctx, _ptr(q_hist, torch.float32, (s, self.B, self.Hq, self.D), "q_hist", self.device), s,
            ctypes.byref(kv), self._stream()))

    def lfps_tables_import(self, phi_ver, phi_sla, seq_lens):
        d, shp = self.device, (self.B, self.Hq, self.Lcap)
        self._check(_lib.lfps_tables_import(
            self._ctx, _ptr(phi_ver, torch.float32, shp, "phi_ver", d), _ptr(phi_sla, torch.float32, shp, "phi_sla", d),
            _ptr(seq_lens, torch.int32, (self.B,), "seq_lens", d), self._stream()))

    def lfps_tables_export(self, phi_ver, phi_sla, seq_lens):
        d, shp = self.device, (self.B, self.Hq, self.Lcap)
        self._check(_lib.lfps_tables_export(
            self._ctx, _ptr(phi_ver, torch.float64, shp, "phi_ver", d), _ptr(phi_sla, torch.float64, shp, "phi_sla", d),
            _ptr(seq_lens, torch.int32, (self.B,), "seq_lens", d), self._stream()))

    def lfps_table_candidates(self, seq_lens, cand, cand_count):
        d = self.device
        self._check(_lib.lfps_table_candidates(
            self._ctx, _ptr(seq_lens, torch.int32, (self.B,), "seq_lens", d),
            _ptr(cand, torch.int32, (self.B, self.Hkv, self.cand_cap), "cand", d),
            _ptr(cand_count, torch.int32, (self.B, self.Hkv), "cand_count", d), self._stream()))

    def lfps_table_update(self, idx, idx_score, k, seq_lens):
        d = self.device
        self._check(_lib.lfps_table_update(
            self._ctx, _ptr(idx, torch.int32, (self.B, self.Hq, self.kmax), "idx", d),
            _ptr(idx_score, torch.float32, (self.B, self.Hq, self.kmax), "idx_score", d),
            _ptr(k, torch.int32, (self.B,), "k", d), _ptr(seq_lens, torch.int32, (self.B,), "seq_lens", d),
            self._stream()))

    def lfps_table_step(self, q, kv: lfps_kv, k, topk_idx, out, topk_score=None):
        d = self.device
        self._check(_lib.lfps_table_step(
            self._ctx, _ptr(q, torch.float32, (self.B, self.Hq, self.D), "q", d), ctypes.byref(kv),
            _ptr(k, torch.int32, (self.B,), "k", d),
            _ptr(topk_idx, torch.int32, (self.B, self.Hq, self.kmax), "topk_idx", d),
            _ptr(topk_score, torch.float32, (self.B, self.Hq, self.kmax), "topk_score", d),
            _ptr(out, torch.float32, (self.B, self.Hq, self.D), "out", d), self._stream()))

    # ------------------------------------------------------------------ head sparsity bypass
    def lfps_priors(self, q, kv: lfps_kv, kbar, vbar, sigma2_hat):
        d = self.device
        self._check(_lib.lfps_priors(
            self._ctx, _ptr(q, torch.float32, (self.B, self.Hq, self.D), "q", d), ctypes.byref(kv),
            _ptr(kbar, torch.float32, (self.B, self.Hkv, self.D), "kbar", d),
            _ptr(vbar, torch.float32, (self.B, self.Hkv, self.D), "vbar", d),
            _ptr(sigma2_hat, torch.float32, (self.B, self.Hq), "sigma2_hat", d), self._stream()))

    def lfps_head_sparsity(self, q, kv: lfps_kv, kbar, sigma2_hat, n_local, eps, rho, gate):
        d = self.device
        self._check(_lib.lfps_head_sparsity(
            self._ctx, _ptr(q, torch.float32, (self.B, self.Hq, self.D), "q", d), ctypes.byref(kv),
            _ptr(kbar, torch.float32, (self.B, self.Hkv, self.D), "kbar", d),
            _ptr(sigma2_hat, torch.float32, (self.B, self.Hq), "sigma2_hat", d), int(n_local), float(eps),
            _ptr(rho, torch.float32, (self.B, self.Hq), "rho", d),
            _ptr(gate, torch.int32, (self.B, self.Hq), "gate", d), self._stream()))

    def lfps_table_step_gated(self, q, kv: lfps_kv, k, kbar, vbar, sigma2_hat, n_local, eps, topk_idx, out,
                              topk_score=None, gate_out=None):
        d = self.device
        self._check(_lib.lfps_table_step_gated(
            self._ctx, _ptr(q, torch.float32, (self.B, self.Hq, self.D), "q", d), ctypes.byref(kv),
            _ptr(k, torch.int32, (self.B,), "k", d),
            _ptr(kbar, torch.float32, (self.B, self.Hkv, self.D), "kbar", d),
            _ptr(vbar, torch.float32, (self.B, self.Hkv, self.D), "vbar", d),
            _ptr(sigma2_hat, torch.float32, (self.B, self.Hq), "sigma2_hat", d), int(n_local), float(eps),
            _ptr(topk_idx, torch.int32, (self.B, self.Hq, self.kmax), "topk_idx", d),
            _ptr(topk_score, torch.float32, (self.B, self.Hq, self.kmax), "topk_score", d),
            _ptr(out, torch.float32, (self.B, self.Hq, self.D), "out", d),
            _ptr(gate_out, torch.int32, (self.B, self.Hq), "gate_out", d), self._stream()))

    def lfps_set_filter(self, on: bool):
        self._check(_lib.lfps_set_filter(self._ctx, int(bool(on))))

    def lfps_reset_history(self):
        self._check(_lib.lfps_reset_history(self._ctx, self._stream()))

    def lfps_copy_cand_count(self, dst):
        self._check(_lib.lfps_copy_cand_count(
            self._ctx, _ptr(dst, torch.int32, (self.B, self.Hkv), "dst", self.device), self._stream()))

    def lfps_poll_status(self) -> int:
        flags = ctypes.c_int32(0)
        self._check(_lib.lfps_poll_status(self._ctx, ctypes.byref(flags), self._stream()))
        return flags.value

    def lfps_poll_rescored(self) -> int:
        n = ctypes.c_int32(0)
        self._check(_lib.lfps_poll_rescored(self._ctx, ctypes.byref(n), self._stream()))
        return n.value

    def lfps_timing_enable(self, on: bool):
        self._check(_lib.lfps_timing_enable(self._ctx, int(bool(on))))

    def lfps_timing_read(self):
        """-> {kernel name: (total ms, launches)} since the last read."""
        ms = (ctypes.c_float * N_KERNELS)()
        n = (ctypes.c_int32 * N_KERNELS)()
        self._check(_lib.lfps_timing_read(self._ctx, ms, n, self._stream()))
        return {name: (float(ms[i]), int(n[i])) for i, name in enumerate(kernel_names())}
