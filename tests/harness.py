"""Shared plumbing of the GPU parity tests: device tensors for a generated case, per-group
oracle inputs, and the comparison rules (tolerances as stated for the benchmark):

  * candidate sets               bit-exact
  * scores                       |gpu - oracle| <= 1e-4 * max(|oracle|, 1)
  * Top-k sets                   equal, except indices whose oracle score lies within
                                 1e-4 * max(|s_k|, 1) of the oracle's k-th score s_k
  * attention outputs            |gpu - oracle| <= 2e-3 absolute
"""
import functools

import numpy as np
import torch

import gen
from gen import device as gen_device
from oracle import lfps_oracle as orc

SCORE_RTOL = 1e-4
OUT_ATOL = 2e-3
DEV = "cuda:0"


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def stored_values(T):
    """A cache tensor as float32 (FP8 keys are decoded through the generator's table of the 256 E4M3 values)."""
    if T.dtype == torch.float8_e4m3fn:
        lut = torch.from_numpy(gen.cases.E4M3_VALUES).to(T.device)
        return lut[T.view(torch.uint8).long()]
    return T.float()


class DeviceCase:
    """A generated case with its KV cache resident on the GPU."""

    def __init__(self, spec):
        self.spec = spec
        self.case = gen.make_case(spec)
        self.K, self.V = gen_device.fill_kv(self.case, DEV)
        self.k = dev(self.case.k)
        self._groups = {}

    def q(self, t):
        return dev(self.case.q[t])

    def seq_lens(self, t):
        return dev(self.case.seq_lens(t))

    def group(self, b, g):
        """(K, V) float32 arrays of one (b, g), regenerated on the CPU (cached)."""
        if (b, g) not in self._groups:
            self._groups[(b, g)] = self.case.kv_group(b, g)
        return self._groups[(b, g)]

    def make_ctx(self, **kw):
        from paper_2506_15704_amd.binding import Lfps
        s = self.spec
        args = dict(batch=s.B, n_q_heads=s.Hq, n_kv_heads=s.Hkv, head_dim=s.D, kv_dtype=s.kv_dtype,
                    max_seq_len=self.case.Lcap, max_k=self.case.kmax, radius=s.r, n_recent=1, n_sink=0,
                    k_fp8=s.k_dtype == "fp8", v_fp8=s.v_dtype == "fp8")
        args.update(kw)
        return Lfps(**args)


def assert_scores_close(gpu, ref, what=""):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    tol = SCORE_RTOL * np.maximum(np.abs(ref), 1.0)
    bad = np.abs(gpu - ref) > tol
    assert not bad.any(), f"{what}: {bad.sum()} scores off, worst {np.abs(gpu - ref).max():.3e}"


def assert_topk_equal_mod_ties(gpu_idx, orc_idx, orc_scores_of, k, what=""):
    """gpu_idx / orc_idx: selected positions; orc_scores_of(positions) -> oracle fp64 scores."""
    gpu_idx = np.asarray(gpu_idx, dtype=np.int64)
    orc_idx = np.asarray(orc_idx, dtype=np.int64)
    assert len(gpu_idx) == len(orc_idx) == k, f"{what}: sizes {len(gpu_idx)} {len(orc_idx)} k={k}"
    assert len(np.unique(gpu_idx)) == k, f"{what}: duplicate indices"
    diff = np.setxor1d(gpu_idx, orc_idx)
    if len(diff) == 0:
        return 0
    s_k = float(np.min(orc_scores_of(orc_idx)))
    band = SCORE_RTOL * max(abs(s_k), 1.0)
    sd = orc_scores_of(diff)
    assert np.all(np.abs(sd - s_k) <= band), \
        f"{what}: {len(diff)} differing indices, worst distance to the k-th score {np.abs(sd - s_k).max():.3e} > {band:.1e}"
    return len(diff)


def assert_out_close(gpu, ref, what=""):
    err = np.abs(np.asarray(gpu, dtype=np.float64) - np.asarray(ref, dtype=np.float64)).max()
    assert err <= OUT_ATOL, f"{what}: attention output off by {err:.3e}"
    return err


def valid_row(row):
    row = np.asarray(row)
    return row[row >= 0]
