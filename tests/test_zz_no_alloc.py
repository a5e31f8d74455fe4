"""The allocation-free S4 entry point (lfps_sparse_attn_noalloc: no context, scores of the selected rows in the
library's static device array) against the existing lfps_sparse_attn with recomputed scores, through the C ABI:
two calls in a row, the second with a smaller input, each compared bit for bit with the context-based call and
with the oracle at the usual tolerance."""
import numpy as np
import pytest
import torch

import gen
from oracle import lfps_oracle as orc
from tests.harness import DEV, DeviceCase, assert_out_close, dev

pytestmark = pytest.mark.gpu


def _random_idx(rng, B, Hq, kmax, k, n):
    idx = np.full((B, Hq, kmax), -1, dtype=np.int32)
    for b in range(B):
        for h in range(Hq):
            idx[b, h, : k[b]] = np.sort(rng.choice(int(n[b]), size=int(k[b]), replace=False))
    idx[0, 1, 3] = -1                       # padding inside a list
    idx[B - 1, 2, 0] = int(n[B - 1]) + 7      # an entry past the end of the request: skipped
    return idx


def _one_case(spec, seed, first_call=False):
    dc = DeviceCase(spec)
    case = dc.case
    ctx = dc.make_ctx()
    rng = np.random.default_rng(seed)
    t = 1
    n = case.seq_lens(t)
    idx = _random_idx(rng, spec.B, spec.Hq, case.kmax, case.k, n)
    kv = ctx.kv_view(dc.K, dc.V, dc.seq_lens(t))
    want = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
    got = torch.full_like(want, float("nan"))
    idx_d, q_d = dev(idx), dc.q(t)
    ctx.lfps_sparse_attn(q_d, kv, idx_d, None, dc.k, want)                  # the existing entry point (workspace scores)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    ctx.lfps_sparse_attn_noalloc(q_d, kv, idx_d, dc.k, got)                 # the static-scratch entry point
    torch.cuda.synchronize()
    # (the runtime places the library's static device data on a GPU when the library is first used there, so the
    # first call is not held to this)
    assert first_call or torch.cuda.mem_get_info()[0] == free_before, "device memory in use changed across the call"
    assert torch.equal(got, want), f"{spec.name}: static-scratch result differs from the workspace result"
    got_h = got.cpu().numpy()
    G = spec.G
    for (b, g) in ((0, 0), (spec.B - 1, spec.Hkv - 1)):
        K, V = dc.group(b, g)
        for hh in range(G):
            h = G * g + hh
            rows = idx[b, h, : case.k[b]]
            rows = rows[(rows >= 0) & (rows < n[b])]
            assert_out_close(got_h[b, h], orc.sparse_attn(case.q[t, b, h], K, V, rows), f"{spec.name} b{b} h{h}")
    ctx.close()


def test_noalloc_sparse_attention_matches_the_context_entry_point_twice():
    # first call: the larger input (fills more of the static array) ...
    _one_case(gen.tiny_spec("noalloc_a", B=3, L=2600, k=160, r=2, T=2), 1, first_call=True)
    # ... second call: a smaller one, whose entries sit where the first call's scores still are
    _one_case(gen.tiny_spec("noalloc_b", B=2, L=900, k=40, r=2, T=2, kv_dtype="f32"), 2)
    _one_case(gen.tiny_spec("noalloc_c", B=1, L=1500, k=72, r=2, T=2, k_dtype="fp8", v_dtype="fp8"), 3)


def test_noalloc_refuses_what_does_not_fit_and_bad_arguments():
    from paper_2506_15704_amd import binding as b
    spec = gen.tiny_spec("noalloc_big", B=1, L=600, k=32, r=1, T=1)
    dc = DeviceCase(spec)
    ctx = dc.make_ctx()
    kv = ctx.kv_view(dc.K, dc.V, dc.seq_lens(1))
    idx = torch.zeros((1, spec.Hq, dc.case.kmax), dtype=torch.int32, device=DEV)
    out = torch.zeros((1, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
    # a shape whose scores exceed the static array: refused with LFPS_ECAP before anything is launched
    big = b.lfps_config(64, 32, 8, 128, b.LFPS_BF16, 4096, 2048, 2, 1, 0, 0, 0, 0, 0.95, 0.2, 0, 0)
    assert 64 * 32 * 2048 > b.NOALLOC_MAX_SCORES
    import ctypes
    rc = b._lib.lfps_sparse_attn_noalloc(ctypes.byref(big), dc.q(1).data_ptr(), ctypes.byref(kv), idx.data_ptr(),
                                         dc.k.data_ptr(), out.data_ptr(), None)
    assert rc == b.LFPS_ECAP and b"static scratch" in b._lib.lfps_last_error(None)
    # NULL argument and a device that is not the current one
    rc = b._lib.lfps_sparse_attn_noalloc(ctypes.byref(ctx.cfg), None, ctypes.byref(kv), idx.data_ptr(), dc.k.data_ptr(),
                                         out.data_ptr(), None)
    assert rc == b.LFPS_EINVAL
    other = b.lfps_config.from_buffer_copy(ctx.cfg)
    other.device = 3
    rc = b._lib.lfps_sparse_attn_noalloc(ctypes.byref(other), dc.q(1).data_ptr(), ctypes.byref(kv), idx.data_ptr(),
                                         dc.k.data_ptr(), out.data_ptr(), None)
    assert rc == b.LFPS_EINVAL and b"current device" in b._lib.lfps_last_error(None)
    ctx.close()
