"""Paged KV cache (block table + block pool) through the C ABI.

The cache layout changes where a row is read from and nothing else, so every entry point must return
bit for bit what it returns for the same rows in a contiguous cache; one whole step is also compared
with the CPU oracle directly.  The pools come from gen.device.paginate (data movement only): blocks in a
seeded random order, spare blocks filled with 1e4 so that a read of the wrong block cannot go unnoticed.
"""
import numpy as np
import pytest
import torch

import gen
from gen import device as gen_device
from oracle import lfps_oracle as orc
from tests.harness import DEV, DeviceCase, assert_out_close, assert_topk_equal_mod_ties, dev, valid_row

pytestmark = pytest.mark.gpu

LAYOUTS = [("bf16", 16, "block_head_row"), ("bf16", 64, "block_row_head"), ("f32", 32, "block_head_row"),
           ("bf16", 1, "block_head_row"), ("bf16", 4096, "block_row_head"), ("fp8", 16, "block_head_row"),
           ("fp8", 128, "block_row_head"), ("fp8kv", 32, "block_row_head"), ("f16", 16, "block_row_head")]


@pytest.fixture(scope="module")
def cases():
    return {"bf16": DeviceCase(gen.tiny_spec("paged_bf16", B=3, L=2500, k=96, r=2, T=4)),
            "f32": DeviceCase(gen.tiny_spec("paged_f32", B=2, L=1111, k=64, r=3, T=3, kv_dtype="f32")),
            "fp8": DeviceCase(gen.tiny_spec("paged_fp8", B=2, L=1700, k=64, r=2, T=3, k_dtype="fp8")),
            "fp8kv": DeviceCase(gen.tiny_spec("paged_fp8kv", B=2, L=1300, k=64, r=2, T=3, k_dtype="fp8", v_dtype="fp8")),
            "f16": DeviceCase(gen.tiny_spec("paged_f16", B=2, L=1500, k=64, r=2, T=3, kv_dtype="f16"))}


def _views(ctx, dc, t, block_size, layout, seed=5):
    Kp, Vp, table = gen_device.paginate(dc.K, dc.V, block_size, seed=seed, layout=layout)
    sl = dc.seq_lens(t)
    return ctx.kv_view(dc.K, dc.V, sl), ctx.paged_kv_view(Kp, Vp, table, sl), (Kp, Vp, table)


def _bufs(dc):
    spec, case = dc.spec, dc.case
    idx = torch.full((spec.B, spec.Hq, case.kmax), -7, dtype=torch.int32, device=DEV)
    sc = torch.full((spec.B, spec.Hq, case.kmax), -7.0, dtype=torch.float32, device=DEV)
    out = torch.full((spec.B, spec.Hq, spec.D), -7.0, dtype=torch.float32, device=DEV)
    return idx, sc, out


@pytest.mark.parametrize("dtype,block_size,layout", LAYOUTS)
def test_every_entry_point_is_bit_identical_to_the_contiguous_cache(cases, dtype, block_size, layout):
    dc = cases[dtype]
    spec, case = dc.spec, dc.case
    ctx = dc.make_ctx()
    t = 2
    flat, paged, _keep = _views(ctx, dc, t, block_size, layout)
    q = dc.q(t)
    res = {}
    for name, kv in (("flat", flat), ("paged", paged)):
        r = {}
        idx, sc, out = _bufs(dc)
        ctx.lfps_exact_topk(q, kv, dc.k, idx, sc)
        r["exact_idx"], r["exact_sc"] = idx.clone(), sc.clone()
        ctx.lfps_full_attn_decode(q, kv, out)
        r["full"] = out.clone()
        # candidates from the exact Top-k, all candidate scores dumped
        cand = torch.zeros((spec.B, spec.Hkv, ctx.cand_cap), dtype=torch.int32, device=DEV)
        cnt = torch.zeros((spec.B, spec.Hkv), dtype=torch.int32, device=DEV)
        ctx.lfps_candidates(r["exact_idx"], dc.k, dc.seq_lens(t), cand, cnt)
        dump = torch.zeros((spec.B, spec.Hq, ctx.cand_cap), dtype=torch.float32, device=DEV)
        idx2, sc2, out2 = _bufs(dc)
        ctx.lfps_score_topk(q, kv, cand, cnt, dc.k, idx2, sc2, dump)
        c = cnt.cpu().numpy()
        for b in range(spec.B):          # entries past the count are not written
            for g in range(spec.Hkv):
                dump[b, g * spec.G:(g + 1) * spec.G, int(c[b, g]):] = 0
        r["st_idx"], r["st_sc"], r["dump"] = idx2, sc2, dump
        ctx.lfps_sparse_attn(q, kv, idx2, sc2, dc.k, out2)
        r["sparse"] = out2.clone()
        out3 = torch.zeros_like(out2)
        ctx.lfps_sparse_attn(q, kv, idx2, None, dc.k, out3)      # scores recomputed per head
        r["sparse_rescored"] = out3
        res[name] = r
    for key in res["flat"]:
        assert torch.equal(res["flat"][key], res["paged"][key]), f"{key} differs between the two layouts"
    # and the full attention is the oracle's (direct check of the paged read path)
    n = case.seq_lens(t)
    full = res["paged"]["full"].cpu().numpy()
    for b in range(spec.B):
        for h in (0, spec.Hq - 1):
            K, V = dc.group(b, h // spec.G)
            assert_out_close(full[b, h], orc.full_attn(case.q[t, b, h], K, V, int(n[b])), f"paged full b{b} h{h}")


@pytest.mark.parametrize("dtype,block_size,layout", LAYOUTS[:3] + LAYOUTS[5:6] + LAYOUTS[7:9])
def test_chained_steps_paged_equal_contiguous_and_oracle(cases, dtype, block_size, layout):
    """Free-running lfps_step chains (filtered scoring from the second step on) over both layouts give the
    same Top-k and outputs at every step; one more step on the paged view, started from the oracle's exact
    Top-k, is checked against the oracle."""
    dc = cases[dtype]
    spec, case = dc.spec, dc.case
    Kp, Vp, table = gen_device.paginate(dc.K, dc.V, block_size, seed=11, layout=layout)
    runs = {}
    for name in ("flat", "paged"):
        ctx = dc.make_ctx()
        view = (lambda t: ctx.kv_view(dc.K, dc.V, dc.seq_lens(t))) if name == "flat" else \
               (lambda t: ctx.paged_kv_view(Kp, Vp, table, dc.seq_lens(t)))
        prev = torch.zeros((spec.B, spec.Hq, case.kmax), dtype=torch.int32, device=DEV)
        ctx.lfps_exact_topk(dc.q(0), view(0), dc.k, prev)
        hist = []
        for t in range(1, spec.T + 1):
            idx, sc, out = _bufs(dc)
            ctx.lfps_step(dc.q(t), view(t), prev, dc.k, idx, out, sc)
            hist.append((prev.clone(), idx.clone(), sc.clone(), out.clone()))
            prev = idx
        runs[name] = hist
    for t, (a, b_) in enumerate(zip(runs["flat"], runs["paged"]), start=1):
        for what, x, y in zip(("prev", "idx", "score", "out"), a, b_):
            assert torch.equal(x, y), f"step {t}: {what} differs between the two layouts"
    # one teacher-forced step on the paged view against the oracle: the oracle's exact Top-k of step 0 is the history
    ctx = dc.make_ctx()
    G = spec.G
    groups = [(b, g) for b in range(spec.B) for g in (0, spec.Hkv - 1)]
    prev = np.full((spec.B, spec.Hq, case.kmax), -1, dtype=np.int32)
    for (b, g) in groups:
        K, _ = dc.group(b, g)
        for h in range(G * g, G * g + G):
            prev[b, h, : int(case.k[b])] = orc.exact_topk(case.q[0, b, h], K, int(case.seq_lens0[b]), int(case.k[b]))[0]
    idx, sc, out = _bufs(dc)
    ctx.lfps_step(dc.q(1), ctx.paged_kv_view(Kp, Vp, table, dc.seq_lens(1)), dev(prev), dc.k, idx, out, sc)
    idx, out = idx.cpu().numpy(), out.cpu().numpy()
    n = case.seq_lens(1)
    for (b, g) in groups:
        kb = int(case.k[b])
        K, V = dc.group(b, g)
        res = orc.lfps_step(case.q[1, b, G * g: G * g + G], K, V, [prev[b, G * g + h, :kb] for h in range(G)],
                            int(n[b]), kb, spec.r, 1, 0)
        for hh in range(G):
            h = G * g + hh
            assert_topk_equal_mod_ties(idx[b, h, :kb], res["topk_idx"][hh],
                                       lambda p: orc.scores(case.q[1, b, h], K, p), kb, f"paged step b{b} h{h}")
            assert_out_close(out[b, h], orc.sparse_attn(case.q[1, b, h], K, V, idx[b, h, :kb]), f"paged out b{b} h{h}")


def test_table_mode_and_bypass_paged_equal_contiguous(cases):
    """Score-table steps (Eq. 4 init from two queries, then steps), the prefill priors, the sparsity ratio
    and a gated step: identical over both layouts."""
    dc = cases["bf16"]
    spec, case = dc.spec, dc.case
    Kp, Vp, table = gen_device.paginate(dc.K, dc.V, 32, seed=3, layout="block_row_head")
    runs = {}
    for name in ("flat", "paged"):
        ctx = dc.make_ctx(table_mode=True, table_decay=0.9, table_a=0.2, n_sink=4, n_recent=1)
        view = (lambda t: ctx.kv_view(dc.K, dc.V, dc.seq_lens(t))) if name == "flat" else \
               (lambda t: ctx.paged_kv_view(Kp, Vp, table, dc.seq_lens(t)))
        r = []
        kbar = torch.zeros((spec.B, spec.Hkv, spec.D), dtype=torch.float32, device=DEV)
        vbar = torch.zeros_like(kbar)
        s2 = torch.zeros((spec.B, spec.Hq), dtype=torch.float32, device=DEV)
        ctx.lfps_priors(dc.q(0), view(0), kbar, vbar, s2)
        rho = torch.zeros((spec.B, spec.Hq), dtype=torch.float32, device=DEV)
        gate = torch.zeros((spec.B, spec.Hq), dtype=torch.int32, device=DEV)
        ctx.lfps_head_sparsity(dc.q(1), view(1), kbar, s2, 6, 0.5, rho, gate)
        r += [kbar, vbar, s2, rho, gate.clone()]
        ctx.lfps_tables_init(torch.stack([dc.q(1), dc.q(0)]), view(1))
        for t in (2, 3):
            idx, sc, out = _bufs(dc)
            ctx.lfps_table_step(dc.q(t), view(t), dc.k, idx, out, sc)
            r += [idx, sc, out]
        idx, sc, out = _bufs(dc)
        ctx.lfps_table_step_gated(dc.q(4), view(4), dc.k, kbar, vbar, s2, 6, 0.5, idx, out, sc, gate)
        r += [idx, sc, out, gate.clone()]
        ver = torch.zeros((spec.B, spec.Hq, case.Lcap), dtype=torch.float64, device=DEV)
        sla = torch.zeros_like(ver)
        ctx.lfps_tables_export(ver, sla, dc.seq_lens(4))
        r += [ver, sla]
        torch.cuda.synchronize()
        runs[name] = r
    for i, (x, y) in enumerate(zip(runs["flat"], runs["paged"])):
        assert torch.equal(x, y), f"result {i} differs between the two layouts"


def test_table_entries_outside_the_pool_are_clamped_and_unused_ones_ignored(cases):
    dc = cases["bf16"]
    spec, case = dc.spec, dc.case
    ctx = dc.make_ctx()
    t = 1
    bs = 64
    Kp, Vp, table = gen_device.paginate(dc.K, dc.V, bs, seed=9)
    q = dc.q(t)
    idx0, sc0, out0 = _bufs(dc)
    kv = ctx.paged_kv_view(Kp, Vp, table, dc.seq_lens(t))
    ctx.lfps_exact_topk(q, kv, dc.k, idx0, sc0)
    ctx.lfps_full_attn_decode(q, kv, out0)
    n = case.seq_lens(t)
    bad = table.clone()
    n_blocks = Kp.shape[0]
    last = n_blocks - 1
    for b in range(spec.B):
        used = (int(n[b]) + bs - 1) // bs
        bad[b, used:] = torch.tensor([2 ** 30, -5] * 64, dtype=torch.int32)[: bad.shape[1] - used].to(DEV)   # never read
    # an entry beyond the pool means the pool's last block: point a used entry there
    where = (table == last).nonzero()
    if len(where) == 1 and int(where[0][1]) < (int(n[int(where[0][0])]) + bs - 1) // bs:
        bad[int(where[0][0]), int(where[0][1])] = 2 ** 30
    else:                            # the last block is spare or unread: give it the data of request 0's first block
        first = int(table[0, 0])
        Kp[last] = Kp[first]
        Vp[last] = Vp[first]
        bad[0, 0] = 2 ** 30
    idx1, sc1, out1 = _bufs(dc)
    kv_bad = ctx.paged_kv_view(Kp, Vp, bad, dc.seq_lens(t))
    ctx.lfps_exact_topk(q, kv_bad, dc.k, idx1, sc1)
    ctx.lfps_full_attn_decode(q, kv_bad, out1)
    assert torch.equal(idx0, idx1) and torch.equal(sc0, sc1) and torch.equal(out0, out1)


def test_paged_view_argument_errors(cases):
    from paper_2506_15704_amd.binding import LfpsError, lfps_kv
    dc = cases["bf16"]
    spec = dc.spec
    ctx = dc.make_ctx()
    Kp, Vp, table = gen_device.paginate(dc.K, dc.V, 16, seed=1)
    good = ctx.paged_kv_view(Kp, Vp, table, dc.seq_lens(0))
    out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
    ctx.lfps_full_attn_decode(dc.q(0), good, out)            # the unmodified view is accepted

    def variant(**kw):
        v = lfps_kv(good.k, good.v, good.stride_b, good.stride_h, good.stride_n, good.seq_lens, good.block_table,
                    good.block_size, good.block_table_stride, good.n_blocks)
        for key, val in kw.items():
            setattr(v, key, val)
        return v

    for kw, text in (({"block_size": 24}, "power of two"), ({"block_size": 0}, "power of two"),
                     ({"block_size": 1 << 17}, "power of two"),
                     ({"block_table_stride": (dc.case.Lcap + 15) // 16 - 1}, "cover max_seq_len"),
                     ({"n_blocks": 0}, "n_blocks"), ({"n_blocks": 1 << 28}, "2^31")):
        with pytest.raises(LfpsError) as e:
            ctx.lfps_full_attn_decode(dc.q(0), variant(**kw), out)
        assert text in str(e.value), (kw, str(e.value))
    torch.cuda.synchronize()
