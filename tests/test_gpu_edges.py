"""Edge behaviour of the C ABI that the header promises: bad candidate entries, the fp16 query range,
switching the score filter on a context that was created with it off, and the count of rescored heads."""
import numpy as np
import pytest
import torch

import gen
from oracle import lfps_oracle as orc
from tests.harness import DEV, DeviceCase, assert_out_close, assert_scores_close, assert_topk_equal_mod_ties, dev, valid_row

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kv_dtype", ["bf16", "f32", "f16"])
def test_candidate_entries_outside_the_context_are_never_selected(kv_dtype):
    """cand holds entries < 0 and >= n_b between valid ones: they score -inf, so the Top-k is the oracle's over
    the valid entries; a group with fewer valid entries than k gets -1 where a bad entry would stand."""
    from paper_2506_15704_amd.binding import Lfps
    rng = np.random.default_rng(11)
    B, Hq, Hkv, D, Lcap, kmax = 2, 8, 2, 128, 700, 48
    n = np.array([650, 300], dtype=np.int32)
    K = rng.standard_normal((B, Hkv, Lcap, D)).astype(np.float32)
    tdt = {"bf16": torch.bfloat16, "f32": torch.float32, "f16": torch.float16}[kv_dtype]
    Kd = torch.from_numpy(K).to(tdt).to(DEV)
    Kf = Kd.float().cpu().numpy()
    q = rng.standard_normal((B, Hq, D)).astype(np.float32)
    ctx = Lfps(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, kv_dtype=kv_dtype, max_seq_len=Lcap, max_k=kmax, radius=1,
               cand_cap=Lcap)
    cand = np.zeros((B, Hkv, ctx.cand_cap), dtype=np.int32)
    cnt = np.zeros((B, Hkv), dtype=np.int32)
    lists = {}
    for b in range(B):
        for g in range(Hkv):
            c = 200 if (b, g) != (1, 1) else 60
            good = np.sort(rng.choice(int(n[b]), size=c, replace=False)).astype(np.int32)
            lst = good.copy()
            # (1, 1): only 30 valid entries, fewer than k = 48
            bad_at = rng.choice(c, size=c // 10 if (b, g) != (1, 1) else 30, replace=False)
            lst[bad_at] = rng.choice([-1, -7, int(n[b]), int(n[b]) + 5, Lcap + 100, 2 ** 30], size=len(bad_at))
            cand[b, g, :c] = lst
            cnt[b, g] = c
            lists[(b, g)] = lst
    k = np.array([kmax, kmax], dtype=np.int32)
    idx = torch.zeros((B, Hq, kmax), dtype=torch.int32, device=DEV)
    sc = torch.zeros((B, Hq, kmax), dtype=torch.float32, device=DEV)
    cs = torch.zeros((B, Hq, ctx.cand_cap), dtype=torch.float32, device=DEV)
    kv = ctx.kv_view(Kd, Kd, dev(n))
    ctx.lfps_score_topk(dev(q), kv, dev(cand), dev(cnt), dev(k), idx, sc, cs)
    out = torch.zeros((B, Hq, D), dtype=torch.float32, device=DEV)
    ctx.lfps_sparse_attn(dev(q), kv, idx, sc, dev(k), out)
    idx_h, sc_h, cs_h, out_h = idx.cpu().numpy(), sc.cpu().numpy(), cs.cpu().numpy(), out.cpu().numpy()
    G = Hq // Hkv
    for b in range(B):
        for g in range(Hkv):
            lst = lists[(b, g)]
            ok = (lst >= 0) & (lst < n[b])
            valid = lst[ok]
            for hh in range(G):
                h = G * g + hh
                # bad entries score -inf, the others as the oracle says
                assert np.all(np.isneginf(cs_h[b, h, : len(lst)][~ok]))
                assert_scores_close(cs_h[b, h, : len(lst)][ok], orc.scores(q[b, h], Kf[b, g], valid), f"b{b} h{h}")
                ksel = min(kmax, len(valid))
                want, _ = orc.score_topk(q[b, h], Kf[b, g], valid, ksel)
                row = idx_h[b, h, : min(kmax, len(lst))]
                got = valid_row(row)
                assert np.all(idx_h[b, h, min(kmax, len(lst)):] == -1)
                assert_topk_equal_mod_ties(got, want, lambda p: orc.scores(q[b, h], Kf[b, g], p), ksel, f"b{b} h{h}")
                assert np.all(sc_h[b, h][idx_h[b, h] < 0] == 0)
                assert_out_close(out_h[b, h], orc.sparse_attn(q[b, h], Kf[b, g], Kf[b, g], got), f"out b{b} h{h}")
    assert ctx.lfps_poll_status() == 0
    ctx.close()


def test_fp16_query_beyond_the_format_is_clamped_and_flagged():
    """An fp16 cache with a query element above 65504 (and an infinite one): the scoring kernels clamp it to the
    fp16 range, raise LFPS_FLAG_Q_RANGE, and the scores are those of the clamped query; queries inside the range
    raise nothing."""
    from paper_2506_15704_amd.binding import LFPS_FLAG_Q_RANGE, Lfps
    rng = np.random.default_rng(3)
    L, D, Hq = 320, 128, 4
    K = (rng.standard_normal((L, D)) * 1e-3).astype(np.float32)
    K16 = torch.from_numpy(K).to(torch.float16)
    Kf = K16.float().numpy()
    q = rng.standard_normal((1, Hq, D)).astype(np.float32)
    q[0, 1, 5] = 1.0e6
    q[0, 1, 77] = -3.0e5
    q[0, 2, 9] = np.inf
    q[0, 3] *= 6.0e4 / np.abs(q[0, 3]).max()             # large but inside the range
    qc = np.clip(q, -65504.0, 65504.0)
    ctx = Lfps(batch=1, n_q_heads=Hq, n_kv_heads=1, kv_dtype="f16", max_seq_len=L, max_k=16, radius=0, cand_cap=L)
    Kd = K16.reshape(1, 1, L, D).to(DEV)
    n = torch.tensor([L], dtype=torch.int32, device=DEV)
    kv = ctx.kv_view(Kd, Kd, n)
    cand = torch.arange(L, dtype=torch.int32, device=DEV).reshape(1, 1, L)
    cnt = torch.tensor([[L]], dtype=torch.int32, device=DEV)
    k = torch.tensor([16], dtype=torch.int32, device=DEV)
    idx = torch.zeros((1, Hq, 16), dtype=torch.int32, device=DEV)
    cs = torch.zeros((1, Hq, L), dtype=torch.float32, device=DEV)
    q_in = q.copy()
    q_in[0, 1:3] = qc[0, 1:3] * 0 + q[0, 3]              # first: every head inside the range -> no flag
    ctx.lfps_score_topk(dev(q_in), kv, cand, cnt, k, idx, None, cs)
    assert ctx.lfps_poll_status() == 0
    ctx.lfps_score_topk(dev(q), kv, cand, cnt, k, idx, None, cs)
    assert ctx.lfps_poll_status() == LFPS_FLAG_Q_RANGE
    cs_h, idx_h = cs.cpu().numpy(), idx.cpu().numpy()
    assert np.isfinite(cs_h).all()
    for h in range(Hq):
        assert_scores_close(cs_h[0, h], orc.scores(qc[0, h], Kf, np.arange(L)), f"clamped query h{h}")
        I, _ = orc.exact_topk(qc[0, h], Kf, L, 16)
        assert_topk_equal_mod_ties(idx_h[0, h], I, lambda p: orc.scores(qc[0, h], Kf, p), 16, f"clamped query h{h}")
    # the dense scoring pass (exact Top-k baseline) and the chained step report it too
    ctx.lfps_exact_topk(dev(q), kv, k, idx)
    assert ctx.lfps_poll_status() == LFPS_FLAG_Q_RANGE
    prev = idx.clone()
    nxt = torch.zeros_like(idx)
    out = torch.zeros((1, Hq, D), dtype=torch.float32, device=DEV)
    for _ in range(2):                                   # second call: through the filtered pass
        ctx.lfps_step(dev(q), kv, prev, k, nxt, out)
        assert ctx.lfps_poll_status() == LFPS_FLAG_Q_RANGE
    assert torch.isfinite(out).all()
    ctx.close()


def test_filter_switched_on_after_creation_with_a_large_budget():
    """A context whose budget is too large for the select's survivor list starts with the filter off; switching
    it on must still give the unfiltered result (a head whose survivors overflow the list is rescored), not a
    launch error."""
    spec = gen.tiny_spec("bigk", B=1, L=30000, k=14000, r=0, T=2, Hq=4, Hkv=1)
    dc = DeviceCase(spec)
    case = dc.case
    ref, flt = dc.make_ctx(), dc.make_ctx()
    flt.lfps_set_filter(True)
    flt.lfps_timing_enable(True)
    shp = (1, 4, case.kmax)
    seed = torch.zeros(shp, dtype=torch.int32, device=DEV)
    ref.lfps_exact_topk(dc.q(0), ref.kv_view(dc.K, dc.V, dc.seq_lens(0)), dc.k, seed)
    prev = seed
    for t in (1, 2):
        kv = ref.kv_view(dc.K, dc.V, dc.seq_lens(t))
        res = []
        for ctx in (ref, flt):
            idx = torch.zeros(shp, dtype=torch.int32, device=DEV)
            out = torch.zeros((1, 4, spec.D), dtype=torch.float32, device=DEV)
            ctx.lfps_step(dc.q(t), kv, prev, dc.k, idx, out)
            assert ctx.lfps_poll_status() == 0
            res.append((idx, out))
        assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])
        prev = res[0][0]
    assert ref.lfps_poll_rescored() == 0                  # no filtered pass, nothing to rescore
    tm = flt.lfps_timing_read()                           # the second step went through the filtered kernels
    assert tm["filter_score"][1] == 1 and tm["filter_select_attend"][1] == 1 and tm["select_attend"][1] == 1
    ref.close()
    flt.close()


def test_rescored_heads_are_counted():
    """The first step of a new context takes the unfiltered kernels (nothing is rescored); the following step
    of a slowly drifting query filters with the history that step left; a query scaled down by 100 makes that
    history useless and every head is rescored inside the select kernel; a reset starts over."""
    spec = gen.tiny_spec("resc", B=2, L=3000, k=96, r=2, T=4)
    dc = DeviceCase(spec)
    case = dc.case
    ctx = dc.make_ctx()
    shp = (spec.B, spec.Hq, case.kmax)
    a = torch.zeros(shp, dtype=torch.int32, device=DEV)
    b_ = torch.zeros_like(a)
    out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
    ctx.lfps_exact_topk(dc.q(0), ctx.kv_view(dc.K, dc.V, dc.seq_lens(0)), dc.k, a)
    assert ctx.lfps_poll_rescored() == 0
    ctx.lfps_step(dc.q(1), ctx.kv_view(dc.K, dc.V, dc.seq_lens(1)), a, dc.k, b_, out)
    assert ctx.lfps_poll_rescored() == 0
    ctx.lfps_step(dc.q(2), ctx.kv_view(dc.K, dc.V, dc.seq_lens(2)), b_, dc.k, a, out)
    few = ctx.lfps_poll_rescored()
    assert few < spec.B * spec.Hq // 4, few
    ctx.lfps_step(dc.q(3) * 0.01, ctx.kv_view(dc.K, dc.V, dc.seq_lens(3)), a, dc.k, b_, out)
    assert ctx.lfps_poll_rescored() == spec.B * spec.Hq
    ctx.lfps_reset_history()
    ctx.lfps_step(dc.q(4), ctx.kv_view(dc.K, dc.V, dc.seq_lens(4)), b_, dc.k, a, out)
    assert ctx.lfps_poll_rescored() == 0
    assert ctx.lfps_poll_status() == 0
    ctx.close()


@pytest.mark.parametrize("variant", ["bf16", "fp8", "ragged_small_k", "paged"])
def test_exact_topk_filtered_form_equals_plain_form(variant):
    """Contexts of a million rows and more take the exact Top-k baseline through a sampled threshold and the
    filtered scoring pass; with the filter switched off the same context scores and selects the plain way.  Both
    must return the same rows and scores for every head (ascending positions, ties to the lower position), and
    sampled heads are checked against the oracle."""
    kw = dict(B=4, L=33000, k=512, r=1, T=1, n_hot=8, recency=32)
    if variant == "fp8":
        kw.update(k_dtype="fp8")
    if variant == "ragged_small_k":
        kw.update(L=None, L_range=(20000, 40000), k=None, k_frac=0.004, B=6)
    spec = gen.tiny_spec("xfast_" + variant, **kw)
    dc = DeviceCase(spec)
    case = dc.case
    assert spec.B * spec.Hkv * case.Lcap >= 1 << 20
    fast, plain = dc.make_ctx(), dc.make_ctx()
    plain.lfps_set_filter(False)
    shp = (spec.B, spec.Hq, case.kmax)
    if variant == "paged":
        from gen import device as gen_device
        Kp, Vp, bt = gen_device.paginate(dc.K, dc.V, 32, seed=5, layout="block_head_row")
        view = lambda ctx: ctx.paged_kv_view(Kp, Vp, bt, dc.seq_lens(1))
    else:
        view = lambda ctx: ctx.kv_view(dc.K, dc.V, dc.seq_lens(1))
    res = []
    for ctx in (fast, plain):
        ctx.lfps_timing_enable(True)
        idx = torch.zeros(shp, dtype=torch.int32, device=DEV)
        sc = torch.zeros(shp, dtype=torch.float32, device=DEV)
        ctx.lfps_exact_topk(dc.q(1), view(ctx), dc.k, idx, sc)
        tm = ctx.lfps_timing_read()
        assert ctx.lfps_poll_status() == 0
        res.append((idx, sc, tm))
    assert res[0][2]["filter_score"][1] == 1 and res[1][2]["filter_score"][1] == 0     # the two forms did run
    assert torch.equal(res[0][0], res[1][0])
    assert torch.equal(res[0][1], res[1][1])
    # without the scores output as well
    idx2 = torch.zeros(shp, dtype=torch.int32, device=DEV)
    fast.lfps_exact_topk(dc.q(1), view(fast), dc.k, idx2)
    assert torch.equal(idx2, res[0][0])
    idx_h = res[0][0].cpu().numpy()
    n = case.seq_lens(1)
    for (b, g) in ((0, 0), (spec.B - 1, 5)):
        K, _ = dc.group(b, g)
        kb = int(case.k[b])
        for hh in range(spec.G):
            h = spec.G * g + hh
            I, _ = orc.exact_topk(case.q[1, b, h], K, int(n[b]), kb)
            assert_topk_equal_mod_ties(idx_h[b, h, :kb], I, lambda p: orc.scores(case.q[1, b, h], K, p), kb,
                                       f"{variant} b{b} h{h}")
            assert np.all(idx_h[b, h, kb:] == -1)
    fast.close()
    plain.close()


@pytest.mark.parametrize("fmt", ["bf16", "fp8kv", "f32"])
def test_host_resident_cache_gives_identical_results(fmt):
    """The paper's placement: K and V stay in (pinned) host memory and the kernels fetch the rows they touch over
    the host link.  Same entry points, same kernels; every result must equal the device-resident run bit for bit
    (exact Top-k seed, three chained steps through the filtered pass, full attention, a score-table step)."""
    kw = dict(B=2, L=2200, k=80, r=2, T=3)
    if fmt == "fp8kv":
        kw.update(k_dtype="fp8", v_dtype="fp8")
    if fmt == "f32":
        kw.update(kv_dtype="f32")
    spec = gen.tiny_spec("hostkv_" + fmt, **kw)
    dc = DeviceCase(spec)
    case = dc.case

    def pinned(t):
        raw = t.view(torch.uint8) if t.dtype == torch.float8_e4m3fn else t
        h = torch.empty(raw.shape, dtype=raw.dtype, pin_memory=True)
        h.copy_(raw)
        return h.view(t.dtype) if t.dtype == torch.float8_e4m3fn else h

    Kh, Vh = pinned(dc.K), pinned(dc.V)
    assert Kh.is_pinned() and not Kh.is_cuda
    shp = (spec.B, spec.Hq, case.kmax)
    runs = []
    for K, V in ((dc.K, dc.V), (Kh, Vh)):
        ctx = dc.make_ctx()
        tab = dc.make_ctx(table_mode=True, table_decay=0.9, table_a=0.2, n_sink=2)
        got = []
        prev = torch.zeros(shp, dtype=torch.int32, device=DEV)
        ctx.lfps_exact_topk(dc.q(0), ctx.kv_view(K, V, dc.seq_lens(0)), dc.k, prev)
        got.append(prev.clone())
        for t in (1, 2, 3):
            idx = torch.zeros(shp, dtype=torch.int32, device=DEV)
            sc = torch.zeros(shp, dtype=torch.float32, device=DEV)
            out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
            ctx.lfps_step(dc.q(t), ctx.kv_view(K, V, dc.seq_lens(t)), prev, dc.k, idx, out, sc)
            got += [idx, sc, out]
            prev = idx
        full = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
        ctx.lfps_full_attn_decode(dc.q(3), ctx.kv_view(K, V, dc.seq_lens(3)), full)
        got.append(full)
        tab.lfps_tables_init(dc.q(0), tab.kv_view(K, V, dc.seq_lens(0)))
        t_idx = torch.zeros(shp, dtype=torch.int32, device=DEV)
        t_out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
        tab.lfps_table_step(dc.q(1), tab.kv_view(K, V, dc.seq_lens(1)), dc.k, t_idx, t_out)
        got += [t_idx, t_out]
        torch.cuda.synchronize()
        assert ctx.lfps_poll_status() == 0 and tab.lfps_poll_status() == 0
        runs.append(got)
        ctx.close()
        tab.close()
    for i, (a, b_) in enumerate(zip(*runs)):
        assert torch.equal(a, b_), f"result {i} differs between the device-resident and the host-resident cache"
    # and one oracle check of the host-resident run itself
    K0, V0 = dc.group(1, 3)
    idx3, out3 = runs[1][7].cpu().numpy(), runs[1][9].cpu().numpy()
    h = 4 * 3 + 1
    ref = orc.sparse_attn(case.q[3, 1, h], K0, V0, idx3[1, h, : int(case.k[1])])
    assert_out_close(out3[1, h], ref, "host-resident step 3")
