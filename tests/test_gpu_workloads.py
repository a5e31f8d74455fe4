"""Full-size parity on the five benchmark workloads, in the launch configuration bench.py times
(same context parameters, same cache layout, same entry point), on sampled (request, KV group)
pairs the oracle recomputes one by one from regenerated rows.  Teacher-forced: before each step
the sampled groups' previous Top-k rows are replaced by the oracle's own."""
import numpy as np
import pytest
import torch

import bench
from oracle import lfps_oracle as orc
import gen
from tests.harness import DEV, DeviceCase, assert_out_close, assert_scores_close, assert_topk_equal_mod_ties, dev, valid_row

pytestmark = pytest.mark.gpu

SAMPLES = {
    "C1": [(0, 0), (0, 5), (0, 7)],
    "C2": [(0, 1), (0, 6)],
    "C3": [(2, 0), (7, 7)],
    "C4": [(0, 3), (15, 4)],
    "C5": None,     # chosen below: the shortest and the longest request
}


VARIANTS = {"C4-fp8k": dict(k_dtype="fp8"), "C4-fp8kv": dict(k_dtype="fp8", v_dtype="fp8"), "C4-f16": dict(kv_dtype="f16"),
            "C4-paged16": dict(paged_block=16), "C5-paged64": dict(paged_block=64, paged_layout="block_row_head")}


def _ragged_samples(case):
    """Four requests of a ragged batch: the shortest, the longest and two in between (at one and two thirds of
    the requests sorted by length), each with another KV group."""
    order = np.argsort(case.seq_lens0, kind="stable")
    nb = len(order)
    return [(int(order[0]), 2), (int(order[nb // 3]), 0), (int(order[(2 * nb) // 3]), 5), (int(order[-1]), 6)]


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"] + sorted(VARIANTS))
def test_workload_steps_match_oracle_on_sampled_groups(name):
    """The benchmark's workloads at full size, in the launch configuration bench.py times (also with the cache
    in the other formats and as a paged pool): steps teacher-forced on sampled KV groups against the oracle."""
    variant = VARIANTS.get(name, {})
    name = name.split("-")[0]
    r = bench.Runner(name, **variant)
    try:
        spec, case = r.spec, r.case
        G = spec.G
        samples = SAMPLES[name] or _ragged_samples(case)
        kv_cpu = {bg: case.kv_group(*bg) for bg in samples}
        # seeding step: device exact Top-k vs oracle exact Top-k
        seed = r.seed.cpu().numpy()
        prev_orc = {}
        for (b, g) in samples:
            K, _ = kv_cpu[(b, g)]
            kb, n0 = int(case.k[b]), int(case.seq_lens0[b])
            rows = []
            for hh in range(G):
                h = G * g + hh
                I, _ = orc.exact_topk(case.q[0, b, h], K, n0, kb)
                assert_topk_equal_mod_ties(seed[b, h, :kb], I, lambda p: orc.scores(case.q[0, b, h], K, p), kb,
                                           f"{name} seed b{b} h{h}")
                rows.append(I)
            prev_orc[(b, g)] = rows
        n_steps = 3 if name != "C1" else spec.T
        prev_dev = r.seed.clone()
        out = torch.zeros_like(r.out)
        sc = torch.zeros_like(r.sel_score)
        for t in range(1, n_steps + 1):
            for (b, g) in samples:                               # teacher forcing on the sampled groups
                for hh in range(G):
                    row = np.full(case.kmax, -1, dtype=np.int32)
                    row[: len(prev_orc[(b, g)][hh])] = prev_orc[(b, g)][hh]
                    prev_dev[b, G * g + hh] = torch.from_numpy(row).to(prev_dev.device)
            nxt = torch.zeros_like(prev_dev)
            r.ctx.lfps_step(r.q[t], r.views[t], prev_dev, r.k, nxt, out, sc)
            idx_h, out_h, sc_h = nxt.cpu().numpy(), out.cpu().numpy(), sc.cpu().numpy()
            for (b, g) in samples:
                K, V = kv_cpu[(b, g)]
                kb, n = int(case.k[b]), int(case.seq_lens(t)[b])
                res = orc.lfps_step(case.q[t, b, G * g: G * g + G], K, V, prev_orc[(b, g)], n, kb, spec.r, 1, 0)
                for hh in range(G):
                    h = G * g + hh
                    got = idx_h[b, h, :kb]
                    assert np.all(idx_h[b, h, kb:] == -1)
                    assert set(got.tolist()) <= set(res["cand"].tolist()), "selected rows must be candidates"
                    nd = assert_topk_equal_mod_ties(got, res["topk_idx"][hh], lambda p: orc.scores(case.q[t, b, h], K, p),
                                                    kb, f"{name} t{t} b{b} h{h}")
                    assert_scores_close(sc_h[b, h, :kb], orc.scores(case.q[t, b, h], K, got), f"{name} t{t} b{b} h{h}")
                    assert_out_close(out_h[b, h], orc.sparse_attn(case.q[t, b, h], K, V, got), f"{name} out t{t} b{b} h{h}")
                    if nd == 0:
                        assert_out_close(out_h[b, h], res["out"][hh], f"{name} out t{t} b{b} h{h}")
                prev_orc[(b, g)] = res["topk_idx"]
            prev_dev = nxt
        # baselines at full size on the same sampled groups
        t = n_steps
        full = torch.zeros_like(r.out)
        r.ctx.lfps_full_attn_decode(r.q[t], r.views[t], full)
        full_h = full.cpu().numpy()
        for (b, g) in samples:
            K, V = kv_cpu[(b, g)]
            for hh in (0, G - 1):
                h = G * g + hh
                assert_out_close(full_h[b, h], orc.full_attn(case.q[t, b, h], K, V, int(case.seq_lens(t)[b])),
                                 f"{name} full b{b} h{h}")
    finally:
        r.close()


def test_drift_spike_step_at_full_size_goes_through_the_rescoring_pass():
    """The workload with a query drift of 0.5 on every 16th step, at full size in the benchmark's launch
    configuration: the device chain runs freely through steps 1-14 (so the score filter has its history), the
    oracle chain of two sampled KV groups starts at step 14 from the oracle's exact Top-k, and steps 15, 16 (the
    spike) and 17 are teacher-forced against the oracle.  The spike must send heads through the unfiltered
    rescoring pass (the filter's remembered k-th score is of no use for a query that moved that far)."""
    name = "C3"
    r = bench.Runner(name)
    try:
        spec, case = r.spec, r.case
        G = spec.G
        assert spec.spike_every == 16 and spec.T >= 17
        samples = SAMPLES[name]
        kv_cpu = {bg: case.kv_group(*bg) for bg in samples}
        r.reset()
        r.ctx.lfps_reset_history()
        for _ in range(14):
            r.step()
        assert r.t == 14
        prev_dev = r.prev.clone()
        prev_orc = {}
        for (b, g) in samples:                               # the oracle's own history at t = 14
            K, _ = kv_cpu[(b, g)]
            kb, n14 = int(case.k[b]), int(case.seq_lens(14)[b])
            prev_orc[(b, g)] = [orc.exact_topk(case.q[14, b, G * g + hh], K, n14, kb)[0] for hh in range(G)]
        r.ctx.lfps_poll_rescored()                           # clears the count
        out = torch.zeros_like(r.out)
        sc = torch.zeros_like(r.sel_score)
        rescored = {}
        for t in (15, 16, 17):
            for (b, g) in samples:                           # teacher forcing on the sampled groups
                for hh in range(G):
                    row = np.full(case.kmax, -1, dtype=np.int32)
                    row[: len(prev_orc[(b, g)][hh])] = prev_orc[(b, g)][hh]
                    prev_dev[b, G * g + hh] = torch.from_numpy(row).to(prev_dev.device)
            nxt = torch.zeros_like(prev_dev)
            r.ctx.lfps_step(r.q[t], r.views[t], prev_dev, r.k, nxt, out, sc)
            rescored[t] = r.ctx.lfps_poll_rescored()
            assert r.ctx.lfps_poll_status() == 0
            idx_h, out_h, sc_h = nxt.cpu().numpy(), out.cpu().numpy(), sc.cpu().numpy()
            for (b, g) in samples:
                K, V = kv_cpu[(b, g)]
                kb, n = int(case.k[b]), int(case.seq_lens(t)[b])
                res = orc.lfps_step(case.q[t, b, G * g: G * g + G], K, V, prev_orc[(b, g)], n, kb, spec.r, 1, 0)
                for hh in range(G):
                    h = G * g + hh
                    got = idx_h[b, h, :kb]
                    assert set(got.tolist()) <= set(res["cand"].tolist()), "selected rows must be candidates"
                    nd = assert_topk_equal_mod_ties(got, res["topk_idx"][hh], lambda p: orc.scores(case.q[t, b, h], K, p),
                                                    kb, f"{name} t{t} b{b} h{h}")
                    assert_scores_close(sc_h[b, h, :kb], orc.scores(case.q[t, b, h], K, got), f"{name} t{t} b{b} h{h}")
                    assert_out_close(out_h[b, h], orc.sparse_attn(case.q[t, b, h], K, V, got), f"{name} out t{t} b{b} h{h}")
                    if nd == 0:
                        assert_out_close(out_h[b, h], res["out"][hh], f"{name} out t{t} b{b} h{h}")
                prev_orc[(b, g)] = res["topk_idx"]
            prev_dev = nxt
        heads = spec.B * spec.Hq
        # step 16 carries the drift of 0.5: the rescoring launches had work to do, for most heads; the ordinary
        # steps around it keep (almost) every head on the filtered path
        print(f"rescored heads of {heads}: {rescored}", flush=True)
        assert rescored[16] > 0 and rescored[16] > rescored[15], rescored
        assert rescored[15] < heads // 8, rescored
    finally:
        r.close()


def test_candidate_counts_and_capacity_at_full_size():
    """Properties that hold at any size: counts within [k, min(n, G k (2r+2) + 1)], ascending unique
    positions inside [0, n), previous Top-k contained in the candidates, no overflow flag."""
    r = bench.Runner("C5")
    try:
        spec, case = r.spec, r.case
        cnt = torch.zeros((spec.B, spec.Hkv), dtype=torch.int32, device=r.dev)
        r.ctx.lfps_candidates(r.seed, r.k, r.seq[1], r.cand, cnt)
        assert r.ctx.lfps_poll_status() == 0
        cnt_h, cand_h, seed = cnt.cpu().numpy(), r.cand.cpu().numpy(), r.seed.cpu().numpy()
        for b in range(spec.B):
            kb, n = int(case.k[b]), int(case.seq_lens(1)[b])
            for g in range(spec.Hkv):
                c = int(cnt_h[b, g])
                assert kb <= c <= min(n, spec.G * kb * (2 * spec.r + 2) + 1)
                C = cand_h[b, g, :c]
                assert np.all(np.diff(C) > 0) and C[0] >= 0 and C[-1] == n - 1
                for hh in range(spec.G):
                    assert np.isin(seed[b, spec.G * g + hh, :kb], C).all()
    finally:
        r.close()


def test_worst_case_candidate_count_at_full_size():
    """Maximum sizes: the four heads of every group disagree completely (random previous Top-k), so the
    candidate set approaches its capacity G*k*(2r+2)+1 = 81921 at the 128K workload; the score filter has
    no usable history, and the select streams more scores than its LDS cache holds."""
    r = bench.Runner("C4")
    try:
        spec, case = r.spec, r.case
        G = spec.G
        rng = np.random.default_rng(7)
        n = int(case.seq_lens(1)[0])
        prev = np.stack([np.stack([np.sort(rng.choice(n - 1, size=case.kmax, replace=False)).astype(np.int32)
                                   for _ in range(spec.Hq)]) for _ in range(spec.B)])
        samples = [(3, 5), (12, 0)]
        nxt = torch.zeros_like(r.seed)
        sc = torch.zeros_like(r.sel_score)
        out = torch.zeros_like(r.out)
        cnt = torch.zeros((spec.B, spec.Hkv), dtype=torch.int32, device=r.dev)
        for attempt in range(2):                     # second call: a history exists but is useless for these inputs
            r.ctx.lfps_step(r.q[1], r.views[1], torch.from_numpy(prev).to(r.dev), r.k, nxt, out, sc)
        r.ctx.lfps_copy_cand_count(cnt)
        assert r.ctx.lfps_poll_status() == 0
        cnt_h, idx_h, out_h = cnt.cpu().numpy(), nxt.cpu().numpy(), out.cpu().numpy()
        assert cnt_h.min() > 60000 and cnt_h.max() <= r.ctx.cand_cap
        for (b, g) in samples:
            K, V = case.kv_group(b, g)
            kb = int(case.k[b])
            res = orc.lfps_step(case.q[1, b, G * g: G * g + G], K, V, [prev[b, G * g + i] for i in range(G)], n, kb, spec.r, 1, 0)
            assert len(res["cand"]) == cnt_h[b, g]
            for hh in range(G):
                h = G * g + hh
                assert_topk_equal_mod_ties(idx_h[b, h, :kb], res["topk_idx"][hh], lambda p: orc.scores(case.q[1, b, h], K, p),
                                           kb, f"worst case b{b} h{h}")
                assert_out_close(out_h[b, h], orc.sparse_attn(case.q[1, b, h], K, V, idx_h[b, h, :kb]), f"worst case out b{b} h{h}")
    finally:
        r.close()


@pytest.mark.parametrize("name", ["C2", "C4", "C5"])
def test_score_table_mode_at_full_size_on_sampled_groups(name):
    """The score-table form (Eq. 4 start, Eq. 7-10 steps) in the configuration bench.py times: tables are
    compared with the oracle's Eq. 4 start, and for sampled (request, KV group) pairs the oracle runs the steps
    from its own tables, which the device is given before every step (teacher forcing)."""
    from oracle import lfps_tables_oracle as tor
    from tests.test_gpu_tables import _assert_candidates, assert_tables_close, oracle_on_candidates
    r = bench.Runner(name, table_mode=True, n_sink=4)
    try:
        spec, case = r.spec, r.case
        G, gamma, a, n_sink, n_recent = spec.G, 0.95, 0.2, 4, 1
        samples = SAMPLES[name] or _ragged_samples(case)[::3]
        kv_cpu = {bg: case.kv_group(*bg) for bg in samples}
        shp = (spec.B, spec.Hq, case.Lcap)
        ev = torch.zeros(shp, dtype=torch.float64, device=r.dev)
        es = torch.zeros_like(ev)
        r.ctx.lfps_tables_init(r.q[0], r.views[0])
        r.ctx.lfps_tables_export(ev, es, r.seq[0])
        orc_tab = {}                                         # the oracle's tables of the sampled groups (fp64, per head)
        for (b, g) in samples:                               # Eq. 4 with one query
            K, _ = kv_cpu[(b, g)]
            n0 = int(case.seq_lens0[b])
            orc_tab[(b, g)] = []
            for hh in range(G):
                h = G * g + hh
                s0 = orc.scores(case.q[0, b, h], K[:n0])
                w = np.zeros(n0)
                e = np.exp(s0[n_sink:] - s0[n_sink:].max())
                w[n_sink:] = e / e.sum()
                # one query: both tables are w / (2 (1 - gamma)); the oracle's loop form is used where it is affordable
                ver = tor.init_tables(w[None, :], gamma, n_sink)[0] if n0 <= 4096 else w / (2 * (1 - gamma))
                np.testing.assert_allclose(ev[b, h, :n0].cpu().numpy(), ver, rtol=3e-5, atol=1e-12)
                np.testing.assert_allclose(es[b, h, :n0].cpu().numpy(), ver, rtol=3e-5, atol=1e-12)
                orc_tab[(b, g)].append((ver.copy(), ver.copy()))
        idx = torch.zeros_like(r.seed)
        sc = torch.zeros_like(r.sel_score)
        out = torch.zeros_like(r.out)
        cnt = torch.zeros((spec.B, spec.Hkv), dtype=torch.int32, device=r.dev)
        for t in (1, 2):
            n_t = case.seq_lens(t)
            # Teacher forcing: the device's tables (all heads, as exported) with the sampled groups' heads replaced
            # by the oracle's, rounded to the fp32 the device stores; the oracle continues from the same rounded values.
            v32, s32 = ev.to(torch.float32), es.to(torch.float32)
            before = {}
            for (b, g) in samples:
                before[(b, g)] = []
                for hh in range(G):
                    h = G * g + hh
                    pair = []
                    for dst, src in ((v32, orc_tab[(b, g)][hh][0]), (s32, orc_tab[(b, g)][hh][1])):
                        row = np.zeros(case.Lcap, dtype=np.float32)
                        row[: len(src)] = src[: case.Lcap]
                        dst[b, h] = torch.from_numpy(row).to(r.dev)
                        pair.append(row.astype(np.float64))
                    before[(b, g)].append(tuple(pair))
            r.ctx.lfps_tables_import(v32, s32, r.seq[t])
            r.ctx.lfps_table_candidates(r.seq[t], r.cand, cnt)
            r.ctx.lfps_table_step(r.q[t], r.views[t], r.k, idx, out, sc)
            assert r.ctx.lfps_poll_status() == 0
            r.ctx.lfps_tables_export(ev, es, r.seq[min(t + 1, spec.T)])
            cnt_h, idx_h, out_h = cnt.cpu().numpy(), idx.cpu().numpy(), out.cpu().numpy()
            for (b, g) in samples:
                K, V = kv_cpu[(b, g)]
                n, kb = int(n_t[b]), int(case.k[b])
                t64 = before[(b, g)]
                res = tor.table_step(case.q[t, b, G * g: G * g + G], K, V, t64, n, kb, spec.r, a, gamma, n_recent, n_sink)
                orc_tab[(b, g)] = res["tables"]
                got_c = r.cand[b, g, : int(cnt_h[b, g])].cpu().numpy()
                nd = _assert_candidates(got_c, res["cand"], t64, n, a, spec.r, n_sink, f"{name} t{t} b{b} g{g}")
                assert nd <= 2
                if nd:                                       # a band-explained difference: the oracle's select and Eq. 10 on the device's set
                    res = oracle_on_candidates(case.q[t, b, G * g: G * g + G], K, got_c, t64, n, kb, gamma, n_sink)
                ksel = min(kb, len(got_c))
                for hh in range(G):
                    h = G * g + hh
                    got = idx_h[b, h, :ksel]
                    assert np.all(idx_h[b, h, ksel:] == -1)
                    assert_topk_equal_mod_ties(got, res["topk_idx"][hh], lambda p: orc.scores(case.q[t, b, h], K, p), ksel,
                                               f"{name} t{t} b{b} h{h}")
                    assert_out_close(out_h[b, h], orc.sparse_attn(case.q[t, b, h], K, V, got), f"{name} out t{t} b{b} h{h}")
                    if set(got.tolist()) == set(res["topk_idx"][hh].tolist()):      # Eq. 10 on the same selection
                        wv, ws = res["tables"][hh]
                        m = min(n + 1, case.Lcap)
                        old_v = np.r_[gamma * t64[hh][0][:n], 0.0][:m]
                        old_s = np.r_[0.0, gamma * t64[hh][1][:n]][:m]
                        half = 10 * 0.5 / max(ksel - n_sink, 1)
                        assert_tables_close(ev[b, h, :m].cpu().numpy(), wv[:m], old_v, half, f"{name} vertical t{t} b{b} h{h}")
                        assert_tables_close(es[b, h, :m].cpu().numpy(), ws[:m], old_s, half, f"{name} slash t{t} b{b} h{h}")
    finally:
        r.close()


def test_largest_supported_context():
    """max_seq_len at the capacity of the candidate bitmap (720 896 rows): one KV group, seeded by the exact
    Top-k, then chained steps (the second and third through the score filter) and one score-table step,
    against the oracle."""
    from oracle import lfps_tables_oracle as tor
    from tests.test_gpu_tables import _assert_candidates
    Lcap = 88 * 1024 * 8
    T = 3
    spec = gen.tiny_spec("maxlen", B=1, L=Lcap - T, k=2048, r=4, T=T, Hq=4, Hkv=1, n_hot=16, recency=64)
    dc = DeviceCase(spec)
    case = dc.case
    assert case.Lcap == Lcap
    from paper_2506_15704_amd.binding import LfpsError, workspace_bytes
    with pytest.raises(LfpsError):
        workspace_bytes(batch=1, n_q_heads=4, n_kv_heads=1, head_dim=128, kv_dtype=1, max_seq_len=Lcap + 1, max_k=2048,
                        radius=4, n_recent=1, n_sink=0, cand_cap=0, device=0)
    ctx = dc.make_ctx()
    # the oracle's inputs: every K row (regenerated on the CPU in chunks), V rows only where they are read
    K = np.empty((Lcap, spec.D), dtype=np.float32)
    for r0 in range(0, Lcap, 65536):
        rows = np.arange(r0, min(Lcap, r0 + 65536))
        K[r0:r0 + len(rows)] = case.kv_rows("k", 0, 0, rows)[0]
    V = np.zeros((Lcap, spec.D), dtype=np.float32)

    def need_v(rows):
        rows = np.unique(np.asarray(rows).ravel())
        rows = rows[(rows >= 0) & (rows < Lcap)]
        V[rows] = case.kv_rows("v", 0, 0, rows)[0]

    shp = (1, 4, case.kmax)
    seed = torch.zeros(shp, dtype=torch.int32, device=DEV)
    ctx.lfps_exact_topk(dc.q(0), ctx.kv_view(dc.K, dc.V, dc.seq_lens(0)), dc.k, seed)
    p0 = seed.cpu().numpy()
    p_h = np.zeros(shp, dtype=np.int32)                   # the oracle's Top-k: the history the device is given
    for h in range(4):                                    # 720 896 fp64 dot products per head
        I, _ = orc.exact_topk(case.q[0, 0, h], K, int(case.seq_lens0[0]), 2048)
        assert_topk_equal_mod_ties(p0[0, h], I, lambda p: orc.scores(case.q[0, 0, h], K, p), 2048, f"exact h{h}")
        p_h[0, h] = I
    for t in range(1, T + 1):
        idx = torch.zeros(shp, dtype=torch.int32, device=DEV)
        out = torch.zeros((1, 4, spec.D), dtype=torch.float32, device=DEV)
        ctx.lfps_step(dc.q(t), ctx.kv_view(dc.K, dc.V, dc.seq_lens(t)), dev(p_h), dc.k, idx, out)
        assert ctx.lfps_poll_status() == 0
        i_h, o_h = idx.cpu().numpy(), out.cpu().numpy()
        n = int(case.seq_lens(t)[0])
        cand_rows = np.unique(np.concatenate([p_h[0, h][:, None] + np.arange(-spec.r, spec.r + 2)[None, :] for h in range(4)]))
        need_v(np.concatenate([cand_rows, [n - 1], i_h.ravel()]))
        res = orc.lfps_step(case.q[t, 0], K, V, [p_h[0, h] for h in range(4)], n, 2048, spec.r, 1, 0)
        for h in range(4):
            assert_topk_equal_mod_ties(i_h[0, h], res["topk_idx"][h], lambda p: orc.scores(case.q[t, 0, h], K, p), 2048,
                                       f"t{t} h{h}")
            assert_out_close(o_h[0, h], orc.sparse_attn(case.q[t, 0, h], K, V, i_h[0, h]), f"t{t} h{h}")
        p_h = np.stack(res["topk_idx"])[None].astype(np.int32)
    ctx.close()
    # one score-table step at the same length: Eq. 4 start from the step-0 query (the oracle's tables for the
    # expectation, the device's own for the device), then a step
    tab = dc.make_ctx(table_mode=True, table_decay=0.95, table_a=0.2, n_sink=4, n_recent=1)
    tab.lfps_tables_init(dc.q(0), tab.kv_view(dc.K, dc.V, dc.seq_lens(0)))
    n0 = int(case.seq_lens0[0])
    t64 = []
    for h in range(4):
        sc0 = orc.scores(case.q[0, 0, h], K[:n0])
        w = np.zeros(n0)
        e = np.exp(sc0[4:] - sc0[4:].max())
        w[4:] = e / e.sum()                                  # attention weights of the query over the non-sink rows
        # Eq. 4 with one query: both tables hold w / (2 (1 - gamma)) (written out; the oracle's loop form is
        # checked against the device at small sizes)
        tab0 = np.r_[w / (2.0 * (1.0 - 0.95)), np.zeros(Lcap - n0)]
        t64.append((tab0.copy(), tab0.copy()))
    idx = torch.zeros(shp, dtype=torch.int32, device=DEV)
    out = torch.zeros((1, 4, spec.D), dtype=torch.float32, device=DEV)
    cnt = torch.zeros((1, 1), dtype=torch.int32, device=DEV)
    cand = torch.zeros((1, 1, tab.cand_cap), dtype=torch.int32, device=DEV)
    tab.lfps_table_candidates(dc.seq_lens(1), cand, cnt)
    tab.lfps_table_step(dc.q(1), tab.kv_view(dc.K, dc.V, dc.seq_lens(1)), dc.k, idx, out)
    n1 = int(case.seq_lens(1)[0])
    i_h, o_h = idx.cpu().numpy(), out.cpu().numpy()
    need_v(i_h)
    cand_o = tor.group_candidates(t64, n1, 0.2, spec.r, 1, 4)
    cand_d = cand[0, 0, : int(cnt[0, 0])].cpu().numpy()
    # bit-exact except positions explained by a table entry within 1e-5 (relative) of a threshold or mean
    nd = _assert_candidates(cand_d, cand_o, t64, n1, 0.2, spec.r, 4, "table candidates at the largest context")
    assert nd <= max(4, len(cand_o) // 1000), (nd, len(cand_o))
    for h in range(4):
        got = valid_row(i_h[0, h])
        # the oracle's select over the set the device used (its own set when the two are equal)
        ksel = min(2048, len(cand_d))
        want, _ = orc.score_topk(case.q[1, 0, h], K, cand_d, ksel)
        assert_topk_equal_mod_ties(got, want, lambda p: orc.scores(case.q[1, 0, h], K, p), ksel, f"table step h{h}")
        assert_out_close(o_h[0, h], orc.sparse_attn(case.q[1, 0, h], K, V, got), f"table step h{h}")
    assert tab.lfps_poll_status() == 0
    tab.close()
