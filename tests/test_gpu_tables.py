"""LFPS with score tables (Eq. 4, 7-10; Alg. 1 lines 5-9): HIP path vs the CPU oracle through the C ABI.

Table values are exchanged as true per-position values (import fp32 / export fp64), so both sides can be
started from exactly the same tables.  Comparison rules:
  * candidate sets: bit-exact, except positions explained by a table entry within 1e-5 (relative) of a
    threshold or mean (the device keeps fp32 entries and running fp64 moments, the oracle recomputes in fp64);
  * updated tables: an entry gamma*old + (w - 1/(2k)) may differ by 1e-5 * |oracle| + 2.4e-7 * (|gamma*old| + |w - 1/(2k)| + 1/(2k))
    (the roundings of its fp32 operands; the sum may cancel), see assert_tables_close;
  * Top-k and attention outputs: the rules of the memoryless path (tests/harness.py).
"""
import numpy as np
import pytest
import torch

import gen
from oracle import lfps_oracle as orc
from oracle import lfps_tables_oracle as tor
from tests.harness import DEV, DeviceCase, assert_out_close, assert_topk_equal_mod_ties, dev, valid_row

pytestmark = pytest.mark.gpu

TAB_RTOL, TAB_ATOL, BAND = 1e-5, 1e-9, 1e-5


def assert_tables_close(got, want, decayed_old, half, what=""):
    """Updated table entries gamma*old + (w - half).  The device stores fp32 entries and evaluates the
    softmax weight w with an fp32 exponential, so a sum that nearly cancels carries the rounding of its
    operands (2^-24 each, a few roundings), not of its result:
    |gpu - oracle| <= 1e-5 |oracle| + 2.4e-7 (|gamma*old| + |w - half| + half) + 1e-12   on touched entries."""
    got, want, decayed_old = (np.asarray(x, dtype=np.float64) for x in (got, want, decayed_old))
    delta = np.abs(want - decayed_old)
    tol = TAB_RTOL * np.abs(want) + 2.4e-7 * (np.abs(decayed_old) + delta + np.where(delta > 0, half, 0.0)) + 1e-12
    bad = np.abs(got - want) > tol
    assert not bad.any(), f"{what}: {bad.sum()} table entries off, worst {np.abs(got - want)[bad].max():.3e}"


def _make_tables(rng, B, Hq, Lcap, n, n_sink, peaky=True):
    """fp32 tables [B, Hq, Lcap]: sparse spikes over a small positive floor, zeros outside [n_sink, n_b)."""
    ver = np.zeros((B, Hq, Lcap), dtype=np.float32)
    sla = np.zeros((B, Hq, Lcap), dtype=np.float32)
    for b in range(B):
        nb = int(n[b])
        for h in range(Hq):
            for T in (ver, sla):
                x = rng.gamma(0.05 if peaky else 1.0, size=nb).astype(np.float32) * np.float32(0.01)
                spikes = rng.choice(nb, size=max(1, nb // 60), replace=False)
                x[spikes] += rng.gamma(2.0, size=len(spikes)).astype(np.float32)
                x[:n_sink] = 0
                T[b, h, :nb] = x
    return ver, sla


def _explained_by_band(j, tables64, n, a, r, n_sink):
    """True if position j's membership can flip for some head under a 1e-5 relative change of a threshold/mean."""
    for ver, sla in tables64:
        xv, xs = ver[n_sink:n], sla[n_sink:n]
        tv, ts, mv, ms = tor.tau(xv, a), tor.tau(xs, a), xv.mean(), xs.mean()
        near = lambda x, t: np.isfinite(t) and abs(x - t) <= BAND * max(abs(t), 1e-30)
        if near(ver[j], mv) or near(sla[j], ms):
            return True
        for d in range(-r, r + 2):
            i = j - d
            if n_sink <= i < n and (near(ver[i], tv) or near(sla[i], ts)):
                return True
    return False


def _assert_candidates(got, want, tables64, n, a, r, n_sink, what):
    diff = np.setxor1d(got, want)
    for j in diff.tolist():
        assert _explained_by_band(int(j), tables64, n, a, r, n_sink), f"{what}: position {j} differs ({len(diff)} in all)"
    return len(diff)


def oracle_on_candidates(q_group, K, cand, tables64, n, k, gamma, n_sink):
    """Alg. 1 lines 8-9 of the oracle on a GIVEN candidate set: used when the device's set differs from the
    oracle's own by band-explained positions (a legal difference), so that the device's Top-k, output and
    Eq. 10 update of that step are still checked, against the oracle's arithmetic on the set the device used."""
    cand = np.asarray(cand, dtype=np.int64)
    idx, sc, tabs = [], [], []
    for h in range(len(q_group)):
        I_h, s_h = orc.score_topk(q_group[h], K, cand, k)
        idx.append(I_h)
        sc.append(s_h)
        tabs.append(tor.update_tables(tables64[h][0], tables64[h][1], n, I_h, s_h, gamma, n_sink))
    return dict(cand=cand, topk_idx=idx, topk_score=sc, tables=tabs)


@pytest.mark.parametrize("r,n_recent,n_sink,a", [(1, 0, 0, 0.2), (2, 1, 4, 0.3), (4, 2, 2, 0.1), (0, 0, 0, 0.2), (30, 1, 4, 0.2)])
def test_table_candidates_from_imported_tables(r, n_recent, n_sink, a):
    from paper_2506_15704_amd.binding import Lfps
    rng = np.random.default_rng(7 + r)
    B, Hq, Hkv, kmax, Lcap = 3, 32, 8, 32, 2600
    n = np.array([2600, 70, 1031], dtype=np.int32)
    ctx = Lfps(batch=B, max_seq_len=Lcap, max_k=kmax, radius=r, n_recent=n_recent, n_sink=n_sink,
               table_mode=True, table_decay=0.95, table_a=a, cand_cap=Lcap)
    ver, sla = _make_tables(rng, B, Hq, Lcap, n, n_sink)
    ver[1, 5] = 0                                       # a head with empty tables: no pattern, no candidates
    sla[1, 5] = 0
    ver[2, 7, n_sink:n[2]] = 0.25                       # flat vertical table: kappa undefined
    ctx.lfps_tables_import(dev(ver), dev(sla), dev(n))
    cand = torch.full((B, Hkv, ctx.cand_cap), -7, dtype=torch.int32, device=DEV)
    cnt = torch.zeros((B, Hkv), dtype=torch.int32, device=DEV)
    ctx.lfps_table_candidates(dev(n), cand, cnt)
    torch.cuda.synchronize()
    cand, cnt = cand.cpu().numpy(), cnt.cpu().numpy()
    total_diff = 0
    for b in range(B):
        for g in range(Hkv):
            t64 = [(ver[b, 4 * g + h].astype(np.float64), sla[b, 4 * g + h].astype(np.float64)) for h in range(4)]
            want = tor.group_candidates(t64, int(n[b]), a, r, n_recent, n_sink)
            got = cand[b, g, : cnt[b, g]]
            assert list(got) == sorted(set(got.tolist())), "ascending, no duplicates"
            total_diff += _assert_candidates(got, want, t64, int(n[b]), a, r, n_sink, f"b={b} g={g}")
    assert total_diff <= 2
    assert ctx.lfps_poll_status() == 0
    # exported tables are the imported ones
    ev = torch.zeros((B, Hq, Lcap), dtype=torch.float64, device=DEV)
    es = torch.zeros_like(ev)
    ctx.lfps_tables_export(ev, es, dev(n))
    np.testing.assert_array_equal(ev.cpu().numpy(), ver.astype(np.float64))
    np.testing.assert_array_equal(es.cpu().numpy(), sla.astype(np.float64))
    ctx.close()


def _oracle_update_all(ver, sla, n, idx, sc, k, gamma, n_sink):
    B, Hq, Lcap = ver.shape
    nv, ns = np.zeros((B, Hq, Lcap)), np.zeros((B, Hq, Lcap))
    for b in range(B):
        for h in range(Hq):
            a_, b_ = tor.update_tables(ver[b, h].astype(np.float64), sla[b, h].astype(np.float64), int(n[b]),
                                       idx[b, h, : k[b]], sc[b, h, : k[b]].astype(np.float64), gamma, n_sink)
            nv[b, h, : n[b] + 1], ns[b, h, : n[b] + 1] = a_, b_
    return nv, ns


@pytest.mark.parametrize("gamma,n_sink", [(0.95, 0), (0.6, 3)])
def test_table_update_and_following_candidates(gamma, n_sink):
    from paper_2506_15704_amd.binding import Lfps
    rng = np.random.default_rng(21)
    B, Hq, Hkv, kmax, Lcap, r, a = 2, 32, 8, 40, 900, 1, 0.2
    n = np.array([800, 333], dtype=np.int32)
    k = np.array([40, 17], dtype=np.int32)
    ctx = Lfps(batch=B, max_seq_len=Lcap, max_k=kmax, radius=r, n_recent=1, n_sink=n_sink,
               table_mode=True, table_decay=gamma, table_a=a, cand_cap=Lcap)
    ver, sla = _make_tables(rng, B, Hq, Lcap, n, n_sink)
    idx = np.full((B, Hq, kmax), -1, dtype=np.int32)
    sc = np.zeros((B, Hq, kmax), dtype=np.float32)
    for b in range(B):
        for h in range(Hq):
            kk = int(k[b]) - (h % 3)                    # some padding inside the first k_b entries
            idx[b, h, :kk] = rng.choice(int(n[b]), size=kk, replace=False)
            idx[b, h, 0] = 0                            # a sink row (ignored by the tables when n_sink > 0)
            sc[b, h, :kk] = rng.standard_normal(kk).astype(np.float32) * 2
    steps = 3
    for step in range(steps):
        if step == 0:
            ctx.lfps_tables_import(dev(ver), dev(sla), dev(n))
        ctx.lfps_table_update(dev(idx), dev(sc), dev(k), dev(n))
        nv, ns = _oracle_update_all(ver, sla, n, idx, sc, k, gamma, n_sink)
        n = n + 1
        ev = torch.zeros((B, Hq, Lcap), dtype=torch.float64, device=DEV)
        es = torch.zeros_like(ev)
        ctx.lfps_tables_export(ev, es, dev(n))
        ev, es = ev.cpu().numpy(), es.cpu().numpy()
        old_v = gamma * np.asarray(ver, dtype=np.float64)
        old_s = np.zeros_like(old_v)
        old_s[:, :, 1:] = gamma * np.asarray(sla, dtype=np.float64)[:, :, :-1]       # slash history arrives from i-1
        assert_tables_close(ev, nv, old_v, 0.5 / (int(k.min()) - 3), f"vertical, step {step}")
        assert_tables_close(es, ns, old_s, 0.5 / (int(k.min()) - 3), f"slash, step {step}")
        # Eq. 12 on the device: S' = gamma S + 1/2 per head (valid selections are never empty here)
        s_prev = ver.astype(np.float64).sum(axis=2)
        np.testing.assert_allclose(ev.sum(axis=2), gamma * s_prev + 0.5, rtol=1e-5)
        # candidates of the next step from the device's own tables and running statistics
        cand = torch.zeros((B, Hkv, ctx.cand_cap), dtype=torch.int32, device=DEV)
        cnt = torch.zeros((B, Hkv), dtype=torch.int32, device=DEV)
        ctx.lfps_table_candidates(dev(n), cand, cnt)
        cand, cnt = cand.cpu().numpy(), cnt.cpu().numpy()
        nd = 0
        for b in range(B):
            for g in range(Hkv):
                t64 = [(ev[b, 4 * g + h], es[b, 4 * g + h]) for h in range(4)]
                want = tor.group_candidates(t64, int(n[b]), a, r, 1, n_sink)
                nd += _assert_candidates(cand[b, g, : cnt[b, g]], want, t64, int(n[b]), a, r, n_sink, f"step {step} b={b} g={g}")
        assert nd <= 2
        # The device keeps its own state (scaled representation, running moments); the oracle continues
        # from the exported values, which are that state exactly (fp64 products g * A).
        ver, sla = ev, es
        idx = np.roll(idx, 5, axis=2)
        sc = np.roll(sc, 5, axis=2)
    ctx.close()


def test_many_updates_cross_the_renormalisation():
    from paper_2506_15704_amd.binding import Lfps
    rng = np.random.default_rng(33)
    B, Hq, Hkv, kmax, r, a, gamma = 1, 8, 2, 12, 1, 0.2, 0.5
    n0, steps = 150, 90                                 # 0.5^67 < 1e-20: the scale is folded back on the way
    Lcap = n0 + steps + 2
    ctx = Lfps(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, max_seq_len=Lcap, max_k=kmax, radius=r, n_recent=0, n_sink=0,
               table_mode=True, table_decay=gamma, table_a=a, cand_cap=Lcap)
    n = np.array([n0], dtype=np.int32)
    k = np.array([kmax], dtype=np.int32)
    ver, sla = _make_tables(rng, B, Hq, Lcap, n, 0)
    ctx.lfps_tables_import(dev(ver), dev(sla), dev(n))
    v64, s64 = ver.astype(np.float64), sla.astype(np.float64)
    cand = torch.zeros((B, Hkv, ctx.cand_cap), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((B, Hkv), dtype=torch.int32, device=DEV)
    for step in range(steps):
        idx = np.stack([[rng.choice(int(n[0]), size=kmax, replace=False) for _ in range(Hq)]]).astype(np.int32)
        sc = rng.standard_normal((B, Hq, kmax)).astype(np.float32)
        ctx.lfps_table_candidates(dev(n), cand, cnt)
        ctx.lfps_table_update(dev(idx), dev(sc), dev(k), dev(n))     # folds the scale at the end of update 67
        v64, s64 = _oracle_update_all(v64, s64, n, idx, sc, k, gamma, 0)
        n = n + 1
    ev = torch.zeros((B, Hq, Lcap), dtype=torch.float64, device=DEV)
    es = torch.zeros_like(ev)
    ctx.lfps_tables_export(ev, es, dev(n))
    np.testing.assert_allclose(ev.cpu().numpy(), v64, rtol=1e-4, atol=1e-9)
    np.testing.assert_allclose(es.cpu().numpy(), s64, rtol=1e-4, atol=1e-9)
    ctx.close()


@pytest.fixture(scope="module", params=["bf16", "fp8", "fp8kv", "f16"])
def table_case(request):
    """bf16 cache, the same workload with FP8 (E4M3) keys beside bf16 values, with FP8 keys and values, and
    with an fp16 cache."""
    return DeviceCase(gen.tiny_spec("tables_" + request.param, B=2, L=1800, k=64, r=1, T=6,
                                    kv_dtype="f16" if request.param == "f16" else "bf16",
                                    k_dtype="fp8" if request.param in ("fp8", "fp8kv") else "",
                                    v_dtype="fp8" if request.param == "fp8kv" else ""))


def _softmax64(s):
    e = np.exp(s - s.max())
    return e / e.sum()


def test_tables_init_is_eq4_with_one_query(table_case):
    dc = table_case
    s, case = dc.spec, dc.case
    gamma, n_sink = 0.95, 4
    ctx = dc.make_ctx(table_mode=True, table_decay=gamma, table_a=0.2, n_sink=n_sink, n_recent=0)
    ctx.lfps_tables_init(dc.q(0), ctx.kv_view(dc.K, dc.V, dc.seq_lens(0)))
    ev = torch.zeros((s.B, s.Hq, case.Lcap), dtype=torch.float64, device=DEV)
    es = torch.zeros_like(ev)
    ctx.lfps_tables_export(ev, es, dc.seq_lens(0))
    ev, es = ev.cpu().numpy(), es.cpu().numpy()
    for (b, g) in ((0, 0), (1, 5)):
        K, _ = dc.group(b, g)
        n = int(case.seq_lens0[b])
        for h in range(s.G):
            sc = orc.scores(case.q[0, b, s.G * g + h], K[:n])
            w = np.zeros(n)
            w[n_sink:] = _softmax64(sc[n_sink:])
            ver, sla = tor.init_tables(w[None, :], gamma, n_sink)
            np.testing.assert_allclose(ev[b, s.G * g + h, :n], ver, rtol=2e-5, atol=1e-12)
            np.testing.assert_allclose(es[b, s.G * g + h, :n], sla, rtol=2e-5, atol=1e-12)
            assert ev[b, s.G * g + h, :n].sum() == pytest.approx(1 / (2 * (1 - gamma)), rel=1e-5)   # Eq. 12
    ctx.close()


def _teacher_forced_table_steps(dc, view, gamma, a, n_sink, n_recent, groups, steps, k_host, seed=5, exact_cands=True):
    """Every step both sides start from the same fp32 tables (the oracle's, rounded): candidates, Top-k,
    attention output and the updated tables are compared for the given (request, KV group) pairs."""
    s, case = dc.spec, dc.case
    r = s.r
    ctx = dc.make_ctx(table_mode=True, table_decay=gamma, table_a=a, n_sink=n_sink, n_recent=n_recent)
    rng = np.random.default_rng(seed)
    n0 = case.seq_lens(1)
    ver, sla = _make_tables(rng, s.B, s.Hq, case.Lcap, n0, n_sink)
    k_dev = dev(k_host)
    idx = torch.zeros((s.B, s.Hq, case.kmax), dtype=torch.int32, device=DEV)
    isc = torch.zeros((s.B, s.Hq, case.kmax), dtype=torch.float32, device=DEV)
    out = torch.zeros((s.B, s.Hq, s.D), dtype=torch.float32, device=DEV)
    cand = torch.zeros((s.B, s.Hkv, ctx.cand_cap), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((s.B, s.Hkv), dtype=torch.int32, device=DEV)
    for t in range(1, steps + 1):
        n = case.seq_lens(t)
        ctx.lfps_tables_import(dev(ver), dev(sla), dev(n))
        ctx.lfps_table_candidates(dev(n), cand, cnt)
        ctx.lfps_table_step(dc.q(t), view(ctx, t), k_dev, idx, out, isc)
        ev = torch.zeros((s.B, s.Hq, case.Lcap), dtype=torch.float64, device=DEV)
        es = torch.zeros_like(ev)
        ctx.lfps_tables_export(ev, es, dev(n + 1))
        torch.cuda.synchronize()
        c_, cn_, i_, o_ = cand.cpu().numpy(), cnt.cpu().numpy(), idx.cpu().numpy(), out.cpu().numpy()
        ev, es = ev.cpu().numpy(), es.cpu().numpy()
        new_ver, new_sla = ev.copy(), es.copy()         # heads that are not sampled continue from the device's values
        for (b, g) in groups:
            K, V = dc.group(b, g)
            nb, kb = int(n[b]), int(k_host[b])
            t64 = [(ver[b, s.G * g + h].astype(np.float64), sla[b, s.G * g + h].astype(np.float64)) for h in range(s.G)]
            res = tor.table_step(case.q[t, b, s.G * g: s.G * (g + 1)], K, V, t64, nb, kb, r, a, gamma, n_recent, n_sink)
            nd = _assert_candidates(c_[b, g, : cn_[b, g]], res["cand"], t64, nb, a, r, n_sink, f"t={t} b={b} g={g}")
            if exact_cands:
                assert nd == 0, "sampled groups are expected to match exactly"
            mm = min(nb + 1, case.Lcap)
            for h in range(s.G):                         # teacher forcing: the next step starts from the oracle's tables
                new_ver[b, s.G * g + h, :mm] = res["tables"][h][0][:mm]
                new_sla[b, s.G * g + h, :mm] = res["tables"][h][1][:mm]
            if nd:                                       # a different (band-explained) candidate set: the rest of the step
                got_c = c_[b, g, : cn_[b, g]]            # is checked against the oracle's arithmetic on the device's set
                res = oracle_on_candidates(case.q[t, b, s.G * g: s.G * (g + 1)], K, got_c, t64, nb, kb, gamma, n_sink)
            for h in range(s.G):
                bh = s.G * g + h
                got = valid_row(i_[b, bh, :kb])
                ksel = min(kb, len(res["cand"]))
                assert_topk_equal_mod_ties(got, res["topk_idx"][h], lambda p: orc.scores(case.q[t, b, bh], K, p), ksel,
                                           f"t={t} b={b} h={bh}")
                assert (i_[b, bh, ksel:] == -1).all()
                ref = orc.sparse_attn(case.q[t, b, bh], K, V, got)
                assert_out_close(o_[b, bh], ref, f"t={t} b={b} h={bh}")
                if set(got.tolist()) == set(res["topk_idx"][h].tolist()):
                    wv, ws = res["tables"][h]
                    old_v = np.r_[gamma * t64[h][0][:nb], 0.0]
                    old_s = np.r_[0.0, gamma * t64[h][1][:nb]]
                    # (the selected scores differ by fp32 rounding between the two sides: w to ~1e-6 relative)
                    m = min(nb + 1, case.Lcap)           # after the last step the new position lies beyond the capacity
                    assert_tables_close(ev[b, bh, :m], wv[:m], old_v[:m], 10 * 0.5 / max(ksel, 1), f"vertical t={t} h={bh}")
                    assert_tables_close(es[b, bh, :m], ws[:m], old_s[:m], 10 * 0.5 / max(ksel, 1), f"slash t={t} h={bh}")
        ver, sla = new_ver.astype(np.float32), new_sla.astype(np.float32)
    assert ctx.lfps_poll_status() == 0
    ctx.close()


@pytest.mark.parametrize("n_sink,n_recent", [(4, 1), (0, 0)])
def test_table_step_teacher_forced_multi_step(table_case, n_sink, n_recent):
    dc = table_case
    _teacher_forced_table_steps(dc, lambda ctx, t: ctx.kv_view(dc.K, dc.V, dc.seq_lens(t)), 0.9, 0.2, n_sink, n_recent,
                                [(0, 0), (1, 3), (1, 7)], dc.spec.T, dc.case.k)


def _draw_table_config(i):
    rng = np.random.default_rng(9100 + i)
    Hq, Hkv = [(32, 8), (16, 8), (8, 8), (4, 1), (8, 2), (2, 1)][int(rng.integers(0, 6))]
    lo = int(rng.integers(200, 2500))
    kind = "f16" if i >= 12 else ("bf16", "f32", "fp8", "fp8kv")[i % 4]
    return dict(Hq=Hq, Hkv=Hkv, B=int(rng.integers(1, 4)), L_range=(lo, lo + int(rng.integers(0, 1500))),
                kmax=int(rng.integers(8, 97)), r=int(rng.choice([0, 1, 2, 4])), n_recent=int(rng.integers(0, 3)),
                n_sink=int(rng.integers(0, 5)), a=float(rng.choice([0.1, 0.2, 0.3])), gamma=float(rng.choice([0.6, 0.9, 0.95])),
                kv_dtype=kind if kind in ("f32", "f16") else "bf16", k_dtype="fp8" if kind in ("fp8", "fp8kv") else "",
                v_dtype="fp8" if kind == "fp8kv" else "",
                paged=[None, (16, "block_row_head"), (64, "block_head_row")][int(rng.integers(0, 3))])


@pytest.mark.parametrize("i", range(15))
def test_table_step_random_configurations(i):
    """Seeded random configurations of the score-table step (head grouping, ragged lengths, per-request budgets,
    radius, a, decay, sink / recent rows, cache dtype and layout): two teacher-forced steps against the oracle on
    every KV group of the first and the last request."""
    from gen import device as gen_device
    c = _draw_table_config(i)
    spec = gen.tiny_spec(f"tabrnd{i}", B=c["B"], L=None, L_range=c["L_range"], k=c["kmax"], r=c["r"], T=2, Hq=c["Hq"],
                         Hkv=c["Hkv"], kv_dtype=c["kv_dtype"], k_dtype=c["k_dtype"], v_dtype=c["v_dtype"], seed=52000 + i,
                         recency=16)
    dc = DeviceCase(spec)
    rng = np.random.default_rng(i)
    k_host = rng.integers(max(1, c["kmax"] // 2), c["kmax"] + 1, size=c["B"]).astype(np.int32)
    k_host[0] = c["kmax"]
    if c["paged"]:
        Kp, Vp, table = gen_device.paginate(dc.K, dc.V, c["paged"][0], seed=i, layout=c["paged"][1])
        view = lambda ctx, t: ctx.paged_kv_view(Kp, Vp, table, dc.seq_lens(t))
    else:
        view = lambda ctx, t: ctx.kv_view(dc.K, dc.V, dc.seq_lens(t))
    groups = sorted({(b, g) for b in (0, c["B"] - 1) for g in range(c["Hkv"])})
    _teacher_forced_table_steps(dc, view, c["gamma"], c["a"], c["n_sink"], c["n_recent"], groups, 2, k_host, seed=100 + i,
                                exact_cands=False)


def test_table_step_free_running_from_init(table_case):
    """Eq. 4 start, then the device runs alone: the oracle runs alongside from the same start on sampled groups.
    Both chains may drift apart by legal tie choices, so the comparison is statistical; the table sums must
    follow Eq. 12 exactly."""
    dc = table_case
    s, case = dc.spec, dc.case
    gamma, a, n_sink, n_recent = 0.95, 0.2, 4, 1
    ctx = dc.make_ctx(table_mode=True, table_decay=gamma, table_a=a, n_sink=n_sink, n_recent=n_recent)
    ctx.lfps_tables_init(dc.q(0), ctx.kv_view(dc.K, dc.V, dc.seq_lens(0)))
    ev = torch.zeros((s.B, s.Hq, case.Lcap), dtype=torch.float64, device=DEV)
    es = torch.zeros_like(ev)
    b, g = 1, 2
    K, V = dc.group(b, g)
    n0 = int(case.seq_lens0[b])
    t64 = []                                 # the oracle's own Eq. 4 start for the sampled group
    for h in range(s.G):
        sc0 = orc.scores(case.q[0, b, s.G * g + h], K[:n0])
        w = np.zeros(n0)
        w[n_sink:] = _softmax64(sc0[n_sink:])
        ver0, sla0 = tor.init_tables(w[None, :], gamma, n_sink)
        t64.append((np.r_[ver0, np.zeros(case.Lcap - n0)], np.r_[sla0, np.zeros(case.Lcap - n0)]))
    idx = torch.zeros((s.B, s.Hq, case.kmax), dtype=torch.int32, device=DEV)
    out = torch.zeros((s.B, s.Hq, s.D), dtype=torch.float32, device=DEV)
    cand = torch.zeros((s.B, s.Hkv, ctx.cand_cap), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((s.B, s.Hkv), dtype=torch.int32, device=DEV)
    S = 1 / (2 * (1 - gamma))
    jac = []
    for t in range(1, s.T + 1):
        n = case.seq_lens(t)
        ctx.lfps_table_candidates(dev(n), cand, cnt)
        ctx.lfps_table_step(dc.q(t), ctx.kv_view(dc.K, dc.V, dc.seq_lens(t)), dc.k, idx, out)
        res = tor.table_step(case.q[t, b, s.G * g: s.G * (g + 1)], K, V, t64, int(n[b]), int(case.k[b]), s.r, a, gamma,
                             n_recent, n_sink)
        t64 = res["tables"]
        got = set(cand[b, g, : int(cnt[b, g])].cpu().numpy().tolist())
        want = set(res["cand"].tolist())
        jac.append(len(got & want) / max(1, len(got | want)))
        ctx.lfps_tables_export(ev, es, dev(n + 1))
        S = gamma * S + 0.5
        sums = ev.sum(dim=2).cpu().numpy()
        np.testing.assert_allclose(sums, S, rtol=2e-5)
        np.testing.assert_allclose(es.sum(dim=2).cpu().numpy(), S, rtol=2e-5)
        ref = orc.sparse_attn(case.q[t, b, s.G * g], K, V, valid_row(idx[b, s.G * g].cpu().numpy()))
        assert_out_close(out[b, s.G * g].cpu().numpy(), ref, f"t={t}")
    assert min(jac) > 0.9, jac
    ctx.close()


def test_table_entry_points_need_table_mode_and_contents(table_case):
    from paper_2506_15704_amd.binding import LFPS_EINVAL, LfpsError
    dc = table_case
    s, case = dc.spec, dc.case
    cand = torch.zeros((s.B, s.Hkv, 1), dtype=torch.int32, device=DEV)
    plain = dc.make_ctx()
    cand = torch.zeros((s.B, s.Hkv, plain.cand_cap), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((s.B, s.Hkv), dtype=torch.int32, device=DEV)
    with pytest.raises(LfpsError) as ei:
        plain.lfps_table_candidates(dc.seq_lens(1), cand, cnt)
    assert ei.value.code == LFPS_EINVAL
    plain.close()
    tab = dc.make_ctx(table_mode=True)
    cand = torch.zeros((s.B, s.Hkv, tab.cand_cap), dtype=torch.int32, device=DEV)
    with pytest.raises(LfpsError) as ei:
        tab.lfps_table_candidates(dc.seq_lens(1), cand, cnt)       # nothing imported yet
    assert ei.value.code == LFPS_EINVAL
    tab.close()


# ----------------------------------------------------------------------------- head sparsity bypass (Eq. 5-6)
def _sparse_queries(case, t, heads, factor=3.0):
    """The step-t queries with the given (b, h) scaled up: larger logits, so the sink rows take the softmax."""
    q = case.q[t].copy()
    for (b, h) in heads:
        q[b, h] *= np.float32(factor)
    return q


def test_priors_match_oracle(table_case):
    dc = table_case
    s, case = dc.spec, dc.case
    n_sink = 4
    ctx = dc.make_ctx(table_mode=True, n_sink=n_sink)
    kbar = torch.zeros((s.B, s.Hkv, s.D), dtype=torch.float32, device=DEV)
    vbar = torch.zeros_like(kbar)
    s2 = torch.zeros((s.B, s.Hq), dtype=torch.float32, device=DEV)
    ctx.lfps_priors(dc.q(0), ctx.kv_view(dc.K, dc.V, dc.seq_lens(0)), kbar, vbar, s2)
    kb_, vb_, s2_ = kbar.cpu().numpy(), vbar.cpu().numpy(), s2.cpu().numpy()
    for (b, g) in ((0, 1), (1, 6)):
        K, V = dc.group(b, g)
        n = int(case.seq_lens0[b])
        for h in range(s.G):
            ok, ov, os2 = tor.priors(case.q[0, b, s.G * g + h], K, V, n, n_sink)
            np.testing.assert_allclose(kb_[b, g], ok, rtol=0, atol=2e-6)
            np.testing.assert_allclose(vb_[b, g], ov, rtol=0, atol=2e-6)
            assert s2_[b, s.G * g + h] == pytest.approx(os2, rel=2e-5)
    ctx.close()


def test_head_sparsity_ratio_matches_oracle(table_case):
    dc = table_case
    s, case = dc.spec, dc.case
    n_sink, t, eps = 4, 2, 0.85
    ctx = dc.make_ctx(table_mode=True, n_sink=n_sink)
    rng = np.random.default_rng(3)
    kbar = (rng.standard_normal((s.B, s.Hkv, s.D)) * 0.05).astype(np.float32)
    s2 = rng.uniform(0.0, 0.012, size=(s.B, s.Hq)).astype(np.float32)
    sparse = [(0, 1), (0, 2), (1, 13), (1, 31)]
    q = _sparse_queries(case, t, sparse)
    rho = torch.zeros((s.B, s.Hq), dtype=torch.float32, device=DEV)
    gate = torch.zeros((s.B, s.Hq), dtype=torch.int32, device=DEV)
    for n_local in (6, 0):
        ctx.lfps_head_sparsity(dev(q), ctx.kv_view(dc.K, dc.V, dc.seq_lens(t)), dev(kbar), dev(s2), n_local, eps, rho, gate)
        rho_h, gate_h = rho.cpu().numpy(), gate.cpu().numpy()
        for (b, g) in ((0, 0), (1, 3), (1, 7)):
            K, _ = dc.group(b, g)
            n = int(case.seq_lens(t)[b])
            for hh in range(s.G):
                h = s.G * g + hh
                want = tor.sparsity_ratio(q[b, h], K, n, kbar[b, g], float(s2[b, h]), n_sink, n_local)
                assert rho_h[b, h] == pytest.approx(want, rel=2e-4, abs=1e-7), (b, h, n_local)
                if abs(want - eps) > 1e-3:
                    assert bool(gate_h[b, h]) == (want > eps)
        assert gate_h[0, 1] == 1 and gate_h[1, 31] == 1 and gate_h[0, 0] == 0      # the scaled heads are bypassed
    ctx.close()


def test_gated_table_step_matches_oracle(table_case):
    dc = table_case
    s, case = dc.spec, dc.case
    gamma, a, n_sink, n_recent, eps, n_local, t = 0.9, 0.2, 4, 1, 0.97, 6, 3   # eps between the two kinds of head here
    ctx = dc.make_ctx(table_mode=True, table_decay=gamma, table_a=a, n_sink=n_sink, n_recent=n_recent)
    rng = np.random.default_rng(9)
    n = case.seq_lens(t)
    ver, sla = _make_tables(rng, s.B, s.Hq, case.Lcap, n, n_sink)
    kbar = (rng.standard_normal((s.B, s.Hkv, s.D)) * 0.05).astype(np.float32)
    vbar = rng.standard_normal((s.B, s.Hkv, s.D)).astype(np.float32)
    s2 = rng.uniform(0.0, 0.012, size=(s.B, s.Hq)).astype(np.float32)
    sparse = [(0, 1), (0, 2), (1, 12), (1, 13), (1, 14), (1, 15), (1, 31)]      # group (1, 3) is bypassed entirely
    q = _sparse_queries(case, t, sparse)
    idx = torch.full((s.B, s.Hq, case.kmax), 77, dtype=torch.int32, device=DEV)
    isc = torch.zeros((s.B, s.Hq, case.kmax), dtype=torch.float32, device=DEV)
    out = torch.zeros((s.B, s.Hq, s.D), dtype=torch.float32, device=DEV)
    gate = torch.zeros((s.B, s.Hq), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((s.B, s.Hkv), dtype=torch.int32, device=DEV)
    ctx.lfps_tables_import(dev(ver), dev(sla), dev(n))
    ctx.lfps_table_step_gated(dev(q), ctx.kv_view(dc.K, dc.V, dc.seq_lens(t)), dc.k, dev(kbar), dev(vbar), dev(s2),
                              n_local, eps, idx, out, isc, gate)
    ctx.lfps_copy_cand_count(cnt)
    ev = torch.zeros((s.B, s.Hq, case.Lcap), dtype=torch.float64, device=DEV)
    es = torch.zeros_like(ev)
    ctx.lfps_tables_export(ev, es, dev(n + 1))
    torch.cuda.synchronize()
    i_, o_, g_, c_ = idx.cpu().numpy(), out.cpu().numpy(), gate.cpu().numpy(), cnt.cpu().numpy()
    ev, es = ev.cpu().numpy(), es.cpu().numpy()
    assert sorted(zip(*np.nonzero(g_))) == sorted(sparse)
    for (b, g) in ((0, 0), (1, 3), (1, 7)):
        K, V = dc.group(b, g)
        nb, kb = int(n[b]), int(case.k[b])
        t64 = [(ver[b, s.G * g + h].astype(np.float64), sla[b, s.G * g + h].astype(np.float64)) for h in range(s.G)]
        res = tor.gated_table_step(q[b, s.G * g: s.G * (g + 1)], K, V, t64, nb, kb, s.r, a, gamma, kbar[b, g], vbar[b, g],
                                   [float(x) for x in s2[b, s.G * g: s.G * (g + 1)]], eps, n_recent, n_sink, n_local)
        assert list(res["gate"]) == [bool(x) for x in g_[b, s.G * g: s.G * (g + 1)]]
        assert c_[b, g] == len(res["cand"])
        m = min(nb + 1, case.Lcap)
        for h in range(s.G):
            bh = s.G * g + h
            if res["gate"][h]:
                np.testing.assert_array_equal(o_[b, bh], vbar[b, g])
                assert (i_[b, bh] == -1).all()
                np.testing.assert_array_equal(ev[b, bh, :m], res["tables"][h][0][:m])     # untouched
                np.testing.assert_array_equal(es[b, bh, :m], res["tables"][h][1][:m])
            else:
                ksel = min(kb, len(res["cand"]))
                got = valid_row(i_[b, bh, :kb])
                assert_topk_equal_mod_ties(got, res["topk_idx"][h], lambda p: orc.scores(q[b, bh], K, p), ksel, f"b={b} h={bh}")
                assert_out_close(o_[b, bh], orc.sparse_attn(q[b, bh], K, V, got), f"b={b} h={bh}")
                if set(got.tolist()) == set(res["topk_idx"][h].tolist()):
                    old_v = np.r_[gamma * t64[h][0][:nb], 0.0][:m]
                    old_s = np.r_[0.0, gamma * t64[h][1][:nb]][:m]
                    assert_tables_close(ev[b, bh, :m], res["tables"][h][0][:m], old_v, 10 * 0.5 / max(ksel, 1), f"ver h={bh}")
                    assert_tables_close(es[b, bh, :m], res["tables"][h][1][:m], old_s, 10 * 0.5 / max(ksel, 1), f"sla h={bh}")
    # the fully bypassed group proposes only the always-present rows
    assert c_[1, 3] == n_sink + n_recent
    ctx.close()


def test_tables_init_from_several_queries_is_eq4(table_case):
    """Eq. 4 with s = 4: query j (j-th most recent) sees rows [0, n - j + 1) and its weights land at i in the
    vertical table and at i + j - 1 in the slash table."""
    dc = table_case
    s, case = dc.spec, dc.case
    gamma, n_sink, nq = 0.95, 4, 4
    ctx = dc.make_ctx(table_mode=True, table_decay=gamma, table_a=0.2, n_sink=n_sink, n_recent=0)
    q_hist = np.stack([case.q[j] for j in range(nq)])            # any four query sets serve as the last prefill queries
    ctx.lfps_tables_init(dev(q_hist), ctx.kv_view(dc.K, dc.V, dc.seq_lens(0)))
    ev = torch.zeros((s.B, s.Hq, case.Lcap), dtype=torch.float64, device=DEV)
    es = torch.zeros_like(ev)
    ctx.lfps_tables_export(ev, es, dc.seq_lens(0))
    ev, es = ev.cpu().numpy(), es.cpu().numpy()
    orc_tab = {}
    for (b, g) in ((0, 2), (1, 5)):
        K, _ = dc.group(b, g)
        n = int(case.seq_lens0[b])
        orc_tab[(b, g)] = []
        for h in range(s.G):
            bh = s.G * g + h
            w = np.zeros((nq, n))
            for j in range(1, nq + 1):
                seen = n - j + 1
                sc = orc.scores(q_hist[j - 1, b, bh], K[:seen])
                w[j - 1, n_sink:seen] = _softmax64(sc[n_sink:])
            ver, sla = tor.init_tables(w, gamma, n_sink)
            orc_tab[(b, g)].append((ver, sla))
            np.testing.assert_allclose(ev[b, bh, :n], ver, rtol=3e-5, atol=1e-12)
            np.testing.assert_allclose(es[b, bh, :n], sla, rtol=3e-5, atol=1e-12)
            assert es[b, bh, :n].sum() == pytest.approx(1 / (2 * (1 - gamma)), rel=1e-5)
    # the statistics that go with them: candidates from the device equal the oracle's from its own tables
    cand = torch.zeros((s.B, s.Hkv, ctx.cand_cap), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((s.B, s.Hkv), dtype=torch.int32, device=DEV)
    ctx.lfps_table_candidates(dc.seq_lens(0), cand, cnt)
    for (b, g) in ((0, 2), (1, 5)):
        n = int(case.seq_lens0[b])
        t64 = orc_tab[(b, g)]
        want = tor.group_candidates(t64, n, 0.2, s.r, 0, n_sink)
        _assert_candidates(cand[b, g, : int(cnt[b, g])].cpu().numpy(), want, t64, n, 0.2, s.r, n_sink, f"b={b} g={g}")
    ctx.close()


def test_gated_steps_with_and_without_the_score_filter_agree(table_case):
    """Chained gated steps in which some heads are bypassed from the first step on (they never get a k-th score
    of their own), then stop being bypassed (eps = 2): the context with the score filter returns bit for bit
    what the unfiltered context returns, at every step."""
    dc = table_case
    s, case = dc.spec, dc.case
    sparse = [(0, 1), (0, 2), (1, 12), (1, 13), (1, 14), (1, 15), (1, 31)]
    rng = np.random.default_rng(10)
    kbar = dev((rng.standard_normal((s.B, s.Hkv, s.D)) * 0.05).astype(np.float32))
    vbar = dev(rng.standard_normal((s.B, s.Hkv, s.D)).astype(np.float32))
    s2 = dev(rng.uniform(0.0, 0.012, size=(s.B, s.Hq)).astype(np.float32))
    runs = []
    for filtered in (False, True):
        ctx = dc.make_ctx(table_mode=True, table_decay=0.9, table_a=0.2, n_sink=4, n_recent=1)
        ctx.lfps_set_filter(filtered)
        ctx.lfps_tables_init(dc.q(0), ctx.kv_view(dc.K, dc.V, dc.seq_lens(0)))
        ctx.lfps_timing_enable(True)
        hist = []
        for t, eps in ((1, 0.97), (2, 0.97), (3, 0.97), (4, 2.0), (5, 2.0), (6, 0.97)):
            q = dev(_sparse_queries(case, t, sparse))
            idx = torch.full((s.B, s.Hq, case.kmax), 77, dtype=torch.int32, device=DEV)
            isc = torch.zeros((s.B, s.Hq, case.kmax), dtype=torch.float32, device=DEV)
            out = torch.zeros((s.B, s.Hq, s.D), dtype=torch.float32, device=DEV)
            gate = torch.zeros((s.B, s.Hq), dtype=torch.int32, device=DEV)
            ctx.lfps_table_step_gated(q, ctx.kv_view(dc.K, dc.V, dc.seq_lens(t)), dc.k, kbar, vbar, s2, 6, eps,
                                      idx, out, isc, gate)
            hist.append((idx, isc, out, gate))
        tm = ctx.lfps_timing_read()
        assert (tm["filter_score"][1] > 0) == filtered
        torch.cuda.synchronize()
        runs.append(hist)
        ctx.close()
    for t, (a_, b_) in enumerate(zip(*runs), start=1):
        for what, x, y in zip(("idx", "score", "out", "gate"), a_, b_):
            assert torch.equal(x, y), f"step {t}: {what} differs with the filter on"
    gates = [int(h[3].sum().item()) for h in runs[1]]
    assert gates[0] == len(sparse) and gates[3] == 0          # bypassed at first, not bypassed with eps = 2


def test_memoryless_and_table_steps_can_be_captured(table_case):
    """lfps_step and lfps_table_step are kernel launches only (the tables' scale and update count live in device
    memory): each is captured once into a graph and replayed three times with eager work in between, and every
    replay equals the eager result of a second context given the same inputs."""
    dc = table_case
    s, case = dc.spec, dc.case
    shp = (s.B, s.Hq, case.kmax)
    ref_ctx, ctx = dc.make_ctx(), dc.make_ctx()
    seed = torch.zeros(shp, dtype=torch.int32, device=DEV)
    ref_ctx.lfps_exact_topk(dc.q(0), ref_ctx.kv_view(dc.K, dc.V, dc.seq_lens(0)), dc.k, seed)
    # fixed buffers the graph works on
    q, sl, prev = dc.q(1).clone(), dc.seq_lens(1).clone(), seed.clone()
    idx = torch.zeros(shp, dtype=torch.int32, device=DEV)
    out = torch.zeros((s.B, s.Hq, s.D), dtype=torch.float32, device=DEV)
    kv = ctx.kv_view(dc.K, dc.V, sl)
    ctx.lfps_step(q, kv, prev, dc.k, idx, out)               # warm-up outside the capture (also sets the history)
    ctx.lfps_reset_history()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ctx.lfps_step(q, kv, prev, dc.k, idx, out)
    want_prev = seed.clone()
    for t in (1, 2, 3):
        e_idx = torch.zeros(shp, dtype=torch.int32, device=DEV)
        e_out = torch.zeros_like(out)
        ref_ctx.lfps_step(dc.q(t), ref_ctx.kv_view(dc.K, dc.V, dc.seq_lens(t)), want_prev, dc.k, e_idx, e_out)
        q.copy_(dc.q(t))                                      # eager work between the replays
        sl.copy_(dc.seq_lens(t))
        prev.copy_(want_prev)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(idx, e_idx) and torch.equal(out, e_out), f"replay {t}"
        want_prev = e_idx
    ref_ctx.close()
    ctx.close()

    # the table step: both contexts start from the same Eq. 4 tables; the graph's context never runs a step eagerly
    warm = dc.make_ctx(table_mode=True, n_sink=4)            # loads every kernel of the step before the capture
    warm.lfps_tables_init(dc.q(0), warm.kv_view(dc.K, dc.V, dc.seq_lens(0)))
    warm.lfps_table_step(dc.q(1), warm.kv_view(dc.K, dc.V, dc.seq_lens(1)), dc.k, idx, out)
    torch.cuda.synchronize()
    warm.close()
    ref_tab, tab = dc.make_ctx(table_mode=True, n_sink=4), dc.make_ctx(table_mode=True, n_sink=4)
    for c in (ref_tab, tab):
        c.lfps_tables_init(dc.q(0), c.kv_view(dc.K, dc.V, dc.seq_lens(0)))
    isc = torch.zeros(shp, dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    g2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g2):
        tab.lfps_table_step(q, tab.kv_view(dc.K, dc.V, sl), dc.k, idx, out, isc)
    for t in (1, 2, 3, 4):
        e_idx = torch.zeros(shp, dtype=torch.int32, device=DEV)
        e_out = torch.zeros_like(out)
        e_isc = torch.zeros_like(isc)
        ref_tab.lfps_table_step(dc.q(t), ref_tab.kv_view(dc.K, dc.V, dc.seq_lens(t)), dc.k, e_idx, e_out, e_isc)
        q.copy_(dc.q(t))
        sl.copy_(dc.seq_lens(t))
        g2.replay()
        torch.cuda.synchronize()
        assert torch.equal(idx, e_idx) and torch.equal(isc, e_isc) and torch.equal(out, e_out), f"table replay {t}"
    ev, es = (torch.zeros((s.B, s.Hq, case.Lcap), dtype=torch.float64, device=DEV) for _ in range(2))
    rv, rs = torch.zeros_like(ev), torch.zeros_like(es)
    tab.lfps_tables_export(ev, es, sl)
    ref_tab.lfps_tables_export(rv, rs, sl)
    assert torch.equal(ev, rv) and torch.equal(es, rs)
    assert tab.lfps_poll_status() == 0
    ref_tab.close()
    tab.close()


def test_replayed_updates_stop_at_the_table_capacity():
    """The slash frame holds max_seq_len - 1 moves.  Updates replayed from a graph are not counted by the host:
    the kernel itself leaves the tables alone from then on and raises LFPS_FLAG_TABLE_FULL; an eager call beyond
    the capacity returns the error code."""
    from paper_2506_15704_amd.binding import LFPS_FLAG_TABLE_FULL, Lfps, LfpsError
    rng = np.random.default_rng(71)
    B, Hq, Hkv, kmax, Lcap, n0 = 1, 8, 2, 6, 40, 20
    ctx = Lfps(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, max_seq_len=Lcap, max_k=kmax, radius=1, n_recent=0, n_sink=0,
               table_mode=True, table_decay=0.9, table_a=0.2, cand_cap=Lcap)
    n = np.array([n0], dtype=np.int32)
    ver, sla = _make_tables(rng, B, Hq, Lcap, n, 0)
    ctx.lfps_tables_import(dev(ver), dev(sla), dev(n))
    idx = dev(np.stack([[rng.choice(n0, size=kmax, replace=False) for _ in range(Hq)]]).astype(np.int32))
    sc = dev(rng.standard_normal((B, Hq, kmax)).astype(np.float32))
    k, nd = dev(np.array([kmax], dtype=np.int32)), dev(n)
    warm = Lfps(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, max_seq_len=Lcap, max_k=kmax, radius=1, n_recent=0, n_sink=0,
                table_mode=True, table_decay=0.9, table_a=0.2, cand_cap=Lcap)
    warm.lfps_tables_import(dev(ver), dev(sla), nd)
    warm.lfps_table_update(idx, sc, k, nd)                   # loads the kernel before the capture
    torch.cuda.synchronize()
    warm.close()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        ctx.lfps_table_update(idx, sc, k, nd)

    def export():
        ev, es = (torch.zeros((B, Hq, Lcap), dtype=torch.float64, device=DEV) for _ in range(2))
        ctx.lfps_tables_export(ev, es, nd)
        torch.cuda.synchronize()
        return ev, es

    for _ in range(Lcap - 2):
        g.replay()
    assert ctx.lfps_poll_status() == 0
    before_last = export()
    g.replay()                                               # update number Lcap - 1: the last one that fits
    assert ctx.lfps_poll_status() == 0
    full = export()
    assert not torch.equal(full[0], before_last[0])
    for _ in range(5):
        g.replay()
    assert ctx.lfps_poll_status() == LFPS_FLAG_TABLE_FULL
    after = export()
    assert torch.equal(after[0], full[0]) and torch.equal(after[1], full[1])
    ctx.close()
    # the host's own count: eager calls beyond the capacity are refused with an error code
    ctx = Lfps(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, max_seq_len=Lcap, max_k=kmax, radius=1, n_recent=0, n_sink=0,
               table_mode=True, table_decay=0.9, table_a=0.2, cand_cap=Lcap)
    ctx.lfps_tables_import(dev(ver), dev(sla), nd)
    for _ in range(Lcap - 1):
        ctx.lfps_table_update(idx, sc, k, nd)
    with pytest.raises(LfpsError):
        ctx.lfps_table_update(idx, sc, k, nd)
    assert ctx.lfps_poll_status() == 0
    ctx.close()


def _assert_candidates_band(got, want, tables64, n, a, r, n_sink, band, what):
    """As _assert_candidates with a wider band: for chains in which the device's fp32 tables and the oracle's fp64
    tables have drifted apart by the accumulated rounding of many updates."""
    global BAND
    keep = BAND
    BAND = band
    try:
        return _assert_candidates(got, want, tables64, n, a, r, n_sink, what)
    finally:
        BAND = keep


@pytest.mark.parametrize("gamma", [0.9, 0.6])
def test_scan_after_many_updates_without_import(gamma):
    """The scan reads the tables only where the per-block upper bounds allow an initial candidate; the bounds are
    maintained by the update alone (raised, never lowered) once the tables have been imported.  Forty updates with
    given lists (clustered around a few positions, the context growing by a row per step, positions repeated now
    and then) on the device and in the oracle from the same start: the candidates of every step must be the
    oracle's, modulo entries within rounding of a threshold or mean."""
    from paper_2506_15704_amd.binding import Lfps
    rng = np.random.default_rng(77)
    B, Hq, Hkv, kmax, r, a = 2, 8, 2, 40, 2, 0.2
    n0, steps = np.array([2900, 1500], dtype=np.int32), 40
    Lcap = int(n0.max()) + steps + 2
    n_sink = 2
    ctx = Lfps(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, max_seq_len=Lcap, max_k=kmax, radius=r, n_recent=1, n_sink=n_sink,
               table_mode=True, table_decay=gamma, table_a=a, cand_cap=Lcap)
    n = n0.copy()
    k = np.array([kmax, 24], dtype=np.int32)
    ver, sla = _make_tables(rng, B, Hq, Lcap, n, n_sink)
    ctx.lfps_tables_import(dev(ver), dev(sla), dev(n))
    v64, s64 = ver.astype(np.float64), sla.astype(np.float64)
    cand = torch.zeros((B, Hkv, ctx.cand_cap), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((B, Hkv), dtype=torch.int32, device=DEV)
    pools = [[np.sort(rng.choice(int(n0[b]) - 64, size=6, replace=False)) + 16 for _ in range(Hq)] for b in range(B)]
    G = Hq // Hkv
    total_diff = 0
    for step in range(steps):
        idx = np.full((B, Hq, kmax), -1, dtype=np.int32)
        sc = rng.standard_normal((B, Hq, kmax)).astype(np.float32)
        for b in range(B):
            for h in range(Hq):
                # most picks fall within +-12 rows of the head's six centres, a few anywhere, the newest row now and then
                near = (rng.choice(pools[b][h], size=k[b] - 6) + rng.integers(-12, 13, size=k[b] - 6)) % int(n[b])
                row = np.unique(np.r_[near, rng.choice(int(n[b]), size=5), [int(n[b]) - 1]])[: k[b]]
                idx[b, h, : len(row)] = row
                if step % 7 == 3 and len(row) < k[b]:
                    idx[b, h, len(row)] = row[0]                     # a position given twice
                sc[b, h, : len(row)] += 3.0 * rng.random(len(row))
        ctx.lfps_table_candidates(dev(n), cand, cnt)
        c_, cn_ = cand.cpu().numpy(), cnt.cpu().numpy()
        for b in range(B):
            for g in range(Hkv):
                t64 = [(v64[b, G * g + h], s64[b, G * g + h]) for h in range(G)]
                want = tor.group_candidates(t64, int(n[b]), a, r, 1, n_sink)
                total_diff += _assert_candidates_band(c_[b, g, : cn_[b, g]], want, t64, int(n[b]), a, r, n_sink, 2e-4,
                                                      f"step {step} b{b} g{g}")
        ctx.lfps_table_update(dev(idx), dev(sc), dev(k), dev(n))
        for b in range(B):                                          # the oracle's Eq. 10 on the same lists
            for h in range(Hq):
                nv, ns = tor.update_tables(v64[b, h], s64[b, h], int(n[b]), idx[b, h, : k[b]], sc[b, h, : k[b]].astype(np.float64),
                                           gamma, n_sink)
                v64[b, h, : n[b] + 1], s64[b, h, : n[b] + 1] = nv, ns
        n = n + 1
    assert total_diff <= 6, total_diff
    assert ctx.lfps_poll_status() == 0
    ctx.close()


def test_table_steps_chained_on_the_device_without_import():
    """lfps_table_step keeps its own tables from step to step (no import in between): the oracle follows from the
    same Eq. 4 start, taking at every step the device's index sets once they have been checked to be legal Top-k
    sets of the oracle's candidates, so both chains see the same selections.  The device's candidates (a scan that
    trusts the upper bounds its own updates maintain) must be the oracle's at every step."""
    spec = gen.tiny_spec("tables_chain", B=2, L=2600, k=96, r=2, T=14, n_hot=12, recency=32)
    dc = DeviceCase(spec)
    s, case = dc.spec, dc.case
    gamma, a, n_sink, n_recent = 0.9, 0.2, 4, 1
    ctx = dc.make_ctx(table_mode=True, table_decay=gamma, table_a=a, n_sink=n_sink, n_recent=n_recent)
    ctx.lfps_tables_init(dc.q(0), ctx.kv_view(dc.K, dc.V, dc.seq_lens(0)))
    groups = [(0, 1), (1, 6)]
    t64 = {}
    for (b, g) in groups:                    # the oracle's own Eq. 4 start
        K, _ = dc.group(b, g)
        n0 = int(case.seq_lens0[b])
        t64[(b, g)] = []
        for h in range(s.G):
            sc0 = orc.scores(case.q[0, b, s.G * g + h], K[:n0])
            w = np.zeros(n0)
            w[n_sink:] = _softmax64(sc0[n_sink:])
            ver0, sla0 = tor.init_tables(w[None, :], gamma, n_sink)
            t64[(b, g)].append((np.r_[ver0, np.zeros(case.Lcap - n0)], np.r_[sla0, np.zeros(case.Lcap - n0)]))
    idx = torch.zeros((s.B, s.Hq, case.kmax), dtype=torch.int32, device=DEV)
    isc = torch.zeros((s.B, s.Hq, case.kmax), dtype=torch.float32, device=DEV)
    out = torch.zeros((s.B, s.Hq, s.D), dtype=torch.float32, device=DEV)
    cand = torch.zeros((s.B, s.Hkv, ctx.cand_cap), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((s.B, s.Hkv), dtype=torch.int32, device=DEV)
    total_diff = 0
    for t in range(1, s.T + 1):
        n = case.seq_lens(t)
        ctx.lfps_table_candidates(dev(n), cand, cnt)
        ctx.lfps_table_step(dc.q(t), ctx.kv_view(dc.K, dc.V, dc.seq_lens(t)), dc.k, idx, out, isc)
        c_, cn_, i_ = cand.cpu().numpy(), cnt.cpu().numpy(), idx.cpu().numpy()
        for (b, g) in groups:
            K, V = dc.group(b, g)
            nb, kb = int(n[b]), int(case.k[b])
            tabs = t64[(b, g)]
            want = tor.group_candidates(tabs, nb, a, s.r, n_recent, n_sink)
            got_c = c_[b, g, : cn_[b, g]]
            total_diff += _assert_candidates_band(got_c, want, tabs, nb, a, s.r, n_sink, 1e-4, f"t={t} b={b} g={g}")
            new_tabs = []
            for h in range(s.G):
                bh = s.G * g + h
                ksel = min(kb, len(got_c))
                got = valid_row(i_[b, bh, :kb])
                I_h, _ = orc.score_topk(case.q[t, b, bh], K, got_c, ksel)     # the oracle's select on the set the device used
                assert_topk_equal_mod_ties(got, I_h, lambda p: orc.scores(case.q[t, b, bh], K, p), ksel, f"t={t} b={b} h={bh}")
                # Eq. 10 in the oracle on the (legal) set the device selected, with the oracle's own scores
                new_tabs.append(tor.update_tables(tabs[h][0], tabs[h][1], nb, got, orc.scores(case.q[t, b, bh], K, got),
                                                  gamma, n_sink))
            pad = lambda x: np.r_[x, np.zeros(max(0, case.Lcap - len(x)))][: case.Lcap]   # (the last step's new position lies past the capacity)
            t64[(b, g)] = [(pad(v_), pad(s_)) for (v_, s_) in new_tabs]
    assert total_diff <= 4, total_diff
    assert ctx.lfps_poll_status() == 0
    ctx.close()
