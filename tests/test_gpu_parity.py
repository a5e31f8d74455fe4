"""HIP path vs CPU oracle, stage by stage, through the C ABI (small cases: several tiles and
ragged tails; full-size sampled checks live in test_gpu_workloads.py)."""
import numpy as np
import pytest
import torch

import gen
from oracle import lfps_oracle as orc
from tests.harness import (DEV, DeviceCase, assert_out_close, assert_scores_close, stored_values,
                           assert_topk_equal_mod_ties, dev, valid_row)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def small_bf16():
    return DeviceCase(gen.tiny_spec("small_bf16", B=3, L=2500, k=96, r=2, T=4))


@pytest.fixture(scope="module")
def small_fp8():
    return DeviceCase(gen.tiny_spec("small_fp8", B=2, L=2100, k=80, r=2, T=4, k_dtype="fp8"))


@pytest.fixture(scope="module")
def small_fp8kv():
    return DeviceCase(gen.tiny_spec("small_fp8kv", B=2, L=1900, k=72, r=2, T=4, k_dtype="fp8", v_dtype="fp8"))


@pytest.fixture(scope="module")
def small_f16():
    return DeviceCase(gen.tiny_spec("small_f16", B=2, L=2300, k=88, r=2, T=4, kv_dtype="f16"))


@pytest.fixture(scope="module")
def small_f32():
    return DeviceCase(gen.tiny_spec("small_f32", B=2, L=1111, k=64, r=3, T=3, kv_dtype="f32"))


# ------------------------------------------------------------------------ generator
@pytest.mark.parametrize("fx", ["small_bf16", "small_f32", "small_fp8", "small_fp8kv", "small_f16"])
def test_device_fill_matches_cpu_generator(fx, request):
    dc = request.getfixturevalue(fx)
    rows = np.array([0, 3, 4, 5, 100, dc.case.seq_lens0[1] - 17, dc.case.seq_lens0[1] - 16, dc.case.seq_lens0[1] + 2,
                     dc.case.Lcap - 1] + dc.case.hot_pos[1, 5].tolist())
    for which, T in (("k", dc.K), ("v", dc.V)):
        want, _ = dc.case.kv_rows(which, 1, 5, rows)
        got = stored_values(T[1, 5])[torch.from_numpy(rows).to(DEV)].cpu().numpy()
        np.testing.assert_array_equal(got, want)
    Kfull, Vfull = dc.group(0, 2)
    np.testing.assert_array_equal(stored_values(dc.K[0, 2, : len(Kfull)]).cpu().numpy(), Kfull)
    np.testing.assert_array_equal(stored_values(dc.V[0, 2, : len(Vfull)]).cpu().numpy(), Vfull)


# ------------------------------------------------------------------------ S1 candidates
def _random_prev(rng, B, Hq, kmax, k, n):
    prev = np.full((B, Hq, kmax), -1, dtype=np.int32)
    for b in range(B):
        for h in range(Hq):
            kb = int(k[b])
            row = rng.choice(int(n[b]) + 6, size=kb, replace=False) - 3      # some entries < 0 and >= n
            prev[b, h, :kb] = row
            prev[b, h, kb:] = rng.integers(0, int(n[b]), size=kmax - kb)     # garbage past k_b must be ignored
    return prev


@pytest.mark.parametrize("r,n_recent,n_sink", [(0, 0, 0), (1, 1, 0), (4, 1, 4), (17, 3, 2), (40, 0, 0)])
def test_candidates_bit_exact(r, n_recent, n_sink):
    from paper_2506_15704_amd.binding import Lfps
    rng = np.random.default_rng(100 + r)
    B, Hq, Hkv, kmax, Lcap = 3, 32, 8, 50, 3000
    n = np.array([3000, 37, 1025], dtype=np.int32)
    k = np.array([50, 20, 33], dtype=np.int32)
    ctx = Lfps(batch=B, max_seq_len=Lcap, max_k=kmax, radius=r, n_recent=n_recent, n_sink=n_sink)
    prev = _random_prev(rng, B, Hq, kmax, k, n)
    cand = torch.full((B, Hkv, ctx.cand_cap), -7, dtype=torch.int32, device=DEV)
    cnt = torch.zeros((B, Hkv), dtype=torch.int32, device=DEV)
    ctx.lfps_candidates(dev(prev), dev(k), dev(n), cand, cnt)
    torch.cuda.synchronize()
    first = (cand.cpu().numpy().copy(), cnt.cpu().numpy().copy())
    for b in range(B):
        for g in range(Hkv):
            want = orc.candidates([prev[b, 4 * g + h, : k[b]] for h in range(4)], int(n[b]), r, n_recent, n_sink)
            c = int(first[1][b, g])
            assert c == len(want), (b, g, c, len(want))
            np.testing.assert_array_equal(first[0][b, g, :c], want)
            assert np.all(first[0][b, g, c:] == -7)
    ctx.lfps_candidates(dev(prev), dev(k), dev(n), cand, cnt)       # run-to-run identical
    torch.cuda.synchronize()
    np.testing.assert_array_equal(cand.cpu().numpy(), first[0])
    assert ctx.lfps_poll_status() == 0


def test_candidates_overflow_is_truncated_and_flagged():
    from paper_2506_15704_amd.binding import Lfps, LFPS_FLAG_CAND_OVERFLOW
    B, Hq, Hkv, kmax, Lcap = 1, 32, 8, 16, 500
    ctx = Lfps(batch=B, max_seq_len=Lcap, max_k=kmax, radius=3, n_recent=1, cand_cap=40)
    prev = np.tile(np.arange(16, dtype=np.int32) * 20, (B, Hq, 1))
    cand = torch.zeros((B, Hkv, 40), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((B, Hkv), dtype=torch.int32, device=DEV)
    ctx.lfps_candidates(dev(prev), dev(np.array([16], np.int32)), dev(np.array([500], np.int32)), cand, cnt)
    assert ctx.lfps_poll_status() == LFPS_FLAG_CAND_OVERFLOW
    want = orc.candidates([prev[0, 0]], 500, 3, 1, 0)
    assert cnt.cpu().numpy().tolist() == [[40] * 8]
    np.testing.assert_array_equal(cand[0, 3].cpu().numpy(), want[:40])
    assert ctx.lfps_poll_status() == 0


# ------------------------------------------------------------------------ S2 + S3
def _teacher_inputs(dc, t, rng=None):
    """Previous Top-k of step t-1 from the oracle (exact Top-k at t-1), per (b, h)."""
    case, spec = dc.case, dc.spec
    prev = np.full((spec.B, spec.Hq, case.kmax), -1, dtype=np.int32)
    n_prev = case.seq_lens(t - 1)
    for b in range(spec.B):
        for h in range(spec.Hq):
            K, _ = dc.group(b, h // spec.G)
            I, _ = orc.exact_topk(case.q[t - 1, b, h], K, int(n_prev[b]), int(case.k[b]))
            prev[b, h, : len(I)] = I
    return prev


@pytest.mark.parametrize("fx", ["small_bf16", "small_f32", "small_fp8", "small_fp8kv", "small_f16"])
def test_score_topk_teacher_forced(fx, request):
    dc = request.getfixturevalue(fx)
    case, spec = dc.case, dc.spec
    ctx = dc.make_ctx()
    t = 2
    prev = _teacher_inputs(dc, t)
    n = case.seq_lens(t)
    cand = torch.zeros((spec.B, spec.Hkv, ctx.cand_cap), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((spec.B, spec.Hkv), dtype=torch.int32, device=DEV)
    ctx.lfps_candidates(dev(prev), dc.k, dc.seq_lens(t), cand, cnt)
    kv = ctx.kv_view(dc.K, dc.V, dc.seq_lens(t))
    idx = torch.zeros((spec.B, spec.Hq, case.kmax), dtype=torch.int32, device=DEV)
    sc = torch.zeros((spec.B, spec.Hq, case.kmax), dtype=torch.float32, device=DEV)
    cs = torch.full((spec.B, spec.Hq, ctx.cand_cap), float("nan"), dtype=torch.float32, device=DEV)
    ctx.lfps_score_topk(dc.q(t), kv, cand, cnt, dc.k, idx, sc, cs)
    torch.cuda.synchronize()
    cand_h, cnt_h, idx_h, sc_h, cs_h = (x.cpu().numpy() for x in (cand, cnt, idx, sc, cs))
    # a second run without the score dump must select the same rows
    idx2 = torch.zeros_like(idx)
    ctx.lfps_score_topk(dc.q(t), kv, cand, cnt, dc.k, idx2, None, None)
    np.testing.assert_array_equal(idx2.cpu().numpy(), idx_h)
    for b in range(spec.B):
        for g in range(spec.Hkv):
            K, _ = dc.group(b, g)
            C = orc.candidates([prev[b, 4 * g + h, : case.k[b]] for h in range(4)], int(n[b]), spec.r, 1, 0)
            c = int(cnt_h[b, g])
            np.testing.assert_array_equal(cand_h[b, g, :c], C)
            for hh in range(4):
                h = 4 * g + hh
                ref = orc.scores(case.q[t, b, h], K, C)
                assert_scores_close(cs_h[b, h, :c], ref, f"cand_score b{b} h{h}")
                assert np.all(np.isnan(cs_h[b, h, c:]))
                kb = int(case.k[b])
                I, S = orc.score_topk(case.q[t, b, h], K, C, kb)
                got = idx_h[b, h, :kb]
                assert np.all(np.diff(got) > 0), "selected positions must be ascending"
                assert np.all(idx_h[b, h, kb:] == -1) and np.all(sc_h[b, h, kb:] == 0)
                assert_topk_equal_mod_ties(got, I, lambda p: orc.scores(case.q[t, b, h], K, p), kb, f"topk b{b} h{h}")
                assert_scores_close(sc_h[b, h, :kb], orc.scores(case.q[t, b, h], K, got), f"topk_score b{b} h{h}")


def test_select_ties_take_lowest_positions_and_k_exceeding_candidates():
    """Degenerate scores: all keys equal -> every score ties; and k_b > |C|."""
    from paper_2506_15704_amd.binding import Lfps
    B, Hq, Hkv, D, Lcap, kmax = 1, 32, 8, 128, 600, 40
    ctx = Lfps(batch=B, max_seq_len=Lcap, max_k=kmax, radius=1, n_recent=0, kv_dtype="f32")
    K = torch.ones((B, Hkv, Lcap, D), dtype=torch.float32, device=DEV)
    q = torch.ones((B, Hq, D), dtype=torch.float32, device=DEV)
    n = dev(np.array([600], np.int32))
    kv = ctx.kv_view(K, K, n)
    C = np.arange(5, 5 + 70, dtype=np.int32) * 3
    cand = torch.zeros((B, Hkv, ctx.cand_cap), dtype=torch.int32, device=DEV)
    cand[:, :, :70] = dev(C)
    cnt = torch.full((B, Hkv), 70, dtype=torch.int32, device=DEV)
    cnt[0, 1] = 25                                       # fewer candidates than k
    idx = torch.zeros((B, Hq, kmax), dtype=torch.int32, device=DEV)
    sc = torch.zeros((B, Hq, kmax), dtype=torch.float32, device=DEV)
    ctx.lfps_score_topk(q, kv, cand, cnt, dev(np.array([40], np.int32)), idx, sc, None)
    idx_h, sc_h = idx.cpu().numpy(), sc.cpu().numpy()
    np.testing.assert_array_equal(idx_h[0, 0], C[:40])   # ties -> lowest positions (the oracle's rule)
    I, _ = orc.score_topk(np.ones(D), np.ones((Lcap, D)), C, 40)
    assert sorted(I.tolist()) == C[:40].tolist()
    np.testing.assert_array_equal(idx_h[0, 4, :25], C[:25])
    assert np.all(idx_h[0, 4, 25:] == -1) and np.all(sc_h[0, 4, 25:] == 0)
    np.testing.assert_allclose(sc_h[0, 0], 128 / np.sqrt(128), rtol=1e-6)


# ------------------------------------------------------------------------ S4
@pytest.mark.parametrize("fx", ["small_bf16", "small_f32", "small_fp8", "small_fp8kv", "small_f16"])
@pytest.mark.parametrize("with_scores", [True, False])
def test_sparse_attn_parity(fx, with_scores, request):
    dc = request.getfixturevalue(fx)
    case, spec = dc.case, dc.spec
    ctx = dc.make_ctx()
    rng = np.random.default_rng(7)
    t = 1
    n = case.seq_lens(t)
    idx = np.full((spec.B, spec.Hq, case.kmax), -1, dtype=np.int32)
    scs = np.zeros((spec.B, spec.Hq, case.kmax), dtype=np.float32)
    for b in range(spec.B):
        for h in range(spec.Hq):
            kb = int(case.k[b])
            I = rng.choice(int(n[b]), size=kb, replace=False)
            I[:3] = [0, 1, int(n[b]) - 1]                 # sinks and the newest row
            if h % 5 == 0:
                I[5] = -1                                 # padding inside the list
            idx[b, h, :kb] = I
            K, _ = dc.group(b, h // 4)
            v = I >= 0
            scs[b, h, :kb][v] = orc.scores(case.q[t, b, h], K, I[v]).astype(np.float32)
    kv = ctx.kv_view(dc.K, dc.V, dc.seq_lens(t))
    out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
    ctx.lfps_sparse_attn(dc.q(t), kv, dev(idx), dev(scs) if with_scores else None, dc.k, out)
    out_h = out.cpu().numpy()
    worst = 0.0
    for b in range(spec.B):
        for h in range(spec.Hq):
            K, V = dc.group(b, h // 4)
            ref = orc.sparse_attn(case.q[t, b, h], K, V, idx[b, h, : case.k[b]])
            worst = max(worst, assert_out_close(out_h[b, h], ref, f"sparse_attn b{b} h{h}"))
    assert worst > 0


def test_k_equals_n_sparse_attention_is_full_attention(small_bf16):
    """The k = n invariant on the device: both kernels against the oracle's full attention."""
    dc = small_bf16
    case, spec = dc.case, dc.spec
    n0 = 300
    ctx = dc.make_ctx(max_k=n0)
    seq = dev(np.full(spec.B, n0, np.int32))
    kk = dev(np.full(spec.B, n0, np.int32))
    kv = ctx.kv_view(dc.K, dc.V, seq)
    idx = dev(np.tile(np.random.default_rng(1).permutation(n0).astype(np.int32), (spec.B, spec.Hq, 1)))
    o_sparse = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
    o_full = torch.zeros_like(o_sparse)
    ctx.lfps_sparse_attn(dc.q(0), kv, idx, None, kk, o_sparse)
    ctx.lfps_full_attn_decode(dc.q(0), kv, o_full)
    for b in range(spec.B):
        for h in (0, 13, 31):
            K, V = dc.group(b, h // 4)
            ref = orc.full_attn(case.q[0, b, h], K, V, n0)
            assert_out_close(o_sparse[b, h].cpu().numpy(), ref, "sparse k=n")
            assert_out_close(o_full[b, h].cpu().numpy(), ref, "full")


# ------------------------------------------------------------------------ baselines
@pytest.mark.parametrize("fx", ["small_bf16", "small_f32", "small_fp8", "small_fp8kv", "small_f16"])
def test_full_attention_and_exact_topk_baselines(fx, request):
    dc = request.getfixturevalue(fx)
    case, spec = dc.case, dc.spec
    ctx = dc.make_ctx()
    t = 3
    n = case.seq_lens(t)
    kv = ctx.kv_view(dc.K, dc.V, dc.seq_lens(t))
    out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
    ctx.lfps_full_attn_decode(dc.q(t), kv, out)
    idx = torch.zeros((spec.B, spec.Hq, case.kmax), dtype=torch.int32, device=DEV)
    sc = torch.zeros((spec.B, spec.Hq, case.kmax), dtype=torch.float32, device=DEV)
    ctx.lfps_exact_topk(dc.q(t), kv, dc.k, idx, sc)
    out_h, idx_h, sc_h = out.cpu().numpy(), idx.cpu().numpy(), sc.cpu().numpy()
    for b in range(spec.B):
        for h in range(spec.Hq):
            K, V = dc.group(b, h // 4)
            assert_out_close(out_h[b, h], orc.full_attn(case.q[t, b, h], K, V, int(n[b])), f"full b{b} h{h}")
            kb = int(case.k[b])
            I, S = orc.exact_topk(case.q[t, b, h], K, int(n[b]), kb)
            assert_topk_equal_mod_ties(idx_h[b, h, :kb], I, lambda p: orc.scores(case.q[t, b, h], K, p), kb,
                                       f"exact_topk b{b} h{h}")
            assert_scores_close(sc_h[b, h, :kb], orc.scores(case.q[t, b, h], K, idx_h[b, h, :kb]))


def test_cover_invariant_on_device(small_bf16):
    """Radius >= n: the candidate set covers every row, so LFPS Top-k == exact Top-k (same device scores)."""
    dc = small_bf16
    case, spec = dc.case, dc.spec
    ctx = dc.make_ctx(radius=case.Lcap)
    t = 1
    kv = ctx.kv_view(dc.K, dc.V, dc.seq_lens(t))
    prev = dev(np.zeros((spec.B, spec.Hq, case.kmax), np.int32))
    a = torch.zeros((spec.B, spec.Hq, case.kmax), dtype=torch.int32, device=DEV)
    b_ = torch.zeros_like(a)
    out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
    ctx.lfps_step(dc.q(t), kv, prev, dc.k, a, out)
    ctx.lfps_exact_topk(dc.q(t), kv, dc.k, b_)
    np.testing.assert_array_equal(a.cpu().numpy(), b_.cpu().numpy())


# ------------------------------------------------------------------------ whole step
@pytest.mark.parametrize("fx", ["small_bf16", "small_f32", "small_fp8", "small_fp8kv", "small_f16"])
def test_lfps_step_teacher_forced_multi_step(fx, request):
    """Each step the device gets the ORACLE's previous Top-k; candidates/Top-k/outputs must match."""
    dc = request.getfixturevalue(fx)
    case, spec = dc.case, dc.spec
    ctx = dc.make_ctx()
    prev = _teacher_inputs(dc, 1)            # exact Top-k of the seeding step
    for t in range(1, spec.T + 1):
        n = case.seq_lens(t)
        kv = ctx.kv_view(dc.K, dc.V, dc.seq_lens(t))
        idx = torch.zeros((spec.B, spec.Hq, case.kmax), dtype=torch.int32, device=DEV)
        sc = torch.zeros((spec.B, spec.Hq, case.kmax), dtype=torch.float32, device=DEV)
        out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
        ctx.lfps_step(dc.q(t), kv, dev(prev), dc.k, idx, out, sc)
        idx_h, out_h = idx.cpu().numpy(), out.cpu().numpy()
        nxt = np.full_like(prev, -1)
        for b in range(spec.B):
            kb = int(case.k[b])
            for g in range(spec.Hkv):
                K, V = dc.group(b, g)
                res = orc.lfps_step(case.q[t, b, 4 * g: 4 * g + 4], K, V,
                                    [prev[b, 4 * g + h, :kb] for h in range(4)], int(n[b]), kb, spec.r, 1, 0)
                for hh in range(4):
                    h = 4 * g + hh
                    got = idx_h[b, h, :kb]
                    nd = assert_topk_equal_mod_ties(got, res["topk_idx"][hh],
                                                    lambda p: orc.scores(case.q[t, b, h], K, p), kb, f"t{t} b{b} h{h}")
                    assert_out_close(out_h[b, h], orc.sparse_attn(case.q[t, b, h], K, V, got), f"out t{t} b{b} h{h}")
                    if nd == 0:
                        assert_out_close(out_h[b, h], res["out"][hh], f"out(oracle set) t{t} b{b} h{h}")
                    nxt[b, h, :kb] = res["topk_idx"][hh]
        prev = nxt


def test_lfps_step_free_running_tracks_exact_topk(small_bf16):
    """Chained on-device state: recall vs exact Top-k (Eq. 2) stays high, outputs close to full attention."""
    dc = small_bf16
    case, spec = dc.case, dc.spec
    ctx = dc.make_ctx()
    a = torch.zeros((spec.B, spec.Hq, case.kmax), dtype=torch.int32, device=DEV)
    b_ = torch.zeros_like(a)
    ex = torch.zeros_like(a)
    out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
    kv0 = ctx.kv_view(dc.K, dc.V, dc.seq_lens(0))
    ctx.lfps_exact_topk(dc.q(0), kv0, dc.k, a)
    etas = []
    for t in range(1, spec.T + 1):
        kv = ctx.kv_view(dc.K, dc.V, dc.seq_lens(t))
        ctx.lfps_step(dc.q(t), kv, a, dc.k, b_, out)
        ctx.lfps_exact_topk(dc.q(t), kv, dc.k, ex)
        got, want = b_.cpu().numpy(), ex.cpu().numpy()
        etas.append(np.mean([orc.overlap(got[b, h], want[b, h]) for b in range(spec.B) for h in range(spec.Hq)]))
        a, b_ = b_, a
    assert min(etas) > 0.8, etas


# ------------------------------------------------------------------------ edge cases and errors
def test_degenerate_lengths_and_budgets():
    from paper_2506_15704_amd.binding import Lfps
    B, Hq, Hkv, D, Lcap, kmax = 4, 32, 8, 128, 300, 8
    rng = np.random.default_rng(3)
    ctx = Lfps(batch=B, max_seq_len=Lcap, max_k=kmax, radius=2, n_recent=1)
    K = torch.randn((B, Hkv, Lcap, D), device=DEV).to(torch.bfloat16)
    V = torch.randn((B, Hkv, Lcap, D), device=DEV).to(torch.bfloat16)
    q = torch.randn((B, Hq, D), device=DEV)
    n = np.array([1, 5, 300, 0], dtype=np.int32)            # single row; n < k; full; empty request
    k = np.array([8, 8, 0, 4], dtype=np.int32)              # k_b = 0 for request 2
    prev = rng.integers(0, 300, size=(B, Hq, kmax)).astype(np.int32)
    kv = ctx.kv_view(K, V, dev(n))
    idx = torch.full((B, Hq, kmax), 77, dtype=torch.int32, device=DEV)
    out = torch.full((B, Hq, D), 5.0, dtype=torch.float32, device=DEV)
    ctx.lfps_step(q, kv, dev(prev), dev(k), idx, out)
    idx_h, out_h = idx.cpu().numpy(), out.cpu().numpy()
    Kh, Vh, qh = K.float().cpu().numpy(), V.float().cpu().numpy(), q.cpu().numpy()
    for b in range(B):
        for h in range(Hq):
            g = h // 4
            res = orc.lfps_step(qh[b, 4 * g:4 * g + 4], Kh[b, g], Vh[b, g], [prev[b, 4 * g + i, : k[b]] for i in range(4)],
                                int(n[b]), int(k[b]), 2, 1, 0)
            want = np.sort(res["topk_idx"][h % 4])
            np.testing.assert_array_equal(valid_row(idx_h[b, h]), want)
            assert np.all(idx_h[b, h, len(want):] == -1)
            if len(want):
                assert_out_close(out_h[b, h], res["out"][h % 4], f"b{b} h{h}")
            else:
                assert np.all(out_h[b, h] == 0)
    full = torch.full((B, Hq, D), 5.0, dtype=torch.float32, device=DEV)
    ctx.lfps_full_attn_decode(q, kv, full)
    f = full.cpu().numpy()
    np.testing.assert_allclose(f[0, 0], Vh[0, 0, 0], atol=1e-6)   # one row: its value
    assert np.all(f[3] == 0)                                      # empty request


def test_argument_errors_return_einval():
    from paper_2506_15704_amd import binding as b
    ctx = b.Lfps(batch=1, max_seq_len=256, max_k=16, radius=1)
    K = torch.zeros((1, 8, 256, 128), dtype=torch.bfloat16, device=DEV)
    n = dev(np.array([256], np.int32))
    kk = dev(np.array([16], np.int32))
    q = torch.zeros((1, 32, 128), device=DEV)
    buf = torch.zeros((1, 32, 16), dtype=torch.int32, device=DEV)
    out = torch.zeros((1, 32, 128), device=DEV)
    kv = ctx.kv_view(K, K, n)
    with pytest.raises(b.LfpsError) as ei:                       # aliasing prev_topk / topk_idx
        ctx.lfps_step(q, kv, buf, kk, buf, out)
    assert ei.value.code == b.LFPS_EINVAL and "overlap" in str(ei.value)
    bad = b.lfps_kv(K.data_ptr(), K.data_ptr(), K.stride(0), K.stride(1), 64, n.data_ptr())
    with pytest.raises(b.LfpsError) as ei:                       # row stride smaller than head_dim
        ctx.lfps_full_attn_decode(q, bad, out)
    assert ei.value.code == b.LFPS_EINVAL
    nov = b.lfps_kv(K.data_ptr(), None, K.stride(0), K.stride(1), K.stride(2), n.data_ptr())
    with pytest.raises(b.LfpsError):                             # V missing where it is needed
        ctx.lfps_full_attn_decode(q, nov, out)
    with pytest.raises(b.LfpsError):                             # NULL output
        ctx.lfps_exact_topk(q, kv, kk, None)
    with pytest.raises(TypeError):                               # wrong dtype caught by the binding
        ctx.lfps_exact_topk(q, kv, kk, buf.float())
    ctx.lfps_exact_topk(q, kv, kk, buf)                          # context still usable afterwards
    torch.cuda.synchronize()


def test_strided_cache_layout_b_l_h_d(small_bf16):
    """[B, Lcap, Hkv, D] storage viewed as [B, Hkv, Lcap, D] gives the same results."""
    dc = small_bf16
    case, spec = dc.case, dc.spec
    ctx = dc.make_ctx()
    Kt = dc.K.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    Vt = dc.V.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert Kt.stride(2) == spec.Hkv * spec.D
    prev = dev(_teacher_inputs(dc, 1))
    outs = []
    for K, V in ((dc.K, dc.V), (Kt, Vt)):
        kv = ctx.kv_view(K, V, dc.seq_lens(1))
        idx = torch.zeros((spec.B, spec.Hq, case.kmax), dtype=torch.int32, device=DEV)
        out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
        ctx.lfps_step(dc.q(1), kv, prev, dc.k, idx, out)
        full = torch.zeros_like(out)
        ctx.lfps_full_attn_decode(dc.q(1), kv, full)
        outs.append((idx.cpu().numpy(), out.cpu().numpy(), full.cpu().numpy()))
    for x, y in zip(*outs):
        np.testing.assert_array_equal(x, y)


def test_timing_interface(small_bf16):
    dc = small_bf16
    case, spec = dc.case, dc.spec
    ctx = dc.make_ctx()
    ctx.lfps_timing_enable(True)
    kv = ctx.kv_view(dc.K, dc.V, dc.seq_lens(1))
    a = torch.zeros((spec.B, spec.Hq, case.kmax), dtype=torch.int32, device=DEV)
    b_ = torch.zeros_like(a)
    out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
    ctx.lfps_exact_topk(dc.q(0), kv, dc.k, a)
    for _ in range(3):
        ctx.lfps_step(dc.q(1), kv, a, dc.k, b_, out)
    tm = ctx.lfps_timing_read()
    assert tm["candidates"][1] == 3 and tm["dense_score"][1] == 1 and tm["select"][1] == 1
    # the first step of a new context has no history and takes the unfiltered pair of kernels
    assert tm["gather_score"][1] == 1 and tm["select_attend"][1] == 1 and tm["gather_score"][0] > 0
    # a filtered step is three launches: the heads the filter leaves short are rescored inside the select kernel
    assert tm["filter_score"][1] == 2 and tm["filter_select_attend"][1] == 2 and tm["filter_score"][0] > 0
    assert tm["sparse_attn"][1] == 0                   # the chained step attends inside its select kernels
    assert all(v == (0.0, 0) for v in ctx.lfps_timing_read().values())


# ------------------------------------------------------------------------ filtered scoring inside lfps_step
@pytest.mark.parametrize("fx", ["small_bf16", "small_fp8", "small_f16"])
def test_filtered_step_equals_unfiltered_step_whatever_the_history(fx, request):
    """lfps_step with the score filter (history from the previous call, including deliberately wrong
    histories that force the rescoring path) returns bit-identical Top-k and outputs to the
    unfiltered path."""
    dc = request.getfixturevalue(fx)
    case, spec = dc.case, dc.spec
    ref, flt = dc.make_ctx(), dc.make_ctx()
    ref.lfps_set_filter(False)
    shp = (spec.B, spec.Hq, case.kmax)
    prev = dev(_teacher_inputs(dc, 1))
    flt.lfps_timing_enable(True)
    used_filter = 0
    for rnd, (t, qscale) in enumerate([(1, 1.0), (2, 1.0), (3, 1.0), (3, 4.0), (4, 1.0), (2, 0.01), (3, 1.0), (4, 1.0)]):
        kv = ref.kv_view(dc.K, dc.V, dc.seq_lens(t))
        q = dc.q(t) * qscale                      # scaled queries leave a history that is far too high / low
        outs = []
        for ctx in (ref, flt):
            idx = torch.zeros(shp, dtype=torch.int32, device=DEV)
            sc = torch.zeros(shp, dtype=torch.float32, device=DEV)
            out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
            ctx.lfps_step(q, kv, prev, dc.k, idx, out, sc)
            outs.append((idx.cpu().numpy(), sc.cpu().numpy(), out.cpu().numpy()))
        for a, b_ in zip(*outs):
            np.testing.assert_array_equal(a, b_, err_msg=f"round {rnd}")
        tm = flt.lfps_timing_read()
        filtered = 0 if rnd == 0 else 1                # a new context's first step has no history to filter with
        assert tm["filter_score"][1] == filtered and tm["filter_select_attend"][1] == filtered
        assert tm["gather_score"][1] == 1 - filtered and tm["select_attend"][1] == 1 - filtered
        prev = torch.from_numpy(outs[0][0]).to(DEV)
    flt.lfps_reset_history()
    kv = ref.kv_view(dc.K, dc.V, dc.seq_lens(4))
    a = torch.zeros(shp, dtype=torch.int32, device=DEV)
    b_ = torch.zeros_like(a)
    out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
    ref.lfps_step(dc.q(4), kv, prev, dc.k, a, out)
    flt.lfps_step(dc.q(4), kv, prev, dc.k, b_, out)
    np.testing.assert_array_equal(a.cpu().numpy(), b_.cpu().numpy())


# ------------------------------------------------------------------------ other GQA group sizes
@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (16, 8), (4, 1)])
def test_lfps_step_other_group_sizes(Hq, Hkv):
    """G = 1, 2 and a single KV head: two chained steps (the second one through the score filter)."""
    dc = DeviceCase(gen.tiny_spec(f"g{Hq}_{Hkv}", B=2, L=1500, k=64, r=2, T=3, Hq=Hq, Hkv=Hkv))
    case, spec = dc.case, dc.spec
    G = spec.G
    ctx = dc.make_ctx()
    prev = np.full((spec.B, spec.Hq, case.kmax), -1, dtype=np.int32)
    for b in range(spec.B):
        for h in range(spec.Hq):
            K, _ = dc.group(b, h // G)
            prev[b, h] = orc.exact_topk(case.q[0, b, h], K, int(case.seq_lens0[b]), int(case.k[b]))[0]
    for t in (1, 2, 3):
        kv = ctx.kv_view(dc.K, dc.V, dc.seq_lens(t))
        idx = torch.zeros((spec.B, spec.Hq, case.kmax), dtype=torch.int32, device=DEV)
        out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
        ctx.lfps_step(dc.q(t), kv, dev(prev), dc.k, idx, out)
        idx_h, out_h = idx.cpu().numpy(), out.cpu().numpy()
        nxt = np.full_like(prev, -1)
        for b in range(spec.B):
            kb, n = int(case.k[b]), int(case.seq_lens(t)[b])
            for g in range(spec.Hkv):
                K, V = dc.group(b, g)
                res = orc.lfps_step(case.q[t, b, G * g: G * g + G], K, V, [prev[b, G * g + i, :kb] for i in range(G)],
                                    n, kb, spec.r, 1, 0)
                for hh in range(G):
                    h = G * g + hh
                    assert_topk_equal_mod_ties(idx_h[b, h, :kb], res["topk_idx"][hh],
                                               lambda p: orc.scores(case.q[t, b, h], K, p), kb, f"G{G} t{t} b{b} h{h}")
                    assert_out_close(out_h[b, h], orc.sparse_attn(case.q[t, b, h], K, V, idx_h[b, h, :kb]), f"G{G} out")
                    nxt[b, h, :kb] = res["topk_idx"][hh]
        prev = nxt
    full = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
    ctx.lfps_full_attn_decode(dc.q(3), ctx.kv_view(dc.K, dc.V, dc.seq_lens(3)), full)
    K, V = dc.group(1, spec.Hkv - 1)
    assert_out_close(full[1, spec.Hq - 1].cpu().numpy(), orc.full_attn(case.q[3, 1, spec.Hq - 1], K, V, int(case.seq_lens(3)[1])), "full")
    tm_ctx = dc.make_ctx()
    del tm_ctx


@pytest.mark.parametrize("seed", [1, 20250616, 987654321])
def test_small_workload_other_seeds(seed):
    """The 4K fp32 workload under three more seeds: teacher-forced steps on two sampled groups."""
    import dataclasses
    dc = DeviceCase(dataclasses.replace(gen.C1, name=f"C1s{seed}", seed=seed, T=4))
    case, spec = dc.case, dc.spec
    ctx = dc.make_ctx()
    samples = [(0, seed % 8), (0, (seed + 3) % 8)]
    seedk = torch.zeros((spec.B, spec.Hq, case.kmax), dtype=torch.int32, device=DEV)
    ctx.lfps_exact_topk(dc.q(0), ctx.kv_view(dc.K, dc.V, dc.seq_lens(0)), dc.k, seedk)
    prev_dev = seedk.clone()
    prev_orc = {}
    for (b, g) in samples:
        K, _ = dc.group(b, g)
        prev_orc[(b, g)] = [orc.exact_topk(case.q[0, b, 4 * g + hh], K, int(case.seq_lens0[b]), int(case.k[b]))[0] for hh in range(4)]
    for t in range(1, spec.T + 1):
        for (b, g) in samples:
            for hh in range(4):
                prev_dev[b, 4 * g + hh] = torch.from_numpy(prev_orc[(b, g)][hh].astype(np.int32)).to(DEV)
        nxt = torch.zeros_like(prev_dev)
        out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
        ctx.lfps_step(dc.q(t), ctx.kv_view(dc.K, dc.V, dc.seq_lens(t)), prev_dev, dc.k, nxt, out)
        idx_h, out_h = nxt.cpu().numpy(), out.cpu().numpy()
        for (b, g) in samples:
            K, V = dc.group(b, g)
            kb, n = int(case.k[b]), int(case.seq_lens(t)[b])
            res = orc.lfps_step(case.q[t, b, 4 * g: 4 * g + 4], K, V, prev_orc[(b, g)], n, kb, spec.r, 1, 0)
            for hh in range(4):
                h = 4 * g + hh
                assert_topk_equal_mod_ties(idx_h[b, h, :kb], res["topk_idx"][hh], lambda p: orc.scores(case.q[t, b, h], K, p), kb,
                                           f"seed {seed} t{t} h{h}")
                assert_out_close(out_h[b, h], orc.sparse_attn(case.q[t, b, h], K, V, idx_h[b, h, :kb]), f"seed {seed} out")
            prev_orc[(b, g)] = res["topk_idx"]
        prev_dev = nxt


def test_fp16_cache_extreme_values():
    """fp16 keys at the ends of the format (subnormal-only rows, rows near the largest finite value) against
    queries of very different size: the fp16 matrix-core path (query split into three scaled fp16 terms) keeps
    the fp32-accumulate accuracy, and subnormal keys are not flushed."""
    from paper_2506_15704_amd.binding import Lfps
    rng = np.random.default_rng(5)
    L, D, Hq = 256, 128, 4
    K = rng.standard_normal((L, D)).astype(np.float32)
    K[64:128] = rng.integers(-1023, 1024, size=(64, D)).astype(np.float32) * np.float32(2.0 ** -24)   # subnormal fp16
    K[128:192] = rng.choice([-1.0, 1.0], size=(64, D)).astype(np.float32) * rng.uniform(2e3, 6e4, size=(64, D)).astype(np.float32)
    K[192:224] *= np.float32(1e-3)
    K16 = torch.from_numpy(K).to(torch.float16)
    Kf = K16.float().numpy()                                  # the stored values
    assert np.abs(Kf[64:128]).max() < 6.2e-5 and np.abs(Kf[64:128]).max() > 0 and np.isfinite(Kf).all()
    q = rng.standard_normal((1, Hq, D)).astype(np.float32)
    q[0, 1] *= np.float32(1e3)
    q[0, 2] *= np.float32(1e-3)
    q[0, 3] *= np.float32(1e4)
    ctx = Lfps(batch=1, n_q_heads=Hq, n_kv_heads=1, kv_dtype="f16", max_seq_len=L, max_k=32, radius=0, cand_cap=L)
    Kd = K16.reshape(1, 1, L, D).to(DEV)
    Vd = torch.zeros_like(Kd)
    n = torch.tensor([L], dtype=torch.int32, device=DEV)
    kv = ctx.kv_view(Kd, Vd, n)
    cand = torch.arange(L, dtype=torch.int32, device=DEV).reshape(1, 1, L)
    cnt = torch.tensor([[L]], dtype=torch.int32, device=DEV)
    k = torch.tensor([32], dtype=torch.int32, device=DEV)
    idx = torch.zeros((1, Hq, 32), dtype=torch.int32, device=DEV)
    cs = torch.zeros((1, Hq, L), dtype=torch.float32, device=DEV)
    ctx.lfps_score_topk(dev(q), kv, cand, cnt, k, idx, None, cs)
    dense = torch.zeros((1, Hq, 32), dtype=torch.int32, device=DEV)
    ctx.lfps_exact_topk(dev(q), kv, k, dense)
    cs_h, idx_h, dense_h = cs.cpu().numpy(), idx.cpu().numpy(), dense.cpu().numpy()
    for h in range(Hq):
        ref = orc.scores(q[0, h], Kf, np.arange(L))
        assert_scores_close(cs_h[0, h], ref, f"fp16 extremes h{h}")
        I, _ = orc.exact_topk(q[0, h], Kf, L, 32)
        for got, what in ((idx_h[0, h], "gathered"), (dense_h[0, h], "dense")):
            assert_topk_equal_mod_ties(got, I, lambda p: orc.scores(q[0, h], Kf, p), 32, f"fp16 extremes {what} h{h}")
    # the subnormal rows carry signal for the large query: a flush to zero would be far outside the tolerance
    assert np.abs(orc.scores(q[0, 1], Kf, np.arange(64, 128))).max() > 0.05
    ctx.close()


def test_non_finite_queries_stay_in_bounds_and_in_their_group(small_bf16):
    """A NaN query and an infinite one (garbage in): the step still ends, every selected index of those heads is a
    valid, distinct row of the request, the count is right, and the heads of the other KV groups get exactly what
    a clean run gives them (a group shares nothing with another).  Two steps, so the second goes through the score filter."""
    dc = small_bf16
    case, spec = dc.case, dc.spec
    shp = (spec.B, spec.Hq, case.kmax)
    clean, dirty = dc.make_ctx(), dc.make_ctx()
    seed = torch.zeros(shp, dtype=torch.int32, device=DEV)
    clean.lfps_exact_topk(dc.q(0), clean.kv_view(dc.K, dc.V, dc.seq_lens(0)), dc.k, seed)
    bad_heads = [(0, 1), (1, 6), (2, 31)]                      # in KV groups 0, 1 and 7
    bad_groups = {(b, h // spec.G) for b, h in bad_heads}
    prev_c, prev_d = seed, seed
    for t in (1, 2):
        q = dc.q(t).clone()
        qd = q.clone()
        qd[0, 1, 5] = float("nan")
        qd[1, 6, :] = float("inf")
        qd[2, 31, 100] = float("-inf")
        res = []
        for ctx, qq, prev in ((clean, q, prev_c), (dirty, qd, prev_d)):
            idx = torch.full(shp, -5, dtype=torch.int32, device=DEV)
            sc = torch.zeros(shp, dtype=torch.float32, device=DEV)
            out = torch.zeros((spec.B, spec.Hq, spec.D), dtype=torch.float32, device=DEV)
            ctx.lfps_step(qq, ctx.kv_view(dc.K, dc.V, dc.seq_lens(t)), prev, dc.k, idx, out, sc)
            assert ctx.lfps_poll_status() == 0
            res.append((idx, out))
        (ic, oc), (id_, od) = res
        n = case.seq_lens(t)
        idh = id_.cpu().numpy()
        for b in range(spec.B):
            kb = int(case.k[b])
            for h in range(spec.Hq):
                if (b, h // spec.G) in bad_groups:
                    got = idh[b, h, :kb]
                    assert np.all((got >= 0) & (got < n[b])) and len(np.unique(got)) == kb, f"t{t} b{b} h{h}"
                    assert np.all(idh[b, h, kb:] == -1)
                else:
                    assert torch.equal(id_[b, h], ic[b, h]) and torch.equal(od[b, h], oc[b, h]), f"t{t} b{b} h{h}"
        prev_c, prev_d = ic, id_
    clean.close()
    dirty.close()


def test_calibration_copy_copies():
    """The counter-calibration kernel is a plain copy: every byte arrives, sizes that are not a multiple of
    16 bytes are refused."""
    from paper_2506_15704_amd.binding import LfpsError, lfps_calib_copy
    src = torch.arange(0, 3 * 1024 * 1024 + 16, dtype=torch.int32, device=DEV)
    dst = torch.zeros_like(src)
    lfps_calib_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    odd_src = torch.zeros(20, dtype=torch.uint8, device=DEV)
    with pytest.raises(LfpsError):
        lfps_calib_copy(torch.zeros_like(odd_src), odd_src)


def test_two_contexts_on_two_streams(small_bf16, small_fp8):
    """Contexts share nothing: two of them stepping at the same time on two streams (default priority) give what
    each gives alone."""
    cases = (small_bf16, small_fp8)
    alone = []
    for dc in cases:
        shp = (dc.spec.B, dc.spec.Hq, dc.case.kmax)
        ctx = dc.make_ctx()
        prev = torch.zeros(shp, dtype=torch.int32, device=DEV)
        ctx.lfps_exact_topk(dc.q(0), ctx.kv_view(dc.K, dc.V, dc.seq_lens(0)), dc.k, prev)
        outs = []
        for t in (1, 2, 3):
            idx = torch.zeros(shp, dtype=torch.int32, device=DEV)
            out = torch.zeros((dc.spec.B, dc.spec.Hq, dc.spec.D), dtype=torch.float32, device=DEV)
            ctx.lfps_step(dc.q(t), ctx.kv_view(dc.K, dc.V, dc.seq_lens(t)), prev, dc.k, idx, out)
            outs.append((idx, out))
            prev = idx
        torch.cuda.synchronize()
        alone.append(outs)
        ctx.close()
    streams = [torch.cuda.Stream(device=DEV) for _ in cases]
    ctxs, prevs, together = [], [], [[], []]
    for i, dc in enumerate(cases):
        shp = (dc.spec.B, dc.spec.Hq, dc.case.kmax)
        ctxs.append(dc.make_ctx())
        prevs.append(torch.zeros(shp, dtype=torch.int32, device=DEV))
        ctxs[i].lfps_exact_topk(dc.q(0), ctxs[i].kv_view(dc.K, dc.V, dc.seq_lens(0)), dc.k, prevs[i])
    inputs = [[(dc.q(t), dc.seq_lens(t)) for t in (1, 2, 3)] for dc in cases]     # made on the default stream
    torch.cuda.synchronize()
    for t in range(3):
        for i, dc in enumerate(cases):
            with torch.cuda.stream(streams[i]):
                shp = (dc.spec.B, dc.spec.Hq, dc.case.kmax)
                idx = torch.zeros(shp, dtype=torch.int32, device=DEV)
                out = torch.zeros((dc.spec.B, dc.spec.Hq, dc.spec.D), dtype=torch.float32, device=DEV)
                q, sl = inputs[i][t]
                ctxs[i].lfps_step(q, ctxs[i].kv_view(dc.K, dc.V, sl), prevs[i], dc.k, idx, out)
                together[i].append((idx, out))
                prevs[i] = idx
    torch.cuda.synchronize()
    for i in range(2):
        for t in range(3):
            assert torch.equal(together[i][t][0], alone[i][t][0]) and torch.equal(together[i][t][1], alone[i][t][1]), (i, t)
        ctxs[i].close()
