"""Seeded random configurations of the chained step: head grouping, batch, ragged lengths, per-request
budgets, radius, always-present rows, cache dtype (bf16 / fp16 / fp32 / FP8 keys / FP8 keys and values) and layout (contiguous / paged)
drawn together, so that combinations no hand-written case names are exercised.  Teacher-forced: every step
the device starts from the oracle's previous Top-k and is checked against the oracle's step (candidate counts
exactly; Top-k, scores and outputs by the rules of tests/harness.py)."""
import numpy as np
import pytest
import torch

import gen
from gen import device as gen_device
from oracle import lfps_oracle as orc
from tests.harness import (DEV, DeviceCase, assert_out_close, assert_scores_close, assert_topk_equal_mod_ties, dev,
                           valid_row)

pytestmark = pytest.mark.gpu

N_CONFIGS = 40


def _draw(i):
    rng = np.random.default_rng(7000 + i)
    Hq, Hkv = [(32, 8), (16, 8), (8, 8), (4, 1), (8, 2), (2, 1)][int(rng.integers(0, 6))]
    lo = int(rng.integers(24, 120)) if i % 6 == 5 else int(rng.integers(24, 3000))     # every sixth: very short contexts
    hi = lo + (int(rng.integers(0, 100)) if i % 6 == 5 else int(rng.integers(0, 2500)))
    kind = "f16" if i % 8 == 6 else ("bf16", "f32", "fp8", "fp8kv")[i % 4]
    cfg = dict(Hq=Hq, Hkv=Hkv, B=int(rng.integers(1, 5)), L_range=(lo, hi), kmax=int(rng.integers(1, min(lo, 160) + 1)),
               r=int(rng.choice([0, 1, 2, 4, 9])), n_recent=int(rng.integers(0, 4)), n_sink=int(rng.integers(0, 5)),
               kv_dtype=kind if kind in ("f32", "f16") else "bf16", k_dtype="fp8" if kind in ("fp8", "fp8kv") else "",
               v_dtype="fp8" if kind == "fp8kv" else "",
               paged=[None, (1, "block_head_row"), (16, "block_row_head"), (64, "block_head_row")][int(rng.integers(0, 4))])
    cfg["k"] = rng.integers(1, cfg["kmax"] + 1, size=cfg["B"]).astype(np.int32)
    cfg["k"][int(rng.integers(0, cfg["B"]))] = cfg["kmax"]
    return cfg


@pytest.mark.parametrize("i", range(N_CONFIGS))
def test_random_configuration_chained_steps(i):
    _run(i, _draw(i), T=3)


# Many requests with short contexts: hundreds of (request, KV group) units, so that one wave of the filtered
# scoring kernel crosses several groups and the group tables are read in more than one batch of 64.
MANY = [dict(Hq=32, Hkv=8, B=48, L_range=(150, 700), kmax=40, r=2, n_recent=1, n_sink=0, kv_dtype="bf16", k_dtype="",
             v_dtype="", paged=None),
        dict(Hq=8, Hkv=8, B=70, L_range=(90, 400), kmax=24, r=1, n_recent=2, n_sink=4, kv_dtype="bf16", k_dtype="fp8",
             v_dtype="", paged=(16, "block_head_row")),
        dict(Hq=16, Hkv=8, B=33, L_range=(64, 900), kmax=33, r=4, n_recent=0, n_sink=1, kv_dtype="f32", k_dtype="",
             v_dtype="", paged=None)]


@pytest.mark.parametrize("j", range(len(MANY)))
def test_many_requests_short_contexts(j):
    c = dict(MANY[j])
    rng = np.random.default_rng(9100 + j)
    c["k"] = rng.integers(1, c["kmax"] + 1, size=c["B"]).astype(np.int32)
    c["k"][int(rng.integers(0, c["B"]))] = c["kmax"]
    _run(1000 + j, c, T=2)


# Longer contexts and larger budgets: the dense select of the seeding step streams its scores (more than fit
# the LDS copy), candidate sets reach the whole context, survivor lists of the filtered pass are long.
MID = [dict(Hq=8, Hkv=2, B=1, L_range=(34317, 37140), kmax=1018, r=4, n_recent=0, n_sink=4, kv_dtype="bf16", k_dtype="fp8",
            v_dtype="fp8", paged=(128, "block_row_head")),
       dict(Hq=4, Hkv=1, B=2, L_range=(33000, 36000), kmax=1500, r=2, n_recent=2, n_sink=0, kv_dtype="f16", k_dtype="",
            v_dtype="", paged=None),
       dict(Hq=16, Hkv=8, B=1, L_range=(25591, 29514), kmax=532, r=4, n_recent=3, n_sink=2, kv_dtype="bf16", k_dtype="",
            v_dtype="", paged=(16, "block_head_row")),
       dict(Hq=8, Hkv=2, B=1, L_range=(9977, 12669), kmax=1265, r=2, n_recent=1, n_sink=4, kv_dtype="f32", k_dtype="",
            v_dtype="", paged=None),
       # a budget beyond what the filtered select holds at two workgroups per CU: the larger survivor list
       dict(Hq=4, Hkv=1, B=1, L_range=(21000, 22000), kmax=4500, r=1, n_recent=1, n_sink=0, kv_dtype="bf16", k_dtype="",
            v_dtype="", paged=None),
       # a budget that no survivor list can hold: such a context runs without the filtered pass
       dict(Hq=4, Hkv=1, B=1, L_range=(15000, 15500), kmax=14000, r=1, n_recent=1, n_sink=2, kv_dtype="bf16", k_dtype="",
            v_dtype="", paged=None)]


@pytest.mark.parametrize("j", range(len(MID)))
def test_mid_size_configurations(j):
    c = dict(MID[j])
    rng = np.random.default_rng(9300 + j)
    c["k"] = rng.integers(c["kmax"] // 2, c["kmax"] + 1, size=c["B"]).astype(np.int32)
    c["k"][int(rng.integers(0, c["B"]))] = c["kmax"]
    _run(2000 + j, c, T=3)


def _run(i, c, T):
    spec = gen.tiny_spec(f"rnd{i}", B=c["B"], L=None, L_range=c["L_range"], k=c["kmax"], r=c["r"], T=T, Hq=c["Hq"],
                         Hkv=c["Hkv"], kv_dtype=c["kv_dtype"], k_dtype=c["k_dtype"], v_dtype=c["v_dtype"], seed=31000 + i,
                         recency=min(16, c["L_range"][0] // 2))
    dc = DeviceCase(spec)
    case, G = dc.case, spec.G
    ctx = dc.make_ctx(n_recent=c["n_recent"], n_sink=c["n_sink"])
    if c["paged"]:
        Kp, Vp, table = gen_device.paginate(dc.K, dc.V, c["paged"][0], seed=i, layout=c["paged"][1])
        view = lambda t: ctx.paged_kv_view(Kp, Vp, table, dc.seq_lens(t))
    else:
        view = lambda t: ctx.kv_view(dc.K, dc.V, dc.seq_lens(t))
    k_dev = dev(c["k"])
    shp = (spec.B, spec.Hq, case.kmax)
    what = f"config {i}: {c}"
    # the seeding step: the oracle's exact Top-k is the history the device is given (teacher forcing: at every
    # step the device starts from the oracle's previous Top-k, never the other way round)
    seed_dev = torch.full(shp, -1, dtype=torch.int32, device=DEV)
    ctx.lfps_exact_topk(dc.q(0), view(0), k_dev, seed_dev)
    seed_h = seed_dev.cpu().numpy()
    prev = np.full(shp, -1, dtype=np.int32)
    for b in range(spec.B):
        kb, nb = int(c["k"][b]), int(case.seq_lens0[b])
        for h in range(spec.Hq):
            K, _ = dc.group(b, h // G)
            I, _ = orc.exact_topk(case.q[0, b, h], K, nb, kb)
            assert_topk_equal_mod_ties(seed_h[b, h, :kb], I, lambda p: orc.scores(case.q[0, b, h], K, p), kb,
                                       f"{what}: exact Top-k b{b} h{h}")
            prev[b, h, :kb] = I
    for t in range(1, T + 1):
        idx = torch.full(shp, -9, dtype=torch.int32, device=DEV)
        sc = torch.zeros(shp, dtype=torch.float32, device=DEV)
        out = torch.full((spec.B, spec.Hq, spec.D), 7.0, dtype=torch.float32, device=DEV)
        cnt = torch.zeros((spec.B, spec.Hkv), dtype=torch.int32, device=DEV)
        ctx.lfps_step(dc.q(t), view(t), dev(prev), k_dev, idx, out, sc)
        ctx.lfps_copy_cand_count(cnt)
        assert ctx.lfps_poll_status() == 0, what
        i_h, s_h, o_h, c_h = (x.cpu().numpy() for x in (idx, sc, out, cnt))
        n = case.seq_lens(t)
        nxt = np.full(shp, -1, dtype=np.int32)
        for b in range(spec.B):
            kb, nb = int(c["k"][b]), int(n[b])
            for g in range(spec.Hkv):
                K, V = dc.group(b, g)
                res = orc.lfps_step(case.q[t, b, G * g: G * g + G], K, V,
                                    [valid_row(prev[b, G * g + h, :kb]) for h in range(G)], nb, kb, spec.r,
                                    c["n_recent"], c["n_sink"])
                assert c_h[b, g] == len(res["cand"]), f"{what}: t{t} b{b} g{g} candidate count"
                ksel = min(kb, len(res["cand"]))
                for hh in range(G):
                    h = G * g + hh
                    assert (i_h[b, h, ksel:] == -1).all(), f"{what}: padding"
                    got = i_h[b, h, :ksel]
                    assert np.all(np.diff(got) > 0), f"{what}: indices not ascending"
                    assert_topk_equal_mod_ties(got, res["topk_idx"][hh], lambda p: orc.scores(case.q[t, b, h], K, p),
                                               ksel, f"{what}: t{t} b{b} h{h}")
                    assert_scores_close(s_h[b, h, :ksel], orc.scores(case.q[t, b, h], K, got), f"{what}: scores")
                    assert_out_close(o_h[b, h], orc.sparse_attn(case.q[t, b, h], K, V, got), f"{what}: t{t} b{b} h{h}")
                    nxt[b, h, :ksel] = res["topk_idx"][hh]
        prev = nxt
    ctx.close()
