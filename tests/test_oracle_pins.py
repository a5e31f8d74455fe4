"""Pins of the CPU oracle against things other than itself: library routines, closed
forms, brute force over all positions, the offset set the paper prints, and the
method's invariants (cover => exact Top-k; k = n => full attention; fixed point)."""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from oracle import lfps_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(seed, n, d=16):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(d), rng.standard_normal((n, d)), rng.standard_normal((n, d)))


# ----------------------------------------------------------------- full attention
@pytest.mark.parametrize("n,d", [(1, 8), (7, 16), (300, 128)])
def test_full_attn_matches_library_softmax(n, d):
    q, K, V = _rand(n * 31 + d, n, d)
    tq, tK, tV = (torch.from_numpy(x) for x in (q, K, V))
    ref = torch.softmax((tK @ tq) / math.sqrt(d), dim=0) @ tV
    np.testing.assert_allclose(orc.full_attn(q, K, V, n), ref.numpy(), rtol=1e-12, atol=1e-13)


def test_full_attn_uses_only_first_n_rows():
    q, K, V = _rand(3, 50)
    a = orc.full_attn(q, K, V, 20)
    K2, V2 = K.copy(), V.copy()
    K2[20:] = 99.0
    V2[20:] = -99.0
    np.testing.assert_array_equal(a, orc.full_attn(q, K2, V2, 20))


def test_full_attn_equal_keys_gives_mean_value():
    q, _, V = _rand(5, 40)
    K = np.tile(np.linspace(-1, 1, 16), (40, 1))
    np.testing.assert_allclose(orc.full_attn(q, K, V, 40), V.mean(axis=0), rtol=1e-12)


def test_full_attn_dominant_key_gives_its_value():
    q, K, V = _rand(6, 40)
    K[17] = 200.0 * q / np.linalg.norm(q)
    np.testing.assert_allclose(orc.full_attn(q, K, V, 40), V[17], atol=1e-9)


def test_scores_are_scaled_dot_products_elementwise():
    q, K, _ = _rand(8, 9, 4)
    s = orc.scores(q, K)
    for i in range(9):
        want = sum(q[c] * K[i, c] for c in range(4)) / 2.0      # sqrt(4) = 2
        assert abs(s[i] - want) < 1e-14
    # not the transposed product: a K with distinct rows/cols must discriminate
    assert not np.allclose(s[:4], (K[:4, :4].T @ q) / 2.0)


# ----------------------------------------------------------------- exact Top-k
@pytest.mark.parametrize("n,k", [(10, 3), (257, 64), (1000, 1000)])
def test_exact_topk_against_full_sort(n, k):
    q, K, _ = _rand(n + k, n)
    idx, sc = orc.exact_topk(q, K, n, k)
    s = (K @ q) / math.sqrt(16)
    want = np.argsort(-s, kind="stable")[:k]
    assert set(idx.tolist()) == set(want.tolist())
    tv, ti = torch.topk(torch.from_numpy(s), k)
    assert set(idx.tolist()) == set(ti.tolist())
    np.testing.assert_allclose(np.sort(sc), np.sort(tv.numpy()), rtol=0, atol=0)
    assert np.all(np.diff(sc) <= 0)                      # best first
    if k == n:
        assert sorted(idx.tolist()) == list(range(n))


def test_exact_topk_ties_prefer_lower_index():
    q = np.ones(4)
    K = np.zeros((6, 4))
    K[[1, 3, 4]] = 1.0                                    # three equal best scores
    idx, _ = orc.exact_topk(q, K, 6, 2)
    assert idx.tolist() == [1, 3]
    idx, _ = orc.exact_topk(q, K, 6, 4)
    assert idx.tolist() == [1, 3, 4, 0]


# ----------------------------------------------------------------- candidates
def _brute_candidates(prev, n, r, n_recent, n_sink):
    """Definition over ALL positions: j is a candidate iff some valid previous hit i has
    -r <= j - i <= r + 1, or j is among the newest n_recent rows or the first n_sink."""
    out = []
    for j in range(n):
        hit = j >= n - n_recent or j < n_sink
        for I_h in prev:
            for i in I_h:
                if 0 <= i < n and -r <= j - i <= r + 1:
                    hit = True
        if hit:
            out.append(j)
    return out


@pytest.mark.parametrize("seed", range(6))
def test_candidates_brute_force_all_positions(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(5, 120))
    r = int(rng.integers(0, 5))
    G = int(rng.integers(1, 5))
    k = int(rng.integers(1, min(n, 12) + 1))
    prev = [rng.choice(n + 3, size=k, replace=False) - 1 for _ in range(G)]   # includes -1 and >= n
    n_recent, n_sink = int(rng.integers(0, 4)), int(rng.integers(0, 3))
    got = orc.candidates(prev, n, r, n_recent, n_sink)
    assert got.tolist() == _brute_candidates(prev, n, r, n_recent, n_sink)


def test_candidates_offsets_at_r1_are_the_papers():
    with open(os.path.join(GOLDEN, "expansion_offsets.txt")) as f:
        printed = [int(l) for l in f if l.strip() and not l.startswith("#")]
    assert printed == [-1, 0, 1, 2]
    got = orc.candidates([np.array([50])], 100, 1, n_recent=0, n_sink=0)
    assert (got - 50).tolist() == printed
    # slash = +1 (not -1): with r = 0 a hit at i proposes exactly {i, i+1}
    assert orc.candidates([np.array([50])], 100, 0, 0, 0).tolist() == [50, 51]


def test_candidates_invariants():
    rng = np.random.default_rng(11)
    n, r, k, G = 500, 3, 20, 4
    prev = [rng.choice(n, size=k, replace=False) for _ in range(G)]
    C = orc.candidates(prev, n, r, 1, 4)
    assert np.all(np.diff(C) > 0) and C[0] >= 0 and C[-1] < n
    for I_h in prev:
        assert set(I_h.tolist()) <= set(C.tolist())
    assert k <= len(C) <= G * k * (2 * r + 2) + 1 + 4
    assert n - 1 in C and {0, 1, 2, 3} <= set(C.tolist())
    # clipping at both ends, and r >= n covers everything
    assert orc.candidates([np.array([0])], 10, 2, 0, 0).tolist() == [0, 1, 2, 3]
    assert orc.candidates([np.array([9])], 10, 2, 0, 0).tolist() == [7, 8, 9]
    assert orc.candidates([np.array([4])], 10, 10, 0, 0).tolist() == list(range(10))
    # the union over heads, not just the first head
    assert orc.candidates([np.array([2]), np.array([30])], 40, 0, 0, 0).tolist() == [2, 3, 30, 31]
    assert orc.candidates([np.array([-1, 77])], 40, 1, 0, 0).tolist() == []


# ----------------------------------------------------------------- score_topk / sparse_attn
def test_cover_invariant_lfps_topk_equals_exact_topk():
    q, K, _ = _rand(21, 200)
    C = np.arange(200)
    for k in (1, 17, 200):
        a, sa = orc.score_topk(q, K, C, k)
        b, sb = orc.exact_topk(q, K, 200, k)
        assert a.tolist() == b.tolist()
        np.testing.assert_array_equal(sa, sb)
        assert orc.overlap(a, b) == 1.0


def test_score_topk_brute_force_subsets():
    q, K, _ = _rand(22, 9, 4)
    C = np.array([0, 2, 3, 5, 8])
    s = {int(i): float(np.dot(q, K[i]) / 2.0) for i in C}
    best = max(itertools.combinations(C.tolist(), 3), key=lambda c: sum(s[i] for i in c))
    got, sc = orc.score_topk(q, K, C, 3)
    assert set(got.tolist()) == set(best)
    assert all(abs(sc[j] - s[int(got[j])]) < 1e-14 for j in range(3))
    # fewer candidates than k: return them all
    got, _ = orc.score_topk(q, K, C, 9)
    assert sorted(got.tolist()) == C.tolist()


def test_sparse_attn_k_equals_n_is_full_attention():
    q, K, V = _rand(23, 64)
    perm = np.random.default_rng(0).permutation(64)
    np.testing.assert_allclose(orc.sparse_attn(q, K, V, perm), orc.full_attn(q, K, V, 64), rtol=1e-12, atol=1e-14)


def test_sparse_attn_closed_forms():
    q, K, V = _rand(24, 30)
    np.testing.assert_allclose(orc.sparse_attn(q, K, V, np.array([7])), V[7], rtol=1e-15)
    # two rows: weights are the logistic function of the score difference
    s = orc.scores(q, K)
    w = 1.0 / (1.0 + math.exp(s[9] - s[4]))
    np.testing.assert_allclose(orc.sparse_attn(q, K, V, np.array([4, 9])), w * V[4] + (1 - w) * V[9], rtol=1e-12)
    # padding entries are ignored
    np.testing.assert_array_equal(orc.sparse_attn(q, K, V, np.array([4, -1, 9, -1])),
                                  orc.sparse_attn(q, K, V, np.array([4, 9])))
    # a convex combination: stays inside the selected rows' hull per channel
    I = np.array([1, 5, 6, 20])
    o = orc.sparse_attn(q, K, V, I)
    assert np.all(o <= V[I].max(axis=0) + 1e-12) and np.all(o >= V[I].min(axis=0) - 1e-12)


def test_overlap_ratio_definition():
    assert orc.overlap(np.array([1, 2, 3, 9]), np.array([2, 3, 4, 5])) == 0.5


# ----------------------------------------------------------------- whole step
def test_lfps_step_static_query_is_a_fixed_point_at_exact_topk():
    rng = np.random.default_rng(5)
    n, d, G, k = 400, 16, 4, 24
    K, V = rng.standard_normal((n, d)), rng.standard_normal((n, d))
    qg = rng.standard_normal((G, d))
    prev = [orc.exact_topk(qg[h], K, n, k)[0] for h in range(G)]
    for _ in range(3):
        res = orc.lfps_step(qg, K, V, prev, n, k, r=1, n_recent=0)
        for h in range(G):
            assert res["topk_idx"][h].tolist() == prev[h].tolist()
            np.testing.assert_allclose(res["out"][h], orc.sparse_attn(qg[h], K, V, prev[h]), rtol=1e-13)
        prev = res["topk_idx"]


def test_lfps_step_recall_monotone_in_radius_and_exact_when_covered():
    rng = np.random.default_rng(6)
    n, d, G, k = 600, 16, 4, 32
    K, V = rng.standard_normal((n, d)), rng.standard_normal((n, d))
    q0 = rng.standard_normal((G, d))
    q1 = q0 + 0.3 * rng.standard_normal((G, d))
    prev = [orc.exact_topk(q0[h], K, n, k)[0] for h in range(G)]
    last = -1.0
    for r in (0, 1, 2, 4, 8, n):
        res = orc.lfps_step(q1, K, V, prev, n, k, r=r)
        eta = np.mean([orc.overlap(res["topk_idx"][h], orc.exact_topk(q1[h], K, n, k)[0]) for h in range(G)])
        assert eta >= last
        last = eta
    assert last == 1.0
    np.testing.assert_allclose(res["out"][0], orc.sparse_attn(q1[0], K, V, orc.exact_topk(q1[0], K, n, k)[0]), rtol=1e-12)
    # per-head selection really uses that head's query
    assert res["topk_idx"][0].tolist() != res["topk_idx"][1].tolist()
