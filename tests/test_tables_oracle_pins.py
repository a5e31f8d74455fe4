"""Pins of the score-table oracle (Eq. 4, 7-10, 12 of the paper) against things other than itself:
a library kurtosis, closed forms, the sum invariant the paper states, geometric-series fixed points,
per-position brute force, and the printed offset set."""
import math
import os

import numpy as np
import pytest
import scipy.stats
import torch

from oracle import lfps_tables_oracle as tor

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _softmax_rows(x):
    return torch.softmax(torch.from_numpy(x), dim=-1).numpy()


# ----------------------------------------------------------------------------- Eq. 8
@pytest.mark.parametrize("seed,n", [(0, 5), (1, 64), (2, 1000)])
def test_kappa_is_library_kurtosis_over_n(seed, n):
    x = np.random.default_rng(seed).gamma(0.3, size=n)
    # Pearson kurtosis (biased) = n * sum d^4 / (sum d^2)^2
    want = scipy.stats.kurtosis(x, fisher=False, bias=True) / n
    assert tor.kappa(x) == pytest.approx(want, rel=1e-12)


@pytest.mark.parametrize("n,m,v", [(100, 1, 2.0), (4096, 7, 0.3), (50, 25, 1.0)])
def test_kappa_closed_form_for_equal_spikes(n, m, v):
    x = np.zeros(n)
    x[np.random.default_rng(n + m).choice(n, m, replace=False)] = v
    p = m / n
    want = ((1 - p) ** 3 + p ** 3) / (n * p * (1 - p))
    assert tor.kappa(x) == pytest.approx(want, rel=1e-10)
    # one spike in a long table: kappa -> 1, so tau -> a * mean
    if m == 1:
        assert tor.tau(x, 0.2) == pytest.approx(0.2 * v / n / want, rel=1e-12)


def test_kappa_undefined_for_a_flat_table_selects_nothing():
    x = np.full(30, 0.25)
    assert math.isnan(tor.kappa(x))
    assert tor.tau(x, 0.2) == float("inf")
    assert len(tor.initial_candidates(x, x, 30, 0.2)) == 0


def test_selection_is_invariant_under_scaling_of_the_tables():
    rng = np.random.default_rng(5)
    ver, sla = rng.gamma(0.2, size=300), rng.gamma(0.2, size=300)
    c0 = tor.head_candidates(ver, sla, 300, 0.3, 2)
    c1 = tor.head_candidates(7.5 * ver, 7.5 * sla, 300, 0.3, 2)
    np.testing.assert_array_equal(c0, c1)
    assert 0 < len(c0) < 300


def test_larger_a_never_adds_initial_candidates():
    rng = np.random.default_rng(6)
    ver, sla = rng.gamma(0.1, size=500), rng.gamma(0.1, size=500)
    prev = None
    for a in (0.05, 0.1, 0.2, 0.4, 0.8):
        c = set(tor.initial_candidates(ver, sla, 500, a).tolist())
        if prev is not None:
            assert c <= prev
        prev = c


# ----------------------------------------------------------------------------- Eq. 7 / Eq. 9 brute force
@pytest.mark.parametrize("seed", range(5))
def test_candidates_by_per_position_predicate(seed):
    rng = np.random.default_rng(100 + seed)
    n, r, a, n_sink = int(rng.integers(20, 200)), int(rng.integers(0, 4)), 0.25, int(rng.integers(0, 3))
    ver, sla = rng.gamma(0.15, size=n + 5), rng.gamma(0.15, size=n + 5)
    ver[:n_sink] = 0
    sla[:n_sink] = 0
    xv, xs = ver[n_sink:n], sla[n_sink:n]

    def t(x):
        d = x - x.mean()
        return a * x.mean() * (d ** 2).sum() ** 2 / (d ** 4).sum()

    tv, ts, mv, ms = t(xv), t(xs), xv.mean(), xs.mean()
    in_c0 = lambda i: n_sink <= i < n and (ver[i] > tv or sla[i] > ts)
    # gather form: j is kept iff it passes the mean test and some offset leads back to an initial candidate
    want = [j for j in range(n_sink, n)
            if (ver[j] > mv or sla[j] > ms) and any(in_c0(j - d) for d in range(-r, r + 2))]
    got = tor.head_candidates(ver, sla, n, a, r, n_sink)
    np.testing.assert_array_equal(got, np.array(want, dtype=np.int64))
    c0 = tor.initial_candidates(ver, sla, n, a, n_sink)
    np.testing.assert_array_equal(c0, np.array([i for i in range(n) if in_c0(i)], dtype=np.int64))


def test_expansion_offsets_at_r1_are_the_papers():
    offsets = [int(l) for l in open(os.path.join(GOLDEN, "expansion_offsets.txt")) if l.strip() and not l.startswith("#")]
    n, p = 60, 30
    ver = np.zeros(n)
    ver[p] = 500.0                     # the one initial candidate
    sla = np.full(n, 1.0)
    sla[p - 4:p + 6] += 1e-3           # the neighbourhood clears the mean filter through the slash table,
                                       # far below tau_sla = a * mean / kappa ~ 2.6
    c0 = tor.initial_candidates(ver, sla, n, 0.2)
    np.testing.assert_array_equal(c0, [p])
    c1 = tor.expand(c0, ver, sla, n, 1)
    assert sorted(int(j) - p for j in c1) == sorted(offsets)


def test_expansion_keeps_only_positions_above_a_mean():
    n, p = 40, 20
    ver = np.zeros(n)
    sla = np.zeros(n)
    ver[p] = 10.0
    ver[p + 1] = 1.0                   # above mean(ver) = 11/40
    sla[p - 1] = 0.5                   # above mean(sla)
    c1 = tor.expand(np.array([p]), ver, sla, n, 2)
    np.testing.assert_array_equal(c1, [p - 1, p, p + 1])


def test_group_candidates_add_recent_and_sink_rows():
    n = 50
    z = np.zeros(n)
    c = tor.group_candidates([(z, z), (z, z)], n, 0.2, 1, n_recent=2, n_sink=3)
    np.testing.assert_array_equal(c, [0, 1, 2, 48, 49])


def test_group_candidates_are_the_union_over_the_heads_written_out_by_hand():
    """Two heads of one KV group whose tables select disjoint positions (a vertical spike for the
    first head, a slash spike for the second): the group's set is the sorted union of both heads'
    sets, written out by hand; dropping either head loses its positions."""
    n = 64
    # head 0: one vertical spike at 10, the neighbourhood 8..13 above the mean through the slash table
    ver0, sla0 = np.zeros(n), np.full(n, 1.0)
    ver0[10] = 500.0
    sla0[8:14] += 1e-3
    # head 1: one slash spike at 40; only 40 and 41 clear a mean (through the vertical table)
    ver1, sla1 = np.full(n, 1.0), np.zeros(n)
    sla1[40] = 300.0
    ver1[40:42] += 1e-3
    # r = 2: offsets -2 .. 3 around each initial candidate, then the mean filter
    want0 = [8, 9, 10, 11, 12, 13]
    want1 = [40, 41]
    np.testing.assert_array_equal(tor.head_candidates(ver0, sla0, n, 0.2, 2), want0)
    np.testing.assert_array_equal(tor.head_candidates(ver1, sla1, n, 0.2, 2), want1)
    got = tor.group_candidates([(ver0, sla0), (ver1, sla1)], n, 0.2, 2, n_recent=1, n_sink=0)
    np.testing.assert_array_equal(got, want0 + want1 + [n - 1])
    # the order of the heads does not matter, and a single head gives only its own positions
    np.testing.assert_array_equal(tor.group_candidates([(ver1, sla1), (ver0, sla0)], n, 0.2, 2, 1, 0), got)
    np.testing.assert_array_equal(tor.group_candidates([(ver1, sla1)], n, 0.2, 2, 1, 0), want1 + [n - 1])


@pytest.mark.parametrize("seed", range(4))
def test_group_candidates_by_per_position_brute_force_over_all_heads(seed):
    """j is in the group's set iff it is a newest / sink row or SOME head keeps it (that head's own
    thresholds and means): a per-position predicate over every head, G = 2..4, overlapping sets."""
    rng = np.random.default_rng(700 + seed)
    G, n, r, a = int(rng.integers(2, 5)), int(rng.integers(40, 160)), int(rng.integers(0, 4)), 0.25
    n_sink, n_recent = int(rng.integers(0, 3)), int(rng.integers(0, 3))
    tables = []
    for _ in range(G):
        ver, sla = rng.gamma(0.12, size=n), rng.gamma(0.12, size=n)
        ver[:n_sink] = 0
        sla[:n_sink] = 0
        tables.append((ver, sla))

    def head_keeps(ver, sla, j):
        xv, xs = ver[n_sink:n], sla[n_sink:n]

        def t(x):
            d = x - x.mean()
            return a * x.mean() * (d ** 2).sum() ** 2 / (d ** 4).sum()

        tv, ts = t(xv), t(xs)
        in_c0 = lambda i: n_sink <= i < n and (ver[i] > tv or sla[i] > ts)
        return n_sink <= j < n and (ver[j] > xv.mean() or sla[j] > xs.mean()) and \
            any(in_c0(j - d) for d in range(-r, r + 2))

    want = [j for j in range(n)
            if j < n_sink or j >= n - n_recent or any(head_keeps(v, s, j) for (v, s) in tables)]
    got = tor.group_candidates(tables, n, a, r, n_recent, n_sink)
    np.testing.assert_array_equal(got, np.array(want, dtype=np.int64))
    per_head = [set(tor.head_candidates(v, s, n, a, r, n_sink).tolist()) for (v, s) in tables]
    assert any(per_head[h] - per_head[0] for h in range(1, G)), "the heads must differ for the pin to bite"


# ----------------------------------------------------------------------------- Eq. 4 and Eq. 12
def test_init_tables_sum_and_diagonal_alignment():
    rng = np.random.default_rng(9)
    n, s, gamma = 40, 5, 0.9
    logits = rng.standard_normal((s, n))
    for j in range(1, s + 1):          # query n-j sees positions <= n-j
        logits[j - 1, n - j + 1:] = -np.inf
    w = _softmax_rows(logits)
    ver, sla = tor.init_tables(w, gamma)
    assert ver.sum() == pytest.approx(1 / (2 * (1 - gamma)), rel=1e-12)      # Eq. 12 / App. B.2
    assert sla.sum() == pytest.approx(1 / (2 * (1 - gamma)), rel=1e-12)
    # one query (s = 1): both tables are its weights over 2 (1 - gamma)
    v1, s1 = tor.init_tables(w[:1], gamma)
    np.testing.assert_allclose(v1, w[0] / (2 * (1 - gamma)), rtol=1e-13)
    np.testing.assert_allclose(s1, v1, rtol=0, atol=0)
    # a query j steps back that looked only at position p predicts p + j - 1 on the slash table
    onehot = np.zeros((3, n))
    onehot[2, 11] = 1.0                # j = 3
    v3, s3 = tor.init_tables(onehot, gamma)
    assert np.argmax(v3) == 11 and np.argmax(s3) == 13
    assert v3[11] == pytest.approx(1 / (6 * (1 - gamma))) and s3[13] == pytest.approx(v3[11])


@pytest.mark.parametrize("gamma", [0.0, 0.5, 0.95])
def test_table_sums_follow_the_stated_recurrence(gamma):
    rng = np.random.default_rng(11)
    n = 64
    ver, sla = rng.random(n), rng.random(n)
    S_v, S_s = ver.sum(), sla.sum()
    for step in range(400):
        k = int(rng.integers(1, 20))
        sel = rng.choice(n, k, replace=False)
        ver, sla = tor.update_tables(ver, sla, n, sel, rng.standard_normal(k) * 3, gamma)
        n += 1
        S_v, S_s = gamma * S_v + 0.5, gamma * S_s + 0.5
        assert ver.sum() == pytest.approx(S_v, rel=1e-10, abs=1e-12)
        assert sla.sum() == pytest.approx(S_s, rel=1e-10, abs=1e-12)
    # Eq. 12: both sums settle at 0.5 / (1 - gamma)
    assert ver.sum() == pytest.approx(0.5 / (1 - gamma), rel=1e-6)
    assert sla.sum() == pytest.approx(0.5 / (1 - gamma), rel=1e-6)


def test_unselected_positions_only_decay_and_slash_moves_by_one():
    rng = np.random.default_rng(12)
    n, gamma = 30, 0.8
    ver, sla = rng.random(n), rng.random(n)
    sel = np.array([4, 17, -1])
    nv, ns = tor.update_tables(ver, sla, n, sel, np.array([0.3, -1.0, 9.9]), gamma)
    assert len(nv) == len(ns) == n + 1
    others = [i for i in range(n) if i not in (4, 17)]
    np.testing.assert_allclose(nv[others], gamma * ver[others], rtol=1e-15)
    np.testing.assert_allclose(ns[[i for i in others if i >= 1]], gamma * sla[[i - 1 for i in others if i >= 1]], rtol=1e-15)
    assert nv[n] == 0.0 and ns[n] == pytest.approx(gamma * sla[n - 1]) and ns[0] == 0.0
    # the two selected positions receive softmax weight minus 1/(2*2); the padding entry is ignored
    w = _softmax_rows(np.array([[0.3, -1.0]]))[0]
    assert nv[4] - gamma * ver[4] == pytest.approx(w[0] - 0.25)
    assert ns[17] - gamma * sla[16] == pytest.approx(w[1] - 0.25)


def test_constant_selection_reaches_the_geometric_series_limit():
    gamma, n0 = 0.7, 25
    sel = np.array([3, 9, 10])
    sc = np.array([1.0, 2.0, 0.5])
    w = _softmax_rows(sc[None])[0]
    ver, sla = np.zeros(n0), np.zeros(n0)
    n = n0
    for _ in range(120):
        ver, sla = tor.update_tables(ver, sla, n, sel, sc, gamma)
        n += 1
    for p, wp in zip(sel, w):
        assert ver[p] == pytest.approx((wp - 1 / 6) / (1 - gamma), rel=1e-9)
    # slash: what position p received m steps ago now sits at p + m, decayed m times
    d = {int(p): wp - 1 / 6 for p, wp in zip(sel, w)}
    for i in (3, 4, 9, 10, 11, 12, 40):
        want = sum(gamma ** m * d.get(i - m, 0.0) for m in range(0, 120))
        assert sla[i] == pytest.approx(want, rel=1e-9, abs=1e-15)


def test_single_hit_travels_down_the_slash_diagonal():
    gamma, n, p = 0.9, 20, 5
    ver, sla = tor.update_tables(np.zeros(n), np.zeros(n), n, np.array([p]), np.array([0.0]), gamma)
    n += 1
    for m in range(1, 8):
        ver, sla = tor.update_tables(ver, sla, n, np.array([], dtype=np.int64), np.array([]), gamma)
        n += 1
        assert ver[p] == pytest.approx(0.5 * gamma ** m) and np.count_nonzero(ver) == 1
        assert sla[p + m] == pytest.approx(0.5 * gamma ** m) and np.count_nonzero(sla) == 1


def test_sink_positions_stay_outside_the_tables():
    rng = np.random.default_rng(13)
    n, gamma, n_sink = 30, 0.9, 4
    ver, sla = rng.random(n), rng.random(n)
    ver[:n_sink] = 0
    sla[:n_sink] = 0
    sel = np.array([0, 2, 10, 20])
    sc = np.array([50.0, 40.0, 1.0, 2.0])          # the sinks would swallow the softmax
    nv, ns = tor.update_tables(ver, sla, n, sel, sc, gamma, n_sink)
    assert not nv[:n_sink].any() and not ns[:n_sink].any()
    w = _softmax_rows(np.array([[1.0, 2.0]]))[0]
    assert nv[10] - gamma * ver[10] == pytest.approx(w[0] - 0.25)
    assert nv.sum() == pytest.approx(gamma * ver.sum() + 0.5)
    c0 = tor.initial_candidates(np.r_[np.full(n_sink, 1e9), ver[n_sink:]], sla, n, 0.2, n_sink)
    assert (c0 >= n_sink).all()


# ----------------------------------------------------------------------------- one whole step
def test_table_step_selects_the_best_candidates_and_attends_over_them():
    rng = np.random.default_rng(14)
    n, d, G, k = 120, 16, 2, 8
    K, V = rng.standard_normal((n + 1, d)), rng.standard_normal((n + 1, d))
    q = rng.standard_normal((G, d))
    tables = []
    for h in range(G):
        ver, sla = rng.gamma(0.1, size=n), rng.gamma(0.1, size=n)
        tables.append((ver, sla))
    res = tor.table_step(q, K, V, tables, n, k, 1, 0.2, 0.95, n_recent=1, n_sink=0)
    C = res["cand"]
    assert n - 1 in C and len(C) == len(set(C.tolist())) and list(C) == sorted(C)
    for h in range(G):
        s_all = (K[:n] @ q[h]) / math.sqrt(d)
        want = C[np.argsort(-s_all[C], kind="stable")[:k]]
        assert set(res["topk_idx"][h].tolist()) == set(want.tolist())
        I = torch.from_numpy(res["topk_idx"][h])
        ref = torch.softmax(torch.from_numpy(s_all)[I], 0) @ torch.from_numpy(V)[I]
        np.testing.assert_allclose(res["out"][h], ref.numpy(), rtol=1e-12, atol=1e-14)
        nv, ns = res["tables"][h]
        assert len(nv) == n + 1
        assert nv.sum() == pytest.approx(0.95 * tables[h][0].sum() + 0.5)


# ----------------------------------------------------------------------------- Eq. 5-6 (head sparsity), priors
def test_priors_are_plain_means_and_logit_variance():
    rng = np.random.default_rng(20)
    n, d, n_sink = 300, 16, 4
    K, V, q = rng.standard_normal((n + 3, d)), rng.standard_normal((n + 3, d)), rng.standard_normal(d) * 1.7
    kbar, vbar, s2 = tor.priors(q, K, V, n, n_sink)
    tK, tV = torch.from_numpy(K[n_sink:n]), torch.from_numpy(V[n_sink:n])
    np.testing.assert_allclose(kbar, tK.mean(0).numpy(), rtol=1e-13)
    np.testing.assert_allclose(vbar, tV.mean(0).numpy(), rtol=1e-13)
    logits = (tK @ torch.from_numpy(q)) / math.sqrt(d)
    assert s2 == pytest.approx(float(torch.var(logits, unbiased=False)) / float(q @ q), rel=1e-12)


def test_global_term_is_exact_for_identical_keys_and_lognormal_in_general():
    rng = np.random.default_rng(21)
    d, n, n_sink = 16, 5000, 2
    q = rng.standard_normal(d)
    # (a) every offloaded key equal: sigma = 0 and n * exp(q.kbar/sqrt(d)) is the exact sum of the weights
    K = np.tile(rng.standard_normal(d), (n, 1))
    K[:n_sink] = rng.standard_normal((n_sink, d)) * 3
    kbar, _, s2 = tor.priors(q, K, K, n, n_sink)
    assert s2 == pytest.approx(0.0, abs=1e-25)
    w = np.exp((K[:n] @ q) / math.sqrt(d))
    rho = tor.sparsity_ratio(q, K, n, kbar, s2, n_sink, n_local=0)
    assert rho == pytest.approx(w[:n_sink].sum() / (w[:n_sink].sum() + n * w[n_sink]), rel=1e-12)
    # (b) Gaussian logits: geometric mean * exp(sigma^2/2) estimates the arithmetic mean of the weights (App. B.1)
    K = rng.standard_normal((n, d))
    kbar, _, s2 = tor.priors(q, K, K, n, n_sink)
    est = n * math.exp(float(kbar @ q) / math.sqrt(d) + float(q @ q) * s2 / 2)
    true = np.exp((K[n_sink:n] @ q) / math.sqrt(d)).sum()
    assert est == pytest.approx(true, rel=0.1)
    # the variance term matters: without it the estimate is the geometric mean, well below the truth
    assert n * math.exp(float(kbar @ q) / math.sqrt(d)) < 0.8 * true


def test_sparsity_ratio_definition_monotone_and_limits():
    rng = np.random.default_rng(22)
    d, n, n_sink = 8, 200, 1
    K = rng.standard_normal((n, d))
    q = rng.standard_normal(d)
    kbar, _, s2 = tor.priors(q, K, K, n, n_sink)
    prev = 0.0
    for scale in (0.0, 1.0, 3.0, 10.0, 40.0):          # a sink key ever more aligned with the query
        K2 = K.copy()
        K2[0] = scale * q / np.linalg.norm(q)
        rho = tor.sparsity_ratio(q, K2, n, kbar, s2, n_sink)
        assert 0.0 < rho <= 1.0 and rho >= prev
        prev = rho
    assert prev > 0.999
    # the local term is the plain sum over the newest six rows
    w = np.exp((K @ q) / math.sqrt(d))
    r6 = tor.sparsity_ratio(q, K, n, kbar, s2, n_sink, n_local=6)
    r0 = tor.sparsity_ratio(q, K, n, kbar, s2, n_sink, n_local=0)
    assert 1 / r6 - 1 / r0 == pytest.approx(w[n - 6:].sum() / w[0], rel=1e-10)


def test_gated_step_bypasses_sparse_heads_and_leaves_their_tables():
    rng = np.random.default_rng(23)
    n, d, G, k, n_sink = 150, 16, 3, 8, 2
    K, V = rng.standard_normal((n + 1, d)), rng.standard_normal((n + 1, d))
    q = rng.standard_normal((G, d))
    u = q[1] / np.linalg.norm(q[1])
    for h in (0, 2):
        q[h] -= (q[h] @ u) * u                          # the other heads do not see that sink
    K[0] = 30.0 * u                                     # head 1 looks at the sink only
    tables = [(rng.gamma(0.1, size=n), rng.gamma(0.1, size=n)) for _ in range(G)]
    for t in tables:
        t[0][:n_sink] = 0
        t[1][:n_sink] = 0
    kbar, vbar, _ = tor.priors(q[0], K, V, n, n_sink)
    s2 = [tor.priors(q[h], K, V, n, n_sink)[2] for h in range(G)]
    res = tor.gated_table_step(q, K, V, tables, n, k, 1, 0.2, 0.9, kbar, vbar, s2, 0.85, n_recent=1, n_sink=n_sink)
    assert list(res["gate"]) == [False, True, False] and res["rho"][1] > 0.85
    np.testing.assert_array_equal(res["out"][1], vbar)
    assert len(res["topk_idx"][1]) == 0
    np.testing.assert_array_equal(res["tables"][1][0], np.r_[tables[1][0], 0.0])
    np.testing.assert_array_equal(res["tables"][1][1], np.r_[tables[1][1], 0.0])
    # the others behave as in table_step over the candidates of the live heads only
    ref = tor.table_step(q[[0, 2]], K, V, [tables[0], tables[2]], n, k, 1, 0.2, 0.9, n_recent=1, n_sink=n_sink)
    np.testing.assert_array_equal(res["cand"], ref["cand"])
    # ... which is the union of the live heads' own sets (each pinned by brute force above) with the newest row
    # and the sinks; the bypassed head's positions are not proposed
    own = [set(tor.head_candidates(t[0], t[1], n, 0.2, 1, n_sink).tolist()) for t in tables]
    want = own[0] | own[2] | {n - 1} | set(range(n_sink))
    assert sorted(want) == res["cand"].tolist()
    assert own[1] - want, "head 1 must have positions of its own for this to test anything"
    np.testing.assert_array_equal(res["topk_idx"][2], ref["topk_idx"][1])
    np.testing.assert_allclose(res["out"][0], ref["out"][0], rtol=1e-14)
