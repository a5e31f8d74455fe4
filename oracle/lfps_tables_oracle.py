"""CPU fp64 oracle for LFPS with score tables (the paper's full candidate rule).  TEST INFRASTRUCTURE ONLY.

Plain, slow, dense, written from the paper ("Learn from the Past: Fast Sparse Indexing for LLM
Decoding"); shares no code with the HIP library and is imported only by tests/, the smoke check and
the bench's cpu_baseline leg.  Every table is a dense float64 vector over positions and every
statistic is recomputed from scratch each step, exactly as the equations are written.

What each function follows:

* init_tables        Sec. 4.2 "Prefilling", Eq. 4: vertical and slash tables from the attention weights
                     of the last s queries; normalisation 1/(2 s (1 - gamma)) (App. B.2, Eq. 12).
* kappa, tau         Eq. 8: kappa(x) = sum (x - mean)^4 / (sum (x - mean)^2)^2, tau(x) = a mean(x) / kappa(x).
* initial_candidates Eq. 7: positions whose vertical score exceeds tau_ver or whose slash score exceeds tau_sla.
* expand             Eq. 9: every offset -r ... r+1 around an initial candidate (r = 1: the printed
                     {-1, 0, 1, 2}), kept only where the vertical or the slash score exceeds its table mean.
* update_tables      Eq. 10: decay by gamma, slash history moved from i-1 to i, the step's normalised
                     attention weights over the selected set added minus 1/(2|C_2|); positions outside the
                     selected set only decay (their w is defined as 1/(2|C_2|)).
* table_step         Alg. 1 lines 5-9 and Eq. 1 for the query heads of one KV group.
* priors             Sec. 4.2 "Prefilling", last paragraph: mean key, mean value, sigma_hat^2.
* sparsity_ratio     Eq. 5 and Eq. 6 (App. B.1: the global term is the log-normal mean of the weights).
* gated_table_step   Alg. 1 lines 1-9: the bypass of sparse heads in front of table_step.

Readings where the paper is silent (the same ones the library takes):
  - w in Eq. 10 is the softmax over the selected set (it must sum to 1 for Eq. 12 to hold).
  - The tables grow by one position per decode step: the new position starts at 0 in the vertical table
    and receives gamma * (slash score of the previous last position) in the slash table.
  - Sink positions (< n_sink) are outside the tables, as in the paper (they stay on the accelerator):
    always candidates, never counted in the statistics, never updated; w is normalised over the
    selected non-sink positions.  The newest n_recent rows are always candidates too.
  - A table whose entries are all equal has no pattern: kappa is undefined and no position passes Eq. 7.
  - With GQA the candidate set of a KV group is the union of its heads' sets; Top-k stays per head.
  - Eq. 5: the sink term sums over the n_sink sink rows; the local term over the newest n_local = 6 rows
    (Eq. 5 writes six terms, the appendix says "e.g. the last five"); sigma^2 is the variance over the
    offloaded rows of the logits of the last prefill query, so |q|^2 sigma_hat^2 is the logit variance the
    current query would see; kbar, vbar are means over the offloaded rows.  A bypassed head keeps its
    tables unchanged (steps 2-4 of Sec. 4.2 are skipped, Eq. 10 among them) and outputs vbar.

Pins (tests/test_tables_oracle_pins.py): scipy's kurtosis, closed forms of kappa for equal spikes,
scale invariance of tau's selection, Eq. 12 (table sums follow S' = gamma S + 1/2 and start at
1/(2(1 - gamma))), geometric-series fixed points of Eq. 10 for a constant selection, the diagonal
motion of slash history, brute force of Eq. 7/9 by per-position predicates, the printed offsets, the union over
the heads of a KV group written out by hand and by a per-position predicate over every head.
"""
from __future__ import annotations

import math
from typing import List, Sequence

import numpy as np


# ----------------------------------------------------------------------------- Eq. 4
def init_tables(w_hist: np.ndarray, gamma: float, n_sink: int = 0):
    """w_hist[j-1, i] = attention weight that query n-j (j = 1..s, the j-th most recent) put on
    position i < n.  Returns (phi_ver, phi_sla), float64 vectors of length n.
    Positions < n_sink are left at 0 (sinks are not part of the tables)."""
    w_hist = np.asarray(w_hist, dtype=np.float64)
    s, n = w_hist.shape
    norm = 1.0 / (2.0 * s * (1.0 - gamma))
    ver = np.zeros(n)
    sla = np.zeros(n)
    for i in range(n):
        for j in range(1, s + 1):
            ver[i] += w_hist[j - 1, i]
            src = i - j + 1
            if src >= 0:
                sla[i] += w_hist[j - 1, src]
    ver *= norm
    sla *= norm
    ver[:n_sink] = 0.0
    sla[:n_sink] = 0.0
    return ver, sla


# ----------------------------------------------------------------------------- Eq. 8
def kappa(x: np.ndarray) -> float:
    """sum (x_i - mean)^4 / (sum (x_i - mean)^2)^2; nan if all entries are equal (or x is empty)."""
    x = np.asarray(x, dtype=np.float64)
    if len(x) == 0:
        return float("nan")
    d = x - np.mean(x)
    s2 = float(np.sum(d ** 2))
    if s2 == 0.0:
        return float("nan")
    return float(np.sum(d ** 4)) / (s2 * s2)


def tau(x: np.ndarray, a: float) -> float:
    """a * mean(x) / kappa(x); +inf when kappa is undefined (no position can exceed it)."""
    k = kappa(x)
    if math.isnan(k):
        return float("inf")
    return a * float(np.mean(x)) / k


# ----------------------------------------------------------------------------- Eq. 7, Eq. 9
def initial_candidates(ver: np.ndarray, sla: np.ndarray, n: int, a: float, n_sink: int = 0) -> np.ndarray:
    """C_0: positions n_sink <= i < n with ver(i) > tau_ver or sla(i) > tau_sla (statistics over the
    same positions)."""
    xv, xs = np.asarray(ver[n_sink:n], dtype=np.float64), np.asarray(sla[n_sink:n], dtype=np.float64)
    tv, ts = tau(xv, a), tau(xs, a)
    keep = (xv > tv) | (xs > ts)
    return np.nonzero(keep)[0].astype(np.int64) + n_sink


def expand(C0: np.ndarray, ver: np.ndarray, sla: np.ndarray, n: int, r: int, n_sink: int = 0) -> np.ndarray:
    """C_1: j = i + delta for i in C_0, delta in {-r, ..., r+1}, n_sink <= j < n, kept when ver(j)
    exceeds the mean of ver or sla(j) exceeds the mean of sla (means over positions n_sink..n-1)."""
    xv, xs = np.asarray(ver[n_sink:n], dtype=np.float64), np.asarray(sla[n_sink:n], dtype=np.float64)
    if len(xv) == 0:
        return np.zeros(0, dtype=np.int64)
    mv, ms = float(np.mean(xv)), float(np.mean(xs))
    out = set()
    for i in np.asarray(C0, dtype=np.int64).tolist():
        for delta in range(-r, r + 2):
            j = i + delta
            if n_sink <= j < n and (ver[j] > mv or sla[j] > ms):
                out.add(j)
    return np.array(sorted(out), dtype=np.int64)


def head_candidates(ver, sla, n, a, r, n_sink=0) -> np.ndarray:
    """Eq. 7 then Eq. 9 for one head."""
    return expand(initial_candidates(ver, sla, n, a, n_sink), ver, sla, n, r, n_sink)


def group_candidates(tables: Sequence, n: int, a: float, r: int, n_recent: int = 0, n_sink: int = 0) -> np.ndarray:
    """Union over the heads of a KV group, plus the always-present newest and sink rows; ascending."""
    S = set()
    for (ver, sla) in tables:
        S.update(head_candidates(ver, sla, n, a, r, n_sink).tolist())
    S.update(range(max(0, n - n_recent), n))
    S.update(range(0, min(n_sink, n)))
    return np.array(sorted(S), dtype=np.int64)


# ----------------------------------------------------------------------------- Eq. 10
def update_tables(ver: np.ndarray, sla: np.ndarray, n: int, sel: np.ndarray, sel_scores: np.ndarray,
                  gamma: float, n_sink: int = 0):
    """Tables after a step that saw n positions and selected `sel` with scaled scores `sel_scores`
    (q.K/sqrt(d)); negative entries of sel are padding.  Returns vectors of length n + 1."""
    ver = np.asarray(ver, dtype=np.float64)
    sla = np.asarray(sla, dtype=np.float64)
    sel = np.asarray(sel, dtype=np.int64)
    sc = np.asarray(sel_scores, dtype=np.float64)
    ok = (sel >= n_sink) & (sel < n)
    sel, sc = sel[ok], sc[ok]
    new_ver = np.zeros(n + 1)
    new_sla = np.zeros(n + 1)
    for i in range(n + 1):
        new_ver[i] = gamma * (ver[i] if i < n else 0.0)
        new_sla[i] = gamma * (sla[i - 1] if 1 <= i <= n else 0.0)
    new_ver[:n_sink] = 0.0
    new_sla[:n_sink] = 0.0
    if len(sel):
        e = np.exp(sc - np.max(sc))
        w = e / np.sum(e)
        half = 1.0 / (2.0 * len(sel))
        for i, wi in zip(sel.tolist(), w.tolist()):
            new_ver[i] += wi - half
            new_sla[i] += wi - half
    return new_ver, new_sla


# ----------------------------------------------------------------------------- Alg. 1 lines 5-9 + Eq. 1
def _scores(q, K, rows):
    q = np.asarray(q, dtype=np.float64)
    Kr = np.asarray(K[np.asarray(rows, dtype=np.int64)], dtype=np.float64)
    return (Kr @ q) / math.sqrt(q.shape[-1])


def _k_best(s, ids, k):
    order = np.lexsort((ids, -s))[:k]            # score descending, then position ascending
    return ids[order], s[order]


def table_step(q_group: np.ndarray, K: np.ndarray, V: np.ndarray, tables: List, n: int, k: int, r: int,
               a: float, gamma: float, n_recent: int = 0, n_sink: int = 0):
    """One decode step with score tables for the G query heads that share a KV head.

    tables: list of (ver, sla) per head, each of length >= n.  Returns dict(cand, topk_idx, topk_score,
    out, tables) where tables are the updated (length n + 1) vectors."""
    C = group_candidates(tables, n, a, r, n_recent, n_sink)
    idx, sc, out, new_tables = [], [], [], []
    for h in range(len(q_group)):
        s = _scores(q_group[h], K, C) if len(C) else np.zeros(0)
        I_h, s_h = _k_best(s, C, min(k, len(C)))
        idx.append(I_h)
        sc.append(s_h)
        if len(I_h):
            e = np.exp(s_h - np.max(s_h))
            out.append((e / np.sum(e)) @ np.asarray(V[I_h], dtype=np.float64))
        else:
            out.append(np.zeros(np.asarray(V).shape[-1]))
        new_tables.append(update_tables(tables[h][0], tables[h][1], n, I_h, s_h, gamma, n_sink))
    return dict(cand=C, topk_idx=idx, topk_score=sc, out=np.array(out), tables=new_tables)


# ----------------------------------------------------------------------------- Eq. 5-6, prefill priors
def priors(q_last: np.ndarray, K: np.ndarray, V: np.ndarray, n: int, n_sink: int = 0):
    """Sec. 4.2 "Prefilling", last paragraph: mean key and mean value over the offloaded rows
    [n_sink, n), and sigma_hat^2 = (variance over those rows of the logits q_last.K_i/sqrt(d)) / |q_last|^2.
    Returns (kbar [d], vbar [d], sigma2_hat)."""
    Kr = np.asarray(K[n_sink:n], dtype=np.float64)
    Vr = np.asarray(V[n_sink:n], dtype=np.float64)
    q = np.asarray(q_last, dtype=np.float64)
    logits = (Kr @ q) / math.sqrt(q.shape[-1])
    return Kr.mean(axis=0), Vr.mean(axis=0), float(np.var(logits)) / float(q @ q)


def sparsity_ratio(q: np.ndarray, K: np.ndarray, n: int, kbar: np.ndarray, sigma2_hat: float, n_sink: int,
                   n_local: int = 6) -> float:
    """Eq. 5 and Eq. 6: rho = w_sink / (w_sink + w_global + w_local) with
    w_sink   = sum over the sink rows of exp(q.K_i/sqrt(d)),
    w_global = n * exp(q.kbar/sqrt(d) + |q|^2 sigma2_hat / 2)   (log-normal mean of the weights, App. B.1),
    w_local  = sum over the newest n_local rows of exp(q.K_i/sqrt(d))."""
    q = np.asarray(q, dtype=np.float64)
    sd = math.sqrt(q.shape[-1])
    Kd = np.asarray(K, dtype=np.float64)
    w_sink = float(np.sum(np.exp((Kd[: min(n_sink, n)] @ q) / sd)))
    w_global = n * math.exp(float(np.asarray(kbar, dtype=np.float64) @ q) / sd + float(q @ q) * sigma2_hat / 2.0)
    lo = max(0, n - n_local)
    w_local = float(np.sum(np.exp((Kd[lo:n] @ q) / sd)))
    return w_sink / (w_sink + w_global + w_local)


def gated_table_step(q_group, K, V, tables, n, k, r, a, gamma, kbar, vbar, sigma2_hat, eps, n_recent=0, n_sink=0,
                     n_local=6):
    """Alg. 1 in full for one KV group: heads whose sparsity ratio exceeds eps return vbar, select nothing
    and leave their tables as they are (steps 2-4 skipped); the others run table_step's lines, with the
    candidate set being the union over the heads that are not bypassed."""
    G = len(q_group)
    rho = [sparsity_ratio(q_group[h], K, n, kbar, sigma2_hat[h], n_sink, n_local) for h in range(G)]
    gate = [rh > eps for rh in rho]
    live = [h for h in range(G) if not gate[h]]
    C = group_candidates([tables[h] for h in live], n, a, r, n_recent, n_sink)
    idx, sc, out, new_tables = [], [], [], []
    for h in range(G):
        if gate[h]:
            idx.append(np.zeros(0, dtype=np.int64))
            sc.append(np.zeros(0))
            out.append(np.asarray(vbar, dtype=np.float64))
            # unchanged; the position the next step appends has no history yet
            new_tables.append((np.r_[np.asarray(tables[h][0][:n], dtype=np.float64), 0.0],
                               np.r_[np.asarray(tables[h][1][:n], dtype=np.float64), 0.0]))
            continue
        s = _scores(q_group[h], K, C) if len(C) else np.zeros(0)
        I_h, s_h = _k_best(s, C, min(k, len(C)))
        idx.append(I_h)
        sc.append(s_h)
        if len(I_h):
            e = np.exp(s_h - np.max(s_h))
            out.append((e / np.sum(e)) @ np.asarray(V[I_h], dtype=np.float64))
        else:
            out.append(np.zeros(np.asarray(V).shape[-1]))
        new_tables.append(update_tables(tables[h][0], tables[h][1], n, I_h, s_h, gamma, n_sink))
    return dict(rho=np.array(rho), gate=np.array(gate), cand=C, topk_idx=idx, topk_score=sc, out=np.array(out),
                tables=new_tables)
