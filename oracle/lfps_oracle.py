"""CPU fp64 oracle for the LFPS decode-step hot path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, written from the paper; it shares no code with the HIP library and is
imported only by tests/, the smoke check and the bench's cpu_baseline leg.  All
floating point is float64 on the *stored* K/V values (bf16 widened exactly) and on
the fp32 query the device path also receives.

What each function follows in the paper ("Learn from the Past: Fast Sparse Indexing
for LLM Decoding"):

* full_attn      Sec. 1 three-step decomposition with idx = every position; Eq. 1 with I = all.
* scores         Sec. 1 Step 1 (w = q K^T), scaled by 1/sqrt(d) as in Eq. 1.
* exact_topk     Sec. 1 Step 2 (idx = TopK(w)); the paper's "exact Top-k" baseline (Sec. 5).
* candidates     Alg. 1 lines 6-7 (Eq. 7 and Eq. 9) in the memoryless form: the initial set is
                 the previous step's Top-k (vertical pattern: same position) together with the
                 same set shifted by one (slash pattern; Eq. 10 moves slash history from i-1
                 to i each step), and each of the two is widened by the expansion radius r.
                 At r = 1 the offsets are the paper's printed {-1, 0, 1, 2} (Sec. 4.2 stage 3,
                 Fig. 4 caption).  No score-table threshold/mean filter (there are no tables).
* score_topk     Alg. 1 line 8: exact dot products over the candidate set only, keep the k best.
* sparse_attn    Eq. 1.
* overlap        Eq. 2.
* lfps_step      Alg. 1 lines 6-8 and 10 followed by Eq. 1, for the query heads of one KV group
                 (candidates are the union over the group's heads; Top-k is per head).

Pins (tests/test_oracle_pins.py): library softmax attention, closed forms (equal keys ->
mean of V; one dominant key -> its V row; k = 1), brute-force sort, per-position brute
force of the candidate predicate, the printed offset set at r = 1, cover => exact Top-k,
k = n => full attention, static-query fixed point.  The heuristic's *values* have no
worked example in the paper (its Fig. 4 did not survive), so beyond the offset set the
pins are structural.
"""
from __future__ import annotations

import math
from typing import Sequence

import numpy as np


def scores(q: np.ndarray, K: np.ndarray, rows=None) -> np.ndarray:
    """s_i = q . K_i / sqrt(d) in float64 for the given rows (default: all rows of K)."""
    q = np.asarray(q, dtype=np.float64)
    Kr = np.asarray(K if rows is None else K[np.asarray(rows, dtype=np.int64)], dtype=np.float64)
    return (Kr @ q) / math.sqrt(q.shape[-1])


def _softmax(s: np.ndarray) -> np.ndarray:
    e = np.exp(s - np.max(s))
    return e / np.sum(e)


def full_attn(q: np.ndarray, K: np.ndarray, V: np.ndarray, n: int) -> np.ndarray:
    """Softmax(q K^T / sqrt(d)) V over rows [0, n)."""
    p = _softmax(scores(q, K[:n]))
    return p @ np.asarray(V[:n], dtype=np.float64)


def _k_best(s: np.ndarray, ids: np.ndarray, k: int):
    """The k entries of largest score; ties go to the lower index.  Returns (ids, scores)
    in that order (best first)."""
    order = np.lexsort((ids, -s))       # primary: score descending, secondary: index ascending
    order = order[:k]
    return ids[order], s[order]


def exact_topk(q: np.ndarray, K: np.ndarray, n: int, k: int):
    """Indices (and scores) of the k largest q.K_i/sqrt(d), i < n."""
    s = scores(q, K[:n])
    return _k_best(s, np.arange(n, dtype=np.int64), min(k, n))


def candidates(prev_topk: Sequence[np.ndarray], n: int, r: int, n_recent: int = 1,
               n_sink: int = 0) -> np.ndarray:
    """Candidate positions of one KV group at a step that sees n rows.

    prev_topk: the previous step's Top-k index array of every query head of the group
    (entries < 0 or >= n are ignored).  Result: sorted unique int64 positions in [0, n).
    """
    S = set()
    for I_h in prev_topk:
        for i in np.asarray(I_h, dtype=np.int64).tolist():
            if i < 0 or i >= n:
                continue
            for base in (i, i + 1):                 # vertical hit, slash prediction
                for d in range(-r, r + 1):          # positional expansion
                    j = base + d
                    if 0 <= j < n:
                        S.add(j)
    for j in range(max(0, n - n_recent), n):        # newest rows were never scored before
        S.add(j)
    for j in range(0, min(n_sink, n)):
        S.add(j)
    return np.array(sorted(S), dtype=np.int64)


def score_topk(q_h: np.ndarray, K: np.ndarray, C: np.ndarray, k: int):
    """Exact dot products over the candidates only; the k best (fewer if |C| < k)."""
    C = np.asarray(C, dtype=np.int64)
    s = scores(q_h, K, C)
    return _k_best(s, C, min(k, len(C)))


def sparse_attn(q_h: np.ndarray, K: np.ndarray, V: np.ndarray, I_h: np.ndarray) -> np.ndarray:
    """O(I) = Softmax(q K_I^T / sqrt(d)) V_I; negative entries of I are padding.
    An empty index set (nothing to attend to) gives the zero vector."""
    I_h = np.asarray(I_h, dtype=np.int64)
    I_h = I_h[I_h >= 0]
    if len(I_h) == 0:
        return np.zeros(np.asarray(V).shape[-1], dtype=np.float64)
    p = _softmax(scores(q_h, K, I_h))
    return p @ np.asarray(V[I_h], dtype=np.float64)


def overlap(C: np.ndarray, I: np.ndarray) -> float:
    """|C intersect I| / k with k = |I|."""
    return len(np.intersect1d(np.asarray(C), np.asarray(I))) / float(len(I))


def lfps_step(q_group: np.ndarray, K: np.ndarray, V: np.ndarray, prev_topk: Sequence[np.ndarray],
              n: int, k: int, r: int, n_recent: int = 1, n_sink: int = 0):
    """One decode step for the G query heads that share one KV head.

    q_group [G, d]; K, V [>= n, d]; prev_topk: G index arrays.
    Returns dict(cand, topk_idx [G] arrays, topk_score [G] arrays, cand_score [G, c], out [G, d])."""
    C = candidates(prev_topk, n, r, n_recent, n_sink)
    G = len(q_group)
    idx, sc, cs, out = [], [], [], []
    for h in range(G):
        cs.append(scores(q_group[h], K, C))
        I_h, s_h = score_topk(q_group[h], K, C, k)
        idx.append(I_h)
        sc.append(s_h)
        out.append(sparse_attn(q_group[h], K, V, I_h))
    return dict(cand=C, topk_idx=idx, topk_score=sc, cand_score=np.array(cs), out=np.array(out))
