"""CPU oracle of the routing analytics the paper reports for budgeted routing
(Section 5, "Analysis of Expert Load Balance" and "Analysis of Budget
Allocation in Alloc-L and Alloc-T").

TEST INFRASTRUCTURE, NOT THE PRODUCT (see oracle/__init__.py).

Inputs: one layer's routing result -- scores [T,E] (softmax over all experts),
each token's sorted candidates (ids, s) [T,K] and its kept count k_t.  "Original"
routing keeps all K candidates of a token, budgeted routing the first k_t.

Definitions, written out with numpy in fp64 (the paper names the statistics and
leaves the details open; these are the readings taken):
  load[e]   number of kept pairs whose expert is e
  wload[e]  sum of their routing scores ("weighted load"); p = wload / sum(wload)
  normalised entropy  -sum p ln p / ln E            (0 ln 0 = 0)
  JS divergence       (KL(p||m) + KL(q||m)) / 2, m = (p+q)/2, natural logarithm
  Spearman            Pearson correlation of average ranks (ties share the mean of
                      their positions); 0 when one side is constant
  token entropy       H_t = -sum_e s[t,e] ln s[t,e]
"""
from __future__ import annotations

import numpy as np


def average_ranks(v: np.ndarray) -> np.ndarray:
    """1-based ranks in ascending order, equal values sharing their mean position."""
    v = np.asarray(v)
    n = len(v)
    ranks = np.empty(n, dtype=np.float64)
    for i in range(n):
        less = int(np.sum(v < v[i]))
        equal = int(np.sum(v == v[i]))
        ranks[i] = less + (equal + 1) / 2.0
    return ranks


def spearman(a, b) -> float:
    ra, rb = average_ranks(a), average_ranks(b)
    da, db = ra - ra.mean(), rb - rb.mean()
    den = np.sqrt(np.sum(da * da) * np.sum(db * db))
    return 0.0 if den == 0 else float(np.sum(da * db) / den)


def normalised_entropy(p: np.ndarray) -> float:
    p = np.asarray(p, dtype=np.float64)
    nz = p[p > 0]
    return float(-np.sum(nz * np.log(nz)) / np.log(len(p))) if len(p) > 1 else 0.0


def js_divergence(p: np.ndarray, q: np.ndarray) -> float:
    p, q = np.asarray(p, dtype=np.float64), np.asarray(q, dtype=np.float64)
    m = 0.5 * (p + q)

    def kl(a, b):
        nz = a > 0
        return float(np.sum(a[nz] * np.log(a[nz] / b[nz])))
    return 0.5 * kl(p, m) + 0.5 * kl(q, m)


def token_entropy(scores: np.ndarray) -> np.ndarray:
    s = np.asarray(scores, dtype=np.float64)
    with np.errstate(divide="ignore", invalid="ignore"):
        terms = np.where(s > 0, -s * np.log(s), 0.0)
    return terms.sum(axis=1)


def routing_stats(scores, topk_ids, topk_s, keep_count, entropy_for_ranks=None) -> dict:
    """All statistics.  entropy_for_ranks: optionally the token entropies to rank
    (lets a test rank exactly the values another implementation produced)."""
    scores = np.asarray(scores)
    ids = np.asarray(topk_ids)
    s = np.asarray(topk_s, dtype=np.float64)
    k = np.asarray(keep_count)
    T, E = scores.shape
    K = ids.shape[1]
    load_o = np.zeros(E, dtype=np.int64)
    load_k = np.zeros(E, dtype=np.int64)
    wl_o = np.zeros(E, dtype=np.float64)
    wl_k = np.zeros(E, dtype=np.float64)
    for t in range(T):
        for j in range(K):
            e = int(ids[t, j])
            load_o[e] += 1
            wl_o[e] += s[t, j]
            if j < k[t]:
                load_k[e] += 1
                wl_k[e] += s[t, j]
    p = wl_o / wl_o.sum() if wl_o.sum() > 0 else np.zeros(E)
    q = wl_k / wl_k.sum() if wl_k.sum() > 0 else np.zeros(E)
    H = token_entropy(scores)
    return dict(load_orig=load_o, load_kept=load_k, wload_orig=wl_o, wload_kept=wl_k,
                spearman_load=spearman(load_o, load_k),
                entropy_orig=normalised_entropy(p), entropy_kept=normalised_entropy(q),
                js_divergence=js_divergence(p, q), token_entropy=H,
                spearman_tokens=spearman(H if entropy_for_ranks is None
                                         else np.asarray(entropy_for_ranks), k))
