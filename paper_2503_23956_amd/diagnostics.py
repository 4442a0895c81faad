"""Host-side diagnostics of the layer budgets and of the importance ranking (nothing here is on the hot path).

The paper compares allocation strategies by the Jensen-Shannon divergence between their layer-budget
vectors (App. D, Tab.14: "ranges from 0 to 1", i.e. logarithms to base 2).  A budget vector k_l is
read as the distribution p_l = k_l / sum_l k_l over the layers.
"""
from __future__ import annotations

import numpy as np


def js_divergence(k_a, k_b) -> float:
    """Jensen-Shannon divergence, base 2, between two layer-budget vectors of the same length."""
    a = np.asarray(k_a, dtype=np.float64)
    b = np.asarray(k_b, dtype=np.float64)
    if a.shape != b.shape or a.ndim != 1:
        raise ValueError("budget vectors must be one-dimensional and of equal length")
    if (a < 0).any() or (b < 0).any() or a.sum() <= 0 or b.sum() <= 0:
        raise ValueError("budgets must be non-negative with a positive sum")
    p, q = a / a.sum(), b / b.sum()
    m = 0.5 * (p + q)

    def kl(x, y):
        nz = x > 0
        return float(np.sum(x[nz] * np.log2(x[nz] / y[nz])))

    return 0.5 * kl(p, m) + 0.5 * kl(q, m)


def importance_ranking(scores_row) -> np.ndarray:
    """Visual-token indices of one (layer, sequence, KV head) from the most to the least important,
    equal scores in index order: the order in which top-k selection takes tokens."""
    x = np.asarray(scores_row)
    if x.ndim != 1:
        raise ValueError("one row of importance scores expected")
    return np.lexsort((np.arange(x.shape[0]), -x.astype(np.float64))).astype(np.int32)


def single_rank_indices(scores, vis_lens, rank: int) -> np.ndarray:
    """Index lists for air_set_indices that keep, per (sequence, KV head), only the token of importance
    rank `rank` (0 = the most important): the one-token-at-a-time study of Sec.4.3 (Fig.4), to be used
    with budgets of 1.  scores: [B][H_kv][max_vis_len] as air_get_scores returns them."""
    sc = np.asarray(scores)
    out = np.zeros(sc.shape, dtype=np.int32)
    for b in range(sc.shape[0]):
        n = int(vis_lens[b])
        if not 0 <= rank < n:
            raise ValueError("rank outside the visual span")
        for h in range(sc.shape[1]):
            out[b, h, 0] = importance_ranking(sc[b, h, :n])[rank]
    return out
