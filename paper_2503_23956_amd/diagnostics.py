"""Host-side diagnostics of the layer budgets (nothing here is on the hot path).

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
