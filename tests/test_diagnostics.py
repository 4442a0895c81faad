"""Closed-form checks of the budget-divergence diagnostic (App. D, Tab.14)."""
import math

import numpy as np
import pytest

from oracle import aircache_oracle as O
from paper_2503_23956_amd.diagnostics import importance_ranking, js_divergence, single_rank_indices


def test_identical_and_rescaled_budgets_have_zero_divergence():
    k = np.array([3, 10, 7, 1])
    assert js_divergence(k, k) == 0.0
    assert js_divergence(k, 5 * k) == pytest.approx(0.0, abs=1e-15)


def test_disjoint_supports_reach_the_upper_bound_one():
    assert js_divergence([4, 0, 0, 0], [0, 0, 9, 0]) == pytest.approx(1.0)


def test_two_layer_closed_form_and_symmetry():
    # p = (1, 0), q = (1/2, 1/2): m = (3/4, 1/4); JS = 1/2 log2(4/3) + 1/2 (1/2 log2(2/3) + 1/2 log2 2)
    want = 0.5 * math.log2(4 / 3) + 0.5 * (0.5 * math.log2(2 / 3) + 0.5)
    assert js_divergence([6, 0], [5, 5]) == pytest.approx(want)
    assert js_divergence([5, 5], [6, 0]) == pytest.approx(want)


def test_bounds_on_random_budgets():
    rng = np.random.default_rng(0)
    for _ in range(50):
        a, b = rng.integers(1, 1000, 28), rng.integers(1, 1000, 28)
        d = js_divergence(a, b)
        assert 0.0 <= d <= 1.0


def test_bad_inputs_are_rejected():
    with pytest.raises(ValueError):
        js_divergence([1, 2], [1, 2, 3])
    with pytest.raises(ValueError):
        js_divergence([0, 0], [1, 1])
    with pytest.raises(ValueError):
        js_divergence([-1, 2], [1, 1])


def test_importance_ranking_is_the_order_top_k_takes_tokens():
    # the oracle's top-(j+1) set minus its top-j set is the token of rank j, ties to the lower index
    rng = np.random.default_rng(3)
    x = rng.random(40).astype(np.float32)
    x[[5, 17, 30]] = x[9]  # a four-way tie
    rank = importance_ranking(x)
    assert sorted(rank.tolist()) == list(range(40))
    for j in range(40):
        (tok,) = set(O.select_topk(x.astype(np.float64), j + 1).tolist()) - set(O.select_topk(x.astype(np.float64), j).tolist())
        assert rank[j] == tok
    pos = {int(t): j for j, t in enumerate(rank)}
    assert pos[5] < pos[9] < pos[17] < pos[30]


def test_single_rank_indices_layout_and_errors():
    sc = np.zeros((2, 3, 8), dtype=np.float32)
    sc[0, :, :5] = [0.1, 0.5, 0.2, 0.5, 0.05]
    sc[1, :, :8] = np.arange(8)
    idx = single_rank_indices(sc, [5, 8], 1)
    assert idx.shape == sc.shape and idx.dtype == np.int32
    assert idx[0, :, 0].tolist() == [3, 3, 3] and idx[1, :, 0].tolist() == [6, 6, 6]
    with pytest.raises(ValueError):
        single_rank_indices(sc, [5, 8], 5)
