"""Closed-form checks of the budget-divergence diagnostic (App. D, Tab.14)."""
import math

import numpy as np
import pytest

from paper_2503_23956_amd.diagnostics import js_divergence


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
