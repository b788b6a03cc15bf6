"""Pins of the oracle's region-aware threshold control (paper Section 5.2, Appendix Algorithm 2)."""
import math

import numpy as np
import pytest

import oracle


def test_tile_std_closed_forms_and_brute_force():
    assert oracle.tile_std([1.0, -1.0] * 50) == pytest.approx(1.0, rel=1e-15)
    n = 1000                                                   # 0..n-1: variance (n^2 - 1) / 12
    assert oracle.tile_std(np.arange(n)) == pytest.approx(math.sqrt((n * n - 1) / 12.0), rel=1e-13)
    assert oracle.tile_std(np.full((3, 4), 7.25)) == 0.0
    rng = np.random.default_rng(0)
    x = rng.normal(3.0, 2.0, size=(2, 3, 5))
    vals = [float(v) for v in x.ravel()]
    m = sum(vals) / len(vals)
    brute = math.sqrt(sum((v - m) ** 2 for v in vals) / len(vals))
    assert oracle.tile_std(x) == pytest.approx(brute, rel=1e-13)
    assert oracle.tile_std(x + 1e3) == pytest.approx(brute, rel=1e-9)   # shift invariance
    assert oracle.tile_std(-2.0 * x) == pytest.approx(2.0 * brute, rel=1e-13)


def test_tracker_is_the_mean_of_the_per_step_values():
    tr = oracle.StdTracker(3)
    steps = [[1.0, 2.0, 4.0], [3.0, 2.0, 0.0], [2.0, 5.0, 2.0], [0.0, 1.0, 6.0]]
    for s in steps:
        tr.update(s)
    np.testing.assert_allclose(tr.mean, np.mean(steps, axis=0), rtol=1e-15)
    np.testing.assert_allclose(tr.normalized(), [0.0, 1.0 / 1.5, 1.0], rtol=1e-15)   # means 1.5, 2.5, 3.0
    flat = oracle.StdTracker(2)
    flat.update([2.0, 2.0])
    assert list(flat.normalized()) == [0.0, 0.0]


def test_policies_on_a_hand_example():
    sigma = [0.2, 0.9, 0.1, 0.5]
    np.testing.assert_allclose(oracle.region_thresholds(sigma, 0.05, 0.4, "MaxMin"),
                               [0.05, 0.05 * 1.4, 0.05 * 0.8, 0.05], rtol=1e-15)
    np.testing.assert_allclose(oracle.region_thresholds(sigma, 0.05, 0.4, "TopSelect"),
                               [0.05, 0.05 * 1.4, 0.05, 0.05 * 1.2], rtol=1e-15)
    with pytest.raises(ValueError):
        oracle.region_thresholds(sigma, 0.05, 0.4, "Other")


def test_only_the_order_matters_and_ties_go_to_the_lowest_index():
    rng = np.random.default_rng(1)
    s = rng.random(9)
    for mode in ("MaxMin", "TopSelect"):
        ref = oracle.region_thresholds(s, 0.09, 0.3, mode)
        np.testing.assert_array_equal(oracle.region_thresholds(5.0 * s + 2.0, 0.09, 0.3, mode), ref)
        np.testing.assert_array_equal(oracle.region_thresholds(np.exp(s), 0.09, 0.3, mode), ref)
    tie = [0.5, 0.9, 0.9, 0.1, 0.1]
    np.testing.assert_allclose(oracle.region_thresholds(tie, 1.0, 0.2, "MaxMin"), [1, 1.2, 1, 0.9, 1], rtol=1e-15)
    np.testing.assert_allclose(oracle.region_thresholds(tie, 1.0, 0.2, "TopSelect"), [1, 1.2, 1.1, 1, 1], rtol=1e-15)
    # all equal: argmax = argmin = tile 0, the later assignment (-alpha / 2) stands
    np.testing.assert_allclose(oracle.region_thresholds([0.3, 0.3], 1.0, 0.2, "MaxMin"), [0.9, 1.0], rtol=1e-15)
    np.testing.assert_allclose(oracle.region_thresholds([0.3], 1.0, 0.2, "TopSelect"), [1.2], rtol=1e-15)


def test_thresholds_sum_rule():
    """MaxMin moves the total by +alpha/2 tau_base, TopSelect by +3 alpha/2 tau_base (for >= 2 distinct tiles)."""
    s = [0.3, 0.1, 0.7, 0.4, 0.2]
    assert oracle.region_thresholds(s, 0.05, 0.5, "MaxMin").sum() == pytest.approx(0.05 * (5 + 0.25), rel=1e-14)
    assert oracle.region_thresholds(s, 0.05, 0.5, "TopSelect").sum() == pytest.approx(0.05 * (5 + 0.75), rel=1e-14)
