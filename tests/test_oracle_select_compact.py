"""Pins for the oracle's stages 4 and 5 (top-k selection with forced window,
lower index wins ties; K/V gather)."""
import numpy as np
import pytest

from oracle import audiokv_oracle as O


def _lexsort_reference(s, budget, W):
    L = len(s)
    nc = L - W
    sc = np.asarray(s[:nc], dtype=np.float64) + 0.0        # -0.0 -> +0.0
    order = np.lexsort((np.arange(nc), -sc))               # primary: score desc, secondary: index asc
    return np.concatenate([np.sort(order[:budget - W]), np.arange(nc, L)])


@pytest.mark.parametrize("L,W,budget", [(50, 4, 20), (33, 1, 33), (64, 8, 8), (1000, 32, 400), (17, 0, 5)])
def test_equals_full_sort(L, W, budget):
    rng = np.random.default_rng(L)
    s = rng.standard_normal(L)
    s[rng.integers(0, L, size=L // 3)] = 0.5               # many exact ties
    idx = O.select(s, budget, W)
    assert np.array_equal(idx, _lexsort_reference(s, budget, W))
    assert len(idx) == budget and np.all(np.diff(idx) > 0)
    assert set(range(L - W, L)) <= set(idx.tolist())


def test_all_equal_scores_pure_tie_break():
    L, W, b = 40, 5, 17
    idx = O.select(np.full(L, 1.25), b, W)
    assert idx.tolist() == list(range(b - W)) + list(range(L - W, L))


def test_budget_extremes():
    s = np.random.default_rng(3).standard_normal(30)
    assert O.select(s, 30, 6).tolist() == list(range(30))
    assert O.select(s, 6, 6).tolist() == list(range(24, 30))


def test_signed_zero_compare_equal():
    s = np.array([0.0, -0.0, 0.0, -0.0, -1.0, -1.0])
    assert O.select(s, 2, 0).tolist() == [0, 1]
    assert O.select(s, 3, 0).tolist() == [0, 1, 2]


def test_threshold_value_property():
    rng = np.random.default_rng(4)
    s = rng.standard_normal(500)
    idx = O.select(s, 120, 20)
    chosen = np.setdiff1d(idx, np.arange(480, 500))
    rest = np.setdiff1d(np.arange(480), chosen)
    assert s[chosen].min() >= s[rest].max()


def test_window_scores_do_not_compete():
    s = np.zeros(20)
    s[-4:] = 100.0                      # forced anyway
    s[3] = 1.0
    assert O.select(s, 5, 4).tolist() == [3, 16, 17, 18, 19]


def test_compact_is_a_byte_exact_gather():
    rng = np.random.default_rng(5)
    k = rng.integers(0, 65536, size=(2, 11, 4)).astype(np.uint16)
    v = rng.integers(0, 65536, size=(2, 11, 4)).astype(np.uint16)
    idx = [np.array([0, 3, 10]), np.array([5])]
    ko, vo = O.compact(k, v, idx)
    assert ko.shape == (4, 4) and ko.dtype == np.uint16
    assert np.array_equal(ko[1], k[0, 3]) and np.array_equal(ko[3], k[1, 5])
    assert np.array_equal(vo[2], v[0, 10])
    full = [np.arange(11), np.arange(11)]
    ko, vo = O.compact(k, v, full)
    assert np.array_equal(ko.reshape(2, 11, 4), k) and np.array_equal(vo.reshape(2, 11, 4), v)
