"""Pins for the oracle's stage 2 (head-wise budget allocation; Sec. 3.1 Eq. 1,
Sec. 3.2 Eq. 12): exact total, bounds, monotonicity, the uniform degenerate
case, the floor relation of Eq. 12, and brute-force optimality on tiny cases."""
import itertools
import math

import numpy as np
import pytest

from oracle import audiokv_oracle as O


def _dirichlet(rng, n, a=1.0):
    g = rng.gamma(a, size=n)
    return g / g.sum()


@pytest.mark.parametrize("n,L,ratio,W,beta,a", [
    (4, 2048, 0.4, 32, 0.1, 1.0),
    (112, 8192, 0.4, 32, 0.1, 1.0),
    (112, 32768, 0.2, 64, 0.1, 1.0),
    (192, 16384, 0.4, 32, 0.1, 0.2),
    (2, 5003, 0.3, 32, 0.1, 1.0),
    (7, 100, 0.5, 4, 0.0, 0.3),
    (5, 64, 1.0, 8, 0.25, 1.0),
])
def test_sum_bounds_monotone(n, L, ratio, W, beta, a):
    rng = np.random.default_rng(n * 1000 + L)
    S = _dirichlet(rng, n, a)
    b, cu = O.allocate(S, L, ratio, window=W, floor_frac=beta)
    nk = O.n_keep_of(ratio, L)
    assert nk == int(math.floor(ratio * L + 0.5))
    assert int(b.sum()) == nk * n                       # exact total
    f = W + int(math.floor(beta * (nk - W)))
    assert b.min() >= f and b.max() <= L                # w + r <= b_h <= L
    order = np.argsort(S, kind="stable")
    assert np.all(np.diff(b[order]) >= 0)               # S_i >= S_j  =>  b_i >= b_j
    assert cu[0] == 0 and np.array_equal(np.diff(cu), b)


def test_equal_weights_give_uniform_budgets():
    # the paper's degenerate case: equal head importance reduces to uniform allocation
    for n, L, ratio in [(4, 2048, 0.4), (28, 8192, 0.4), (3, 1001, 0.37)]:
        b, _ = O.allocate(np.full(n, 0.25), L, ratio, window=32)
        assert np.all(b == O.n_keep_of(ratio, L))


def test_zero_weights_fall_back_to_equal_shares():
    b, _ = O.allocate(np.zeros(6), 1000, 0.4, window=16)
    assert np.all(b == 400)


def test_matches_plain_floor_formula_when_no_window_or_floor():
    # Eq. 12: B^(l,h) = floor(B * S / sum S); the top-up adds at most one unit
    rng = np.random.default_rng(11)
    for _ in range(20):
        n = int(rng.integers(2, 40))
        L = int(rng.integers(50, 5000))
        S = _dirichlet(rng, n, 2.0)              # mild: no head reaches the cap
        b, _ = O.allocate(S, L, 0.3, window=0, floor_frac=0.0)
        B = O.n_keep_of(0.3, L) * n
        fl = np.floor(B * S / S.sum()).astype(np.int64)
        if np.any(B * S / S.sum() > L):
            continue
        d = b - fl
        assert np.all((d == 0) | (d == 1))
        assert int(d.sum()) == B - int(fl.sum())


def test_scale_invariance_in_weights():
    rng = np.random.default_rng(12)
    S = _dirichlet(rng, 16)
    b1, _ = O.allocate(S, 4096, 0.4, window=32)
    b2, _ = O.allocate(S * 8.0, 4096, 0.4, window=32)   # power of two: exact rescale
    assert np.array_equal(b1, b2)


def test_cap_and_waterfill():
    # one dominant head cannot exceed L; its surplus is re-spread proportionally
    S = np.array([0.97, 0.01, 0.01, 0.01])
    L, W = 1000, 10
    b, _ = O.allocate(S, L, 0.5, window=W, floor_frac=0.0)
    assert b[0] == L
    assert int(b.sum()) == 500 * 4
    assert b[1] == b[2] == b[3] or abs(int(b[1]) - int(b[3])) <= 1
    # two heads over the cap after the first re-spread
    S = np.array([0.6, 0.35, 0.03, 0.02])
    b, _ = O.allocate(S, 100, 0.7, window=0, floor_frac=0.0)
    assert b[0] == 100 and b[1] == 100 and int(b.sum()) == 280
    assert b[2] >= b[3] and b[2] + b[3] == 80
    assert b[2] == 48 and b[3] == 32            # 80 split 3:2


def test_every_head_gets_window_plus_uniform_floor_by_hand():
    # Eq. 1: b = w + r + share. n_keep = 50, w = 10, beta = 0.25: r = floor(0.25 * (50 - 10)) = 10 (a share of the
    # non-window mean; not of n_keep, which would give 12). The head with weight 0 gets exactly w + r = 20, the other
    # one the remaining 2 * 50 - 20 = 80.
    b, cu = O.allocate(np.array([1.0, 0.0]), 100, 0.5, window=10, floor_frac=0.25)
    assert list(b) == [80, 20] and list(cu) == [0, 80, 100]
    # beta = 1: nothing left to share, every head gets n_keep whatever the weights
    b, _ = O.allocate(np.array([0.9, 0.1, 0.0]), 100, 0.5, window=10, floor_frac=1.0)
    assert list(b) == [50, 50, 50]
    # round-half-up of ratio * L: 0.5 * 5 = 2.5 -> 3, 0.25 * 10 = 2.5 -> 3, 0.4 * 2048 = 819.2 -> 819
    assert O.n_keep_of(0.5, 5) == 3 and O.n_keep_of(0.25, 10) == 3 and O.n_keep_of(0.4, 2048) == 819


def test_ratio_one_keeps_everything():
    b, _ = O.allocate(_dirichlet(np.random.default_rng(1), 5), 77, 1.0, window=8)
    assert np.all(b == 77)


def test_group_sum_of_query_head_weights():
    rng = np.random.default_rng(13)
    Sq = _dirichlet(rng, 28)
    b1, _ = O.allocate(Sq, 2048, 0.4, window=32, group=7)
    Skv = Sq.reshape(4, 7)
    acc = np.zeros(4)
    for g in range(7):
        acc = acc + Skv[:, g]
    b2, _ = O.allocate(acc, 2048, 0.4, window=32)
    assert np.array_equal(b1, b2) and len(b1) == 4


def test_tie_in_fractional_parts_goes_to_lower_index():
    # shares 2.5, 2.5, 2.5, 2.5 -> 10 units, floors give 8, the 2 spare go to heads 0 and 1
    b, _ = O.allocate(np.ones(4), 10, 0.25, window=0, floor_frac=0.0)   # n_keep = round(2.5) = 3 -> B=12
    assert int(b.sum()) == 12 and np.all(b == 3)
    S = np.array([1.0, 1.0, 2.0])     # B = 3*n_keep; choose so shares have equal fractions
    b, _ = O.allocate(S, 10, 0.2, window=0, floor_frac=0.0)            # n_keep=2, B=6: shares 1.5,1.5,3
    assert list(b) == [2, 1, 3]


@pytest.mark.parametrize("seed", range(12))
def test_brute_force_minimises_deviation(seed):
    # among all integer vectors with the right total and bounds, the result is
    # as close as any to the real-valued proportional shares (L1 and L-inf)
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(2, 5))
    L = int(rng.integers(6, 14))
    W = int(rng.integers(0, 2))
    ratio = float(rng.uniform(0.3, 0.9))
    S = _dirichlet(rng, n, 3.0)
    nk = O.n_keep_of(ratio, L)
    if nk < W:
        pytest.skip("infeasible draw")
    b, _ = O.allocate(S, L, ratio, window=W, floor_frac=0.0)
    f = W
    Bs = n * (nk - f)
    x = Bs * S / S.sum()
    if np.any(x > L - f):
        pytest.skip("cap active; covered elsewhere")
    best1 = best_inf = None
    for e in itertools.product(range(0, L - f + 1), repeat=n):
        if sum(e) != Bs:
            continue
        dev = np.abs(np.array(e) - x)
        best1 = dev.sum() if best1 is None else min(best1, dev.sum())
        best_inf = dev.max() if best_inf is None else min(best_inf, dev.max())
    mine = np.abs((b - f) - x)
    assert mine.sum() <= best1 + 1e-9
    assert mine.max() <= best_inf + 1e-9
