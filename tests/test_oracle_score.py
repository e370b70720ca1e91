"""Pins for the oracle's stage 1 (window attention + pooling).

Each check is something the definition fixes independently of the oracle's own
code: closed forms, a library softmax, and a loop-level brute force written
from the definition (Sec. 3.3 importance sequence; SnapKV-style local pooling).
"""
import math

import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import audiokv_oracle as O


def _brute_window_attention(q, k, causal=True):
    """Pure-Python loops, no vectorisation, written from the definition."""
    H_q, W, d = q.shape
    H_kv, L, _ = k.shape
    G = H_q // H_kv
    raw = [[0.0] * L for _ in range(H_kv)]
    for qh in range(H_q):
        h = qh // G
        for i in range(W):
            last = L - W + i if causal else L - 1
            logits = []
            for j in range(last + 1):
                acc = 0.0
                for c in range(d):
                    acc += float(q[qh, i, c]) * float(k[h, j, c])
                logits.append(acc / math.sqrt(d))
            m = max(logits)
            ex = [math.exp(v - m) for v in logits]
            z = sum(ex)
            for j in range(last + 1):
                raw[h][j] += ex[j] / z
    return np.array(raw)


@pytest.mark.parametrize("H_q,H_kv,W,L,d", [(2, 1, 3, 7, 4), (4, 2, 2, 16, 8), (3, 3, 5, 5, 2), (6, 2, 4, 11, 3)])
@pytest.mark.parametrize("causal", [True, False])
def test_brute_force_tiny(H_q, H_kv, W, L, d, causal):
    rng = np.random.default_rng(7 + L + W)
    q = rng.standard_normal((H_q, W, d)) * 2.0
    k = rng.standard_normal((H_kv, L, d)) * 2.0
    got = O.window_attention(q, k, causal=causal)
    ref = _brute_window_attention(q, k, causal=causal)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-14)


def test_total_mass_is_group_times_window():
    # every softmax row sums to 1, so the summed attention carries exactly G*W
    rng = np.random.default_rng(0)
    H_q, H_kv, W, L, d = 8, 2, 16, 300, 32
    q = rng.standard_normal((H_q, W, d)) * 3
    k = rng.standard_normal((H_kv, L, d)) * 3
    raw = O.window_attention(q, k)
    np.testing.assert_allclose(raw.sum(axis=1), (H_q // H_kv) * W, rtol=1e-12)
    assert np.all(raw >= 0.0)


def test_single_row_equals_library_softmax():
    rng = np.random.default_rng(1)
    L, d = 97, 16
    q = rng.standard_normal((1, 1, d))
    k = rng.standard_normal((1, L, d))
    raw = O.window_attention(q, k)           # W = 1: the one row sees all L keys
    ref = scipy_softmax((k[0] @ q[0, 0]) / math.sqrt(d))
    np.testing.assert_allclose(raw[0], ref, rtol=1e-12, atol=1e-16)


def test_explicit_scale_argument():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((1, 1, 8))
    k = rng.standard_normal((1, 20, 8))
    raw = O.window_attention(q, k, scale=0.37)
    np.testing.assert_allclose(raw[0], scipy_softmax(0.37 * (k[0] @ q[0, 0])), rtol=1e-12)


def test_zero_queries_closed_form_harmonic():
    # all logits equal: row i is uniform over its L-W+i+1 visible keys
    H_q, H_kv, W, L, d = 6, 2, 5, 40, 4
    G = H_q // H_kv
    q = np.zeros((H_q, W, d))
    k = np.random.default_rng(3).standard_normal((H_kv, L, d))
    raw = O.window_attention(q, k)
    expect = np.zeros(L)
    for j in range(L):
        for i in range(W):
            if j <= L - W + i:
                expect[j] += G / (L - W + i + 1)
    for h in range(H_kv):
        np.testing.assert_allclose(raw[h], expect, rtol=1e-13)
    # prefix keys: difference of harmonic numbers H_L - H_{L-W}
    Hn = lambda n: sum(1.0 / t for t in range(1, n + 1))
    np.testing.assert_allclose(raw[0, 0], G * (Hn(L) - Hn(L - W)), rtol=1e-13)
    # non-causal: exactly G*W/L everywhere
    np.testing.assert_allclose(O.window_attention(q, k, causal=False), G * W / L, rtol=1e-13)


def test_causal_mask_hides_later_window_keys():
    # a huge key at the very last position is visible to the last row only
    H_q, H_kv, W, L, d = 1, 1, 4, 12, 2
    q = np.ones((H_q, W, d))
    k = np.zeros((H_kv, L, d))
    k[0, L - 1] = 50.0
    raw = O.window_attention(q, k)
    # last row puts ~all its mass on the last key; other rows never see it
    assert abs(raw[0, L - 1] - 1.0) < 1e-12
    expect_prefix = sum(1.0 / (L - W + i + 1) for i in range(W - 1))
    np.testing.assert_allclose(raw[0, 0], expect_prefix, rtol=1e-9)


def test_gqa_group_mapping():
    # query heads [0,G) belong to KV head 0, [G,2G) to KV head 1
    H_q, H_kv, W, L, d = 4, 2, 1, 6, 2
    q = np.zeros((H_q, W, d))
    q[3] = [[30.0, 0.0]]                    # only a head of group 1 is peaky
    k = np.zeros((H_kv, L, d))
    k[:, 2] = [1.0, 0.0]
    raw = O.window_attention(q, k)
    np.testing.assert_allclose(raw[0], 2.0 / L, rtol=1e-12)        # group 0: two uniform rows
    assert raw[1, 2] > 1.0 + 0.9 * (1.0 / L)                        # group 1: one row ~ delta at key 2


# ------------------------------ pooling ------------------------------------

def test_avg_pool_constant_closed_form():
    k, L, c = 7, 20, 3.5
    out = O.pool(np.full(L, c), k)
    half = k // 2
    for j in range(L):
        over = max(0, half - j) + max(0, j + half - (L - 1))     # taps hanging over an edge
        assert abs(out[j] - c * (k - over) / k) < 1e-14


def test_avg_pool_impulse_response():
    L, k = 15, 5
    x = np.zeros(L)
    x[6] = 2.0
    out = O.pool(x, k)
    expect = np.zeros(L)
    expect[4:9] = 2.0 / k
    np.testing.assert_allclose(out, expect, atol=1e-16)


@pytest.mark.parametrize("mode", ["avg", "max"])
@pytest.mark.parametrize("k", [1, 3, 7])
def test_pool_brute_force(mode, k):
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 13))
    out = O.pool(x, k, mode)
    half = k // 2
    for h in range(2):
        for j in range(13):
            taps = [x[h, t] for t in range(j - half, j + half + 1) if 0 <= t < 13]
            ref = sum(taps) / k if mode == "avg" else max(taps)
            assert abs(out[h, j] - ref) < 1e-14


def test_kernel_one_is_identity():
    x = np.random.default_rng(6).standard_normal(9)
    assert np.array_equal(O.pool(x, 1), x)


def test_score_is_pool_of_window_attention():
    rng = np.random.default_rng(8)
    q = rng.standard_normal((4, 3, 8))
    k = rng.standard_normal((2, 30, 8))
    raw = O.window_attention(q, k)
    s = O.score(q, k, pool_kernel=7)
    # interior positions: plain mean of 7 neighbours
    for j in range(3, 27):
        np.testing.assert_allclose(s[:, j], raw[:, j - 3:j + 4].mean(axis=1), rtol=1e-13)
