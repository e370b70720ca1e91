"""Pins for the oracle's decode-side consumer (single-query attention over the
retained rows of each KV head): closed forms, special cases and brute force."""
import math

import numpy as np

from oracle import audiokv_oracle as O


def brute(q, k_rows, v_rows, scale):
    H_q, d = q.shape
    G = H_q // len(k_rows)
    out = np.zeros((H_q, d))
    for j in range(H_q):
        K, V = k_rows[j // G], v_rows[j // G]
        logits = [scale * sum(q[j][c] * K[t][c] for c in range(d)) for t in range(len(K))]
        m = max(logits)
        w = [math.exp(x - m) for x in logits]
        Z = sum(w)
        for t in range(len(K)):
            for c in range(d):
                out[j][c] += w[t] / Z * V[t][c]
    return out


def test_brute_force_small_ragged_heads():
    rng = np.random.default_rng(0)
    H_q, H_kv, d = 6, 2, 5
    q = rng.normal(size=(H_q, d))
    budgets = [3, 7]
    k_rows = [rng.normal(size=(b, d)) for b in budgets]
    v_rows = [rng.normal(size=(b, d)) for b in budgets]
    for scale in (None, 0.3):
        ref = brute(q, k_rows, v_rows, 1 / math.sqrt(d) if scale is None else scale)
        np.testing.assert_allclose(O.decode_attend(q, k_rows, v_rows, scale=scale), ref, atol=1e-13)


def test_closed_forms():
    rng = np.random.default_rng(1)
    d = 8
    V = rng.normal(size=(11, d))
    K = rng.normal(size=(11, d))
    # zero query: uniform weights, the output is the mean of the retained V rows
    np.testing.assert_allclose(O.decode_attend(np.zeros((2, d)), [K], [V]), np.tile(V.mean(0), (2, 1)), atol=1e-14)
    # one retained row: the output is that row whatever the query
    np.testing.assert_allclose(O.decode_attend(rng.normal(size=(3, d)), [K[:1]], [V[:1]]), np.tile(V[0], (3, 1)), atol=1e-14)
    # equal keys: uniform weights again
    np.testing.assert_allclose(O.decode_attend(rng.normal(size=(1, d)), [np.tile(K[0], (11, 1))], [V]), V.mean(0)[None], atol=1e-13)
    # two rows with logits differing by ln 3: weights 3/4 and 1/4
    q = np.zeros((1, d)); q[0, 0] = 1.0
    K2 = np.zeros((2, d)); K2[0, 0] = math.log(3.0)
    out = O.decode_attend(q, [K2], [V[:2]], scale=1.0)
    np.testing.assert_allclose(out[0], 0.75 * V[0] + 0.25 * V[1], atol=1e-14)
    # a dominant key: the output tends to its value row; huge logits do not overflow
    Kd = K.copy(); Kd[4] = 1e4 * q[0]
    np.testing.assert_allclose(O.decode_attend(q, [Kd], [V], scale=1.0)[0], V[4], atol=1e-12)


def test_invariances_and_group_mapping():
    rng = np.random.default_rng(2)
    H_q, H_kv, d = 8, 4, 16
    q = rng.normal(size=(H_q, d))
    k_rows = [rng.normal(size=(b, d)) for b in (5, 9, 2, 30)]
    v_rows = [rng.normal(size=(b, d)) for b in (5, 9, 2, 30)]
    out = O.decode_attend(q, k_rows, v_rows)
    # the order of the retained rows does not matter
    perm = [rng.permutation(len(k)) for k in k_rows]
    out_p = O.decode_attend(q, [k[p] for k, p in zip(k_rows, perm)], [v[p] for v, p in zip(v_rows, perm)])
    np.testing.assert_allclose(out_p, out, atol=1e-13)
    # query head j reads KV head j // G: changing KV head 2 touches query heads 4 and 5 only
    v2 = [v.copy() for v in v_rows]; v2[2] += 1.0
    out2 = O.decode_attend(q, k_rows, v2)
    changed = np.abs(out2 - out).max(axis=1) > 1e-9
    assert list(np.nonzero(changed)[0]) == [4, 5]
    np.testing.assert_allclose(out2[4:6], out[4:6] + 1.0, atol=1e-12)      # weights sum to one
    # outputs are convex combinations of the value rows
    for j in range(H_q):
        V = v_rows[j // 2]
        assert np.all(out[j] <= V.max(0) + 1e-12) and np.all(out[j] >= V.min(0) - 1e-12)
    # against the library softmax
    from scipy.special import softmax
    for j in range(H_q):
        w = softmax((k_rows[j // 2] @ q[j]) / math.sqrt(d))
        np.testing.assert_allclose(out[j], w @ v_rows[j // 2], atol=1e-13)
