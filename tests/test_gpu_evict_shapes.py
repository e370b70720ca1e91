"""Fused audiokv_evict against the oracle's whole chain over the geometry grid
the kernels are specialised on: head dims 64 / 128 / 256, GQA groups 1..16,
both K/V layouts, causal on / off, per-item budget pools, ragged lengths that
are and are not powers of two. Random inputs (no workload structure): every
head is compared."""
import numpy as np
import pytest
import torch

from oracle import audiokv_oracle as O
from workloads import bf16_bits_to_f64, f64_to_bf16_bits

from gpu_util import SCORE_RTOL, bf16_bits, bf16_tensor, pack_items_head_major, pack_items_token_major

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    import paper_2604_06694_amd as A
    return A


CASES = [
    # H_q, H_kv, d, W, lens, layout, causal, ratio
    (8, 2, 64, 16, [300, 1024], 0, 1, 0.4),
    (8, 8, 64, 8, [512], 1, 1, 0.3),
    (8, 2, 256, 32, [2048], 1, 1, 0.25),
    (32, 4, 128, 32, [1000, 4096], 0, 1, 0.5),
    (16, 1, 128, 16, [640], 0, 1, 0.4),
    (28, 4, 128, 64, [1536], 1, 0, 0.4),
    (4, 4, 256, 8, [129, 64, 2500], 0, 0, 0.6),
]


@pytest.mark.parametrize("H_q,H_kv,d,W,lens,layout,causal,ratio", CASES)
def test_evict_shapes(A, H_q, H_kv, d, W, lens, layout, causal, ratio):
    rng = np.random.default_rng(H_q * 100 + d + W + len(lens))
    G = H_q // H_kv
    items = []
    for L in lens:
        # a smooth drift in the keys gives the scores some low-frequency structure for the smoothing to keep
        drift = np.cumsum(rng.standard_normal((H_kv, L, d)) * 0.15, axis=1)
        items.append({"q_win": f64_to_bf16_bits(rng.standard_normal((H_q, W, d))),
                      "k": f64_to_bf16_bits(rng.standard_normal((H_kv, L, d)) + drift),
                      "v": f64_to_bf16_bits(rng.standard_normal((H_kv, L, d))), "seqlen": L})
    pack = pack_items_token_major if layout else pack_items_head_major
    q = bf16_tensor(np.concatenate([it["q_win"].reshape(-1) for it in items]))
    k, v = bf16_tensor(pack(items, "k")), bf16_tensor(pack(items, "v"))
    w = (rng.dirichlet(np.ones(H_kv), size=len(lens)).reshape(-1)).astype(np.float32)
    p = A.Params(H_q, H_kv, d, W, causal=causal, kv_layout=layout)
    cutoff, alpha = 0.25, 0.75
    out = A.evict(p, q, k, v, torch.from_numpy(w).cuda(), lens, ratio, cutoff, alpha, alloc_scope=A.SCOPE_ITEM)
    torch.cuda.synchronize()
    budgets, cu_b = out["budgets"].cpu().numpy(), out["cu_budgets"].cpu().numpy()
    idx = out["indices"].cpu().numpy()
    ko, vo = bf16_bits(out["k_out"]), bf16_bits(out["v_out"])
    beta = float(np.float32(p.floor_frac))
    agree = []
    for i, it in enumerate(items):
        L = it["seqlen"]
        ref_b, _ = O.allocate(w[i * H_kv:(i + 1) * H_kv].astype(np.float64), L, ratio, window=W, floor_frac=beta)
        assert np.array_equal(budgets[i * H_kv:(i + 1) * H_kv], ref_b)
        s = O.score(bf16_bits_to_f64(it["q_win"]), bf16_bits_to_f64(it["k"]), causal=bool(causal))
        for h in range(H_kv):
            g = i * H_kv + h
            s_hat = O.smooth(s[h], cutoff, alpha)
            ref = O.select(s_hat, int(ref_b[h]), W)
            mine = idx[cu_b[g]:cu_b[g + 1]]
            assert len(mine) == ref_b[h] and np.all(np.diff(mine) > 0)
            assert np.array_equal(mine[-W:], np.arange(L - W, L))
            assert np.array_equal(ko[cu_b[g]:cu_b[g + 1]], it["k"][h][mine])
            assert np.array_equal(vo[cu_b[g]:cu_b[g + 1]], it["v"][h][mine])
            agree.append(len(np.intersect1d(mine, ref)) / len(ref))
            diff = np.setxor1d(mine, ref)
            if len(diff):
                want = int(ref_b[h]) - W
                thr = np.sort(s_hat[:L - W])[::-1][want - 1]
                assert np.all(np.abs(s_hat[diff] - thr) <= SCORE_RTOL * np.abs(s_hat).max())
    assert np.mean(agree) >= 0.999, agree


@pytest.mark.parametrize("L,W,ratio", [(64, 64, 1.0), (128, 32, 0.25), (96, 16, 1.0), (33, 1, 0.5), (4096, 1, 0.01)])
def test_evict_degenerate_budgets(A, L, W, ratio):
    """Window as long as the sequence, budgets equal to the window (nothing but the forced tail is kept),
    everything kept, a one-token window, one percent kept."""
    rng = np.random.default_rng(L + W)
    H_q, H_kv, d = 4, 2, 64
    it = {"q_win": f64_to_bf16_bits(rng.standard_normal((H_q, W, d))),
          "k": f64_to_bf16_bits(rng.standard_normal((H_kv, L, d))),
          "v": f64_to_bf16_bits(rng.standard_normal((H_kv, L, d)))}
    p = A.Params(H_q, H_kv, d, W)
    w = np.array([0.3, 0.7], dtype=np.float32)
    out = A.evict(p, bf16_tensor(it["q_win"].reshape(-1)), bf16_tensor(it["k"].reshape(-1)), bf16_tensor(it["v"].reshape(-1)),
                  torch.from_numpy(w).cuda(), [L], ratio, 0.25, 1.0, alloc_scope=A.SCOPE_ITEM)
    torch.cuda.synchronize()
    b, cu = out["budgets"].cpu().numpy(), out["cu_budgets"].cpu().numpy()
    ref_b, _ = O.allocate(w.astype(np.float64), L, ratio, window=W, floor_frac=float(np.float32(p.floor_frac)))
    assert np.array_equal(b, ref_b) and b.sum() == O.n_keep_of(ratio, L) * H_kv
    idx = out["indices"].cpu().numpy()
    ko = bf16_bits(out["k_out"])
    s = O.score(bf16_bits_to_f64(it["q_win"]), bf16_bits_to_f64(it["k"]))
    for h in range(H_kv):
        mine = idx[cu[h]:cu[h + 1]]
        assert np.array_equal(mine[-W:], np.arange(L - W, L)) and np.all(np.diff(mine) > 0)
        assert np.array_equal(ko[cu[h]:cu[h + 1]], it["k"][h][mine])
        if b[h] == W:
            assert np.array_equal(mine, np.arange(L - W, L))
        if b[h] == L:
            assert np.array_equal(mine, np.arange(L))
        ref = O.select(O.smooth(s[h], 0.25, 1.0), int(b[h]), W)
        diff = np.setxor1d(mine, ref)
        if len(diff):
            s_hat = O.smooth(s[h], 0.25, 1.0)
            thr = np.sort(s_hat[:L - W])[::-1][int(b[h]) - W - 1]
            assert np.all(np.abs(s_hat[diff] - thr) <= SCORE_RTOL * np.abs(s_hat).max())


def test_empty_batch_through_the_binding(A):
    """No items: the fused call and the stage calls return without enqueueing anything."""
    p = A.Params(8, 2, 128, 16)
    e16 = torch.empty(0, dtype=torch.bfloat16, device="cuda")
    out = A.evict(p, e16, e16, e16, torch.empty(0, dtype=torch.float32, device="cuda"), [], 0.4, 0.125, 1.0)
    assert out["total_rows"] == 0
    s = A.score(p, e16, e16, [])
    assert s.numel() == 0
    torch.cuda.synchronize()
