"""The score / evict variants that take the window rows' log-sum-exp from the
caller (what the prefill attention kernel returns) instead of rebuilding it
with a first pass over K. The values are made here in float64 from the same
bf16 inputs, rounded to fp32; results must match the oracle to the usual
tolerance and the two-pass kernels far more closely."""
import numpy as np
import pytest
import torch
from scipy.special import logsumexp

from oracle import audiokv_oracle as O
from workloads import bf16_bits_to_f64, gen_item, gen_weights, get_config

from gpu_util import SCORE_RTOL, bf16_tensor, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    import paper_2604_06694_amd as A
    return A


def window_lse(q_win, k, G, causal=True):
    """[H_q, W] natural-log softmax denominators of the window rows (float64)."""
    H_q, W, d = q_win.shape
    L = k.shape[1]
    out = np.empty((H_q, W))
    for j in range(H_q):
        z = (q_win[j] @ k[j // G].T) / np.sqrt(d)                 # [W, L]
        for i in range(W):
            last = L - W + i if causal else L - 1
            out[j, i] = logsumexp(z[i, :last + 1])
    return out


@pytest.mark.parametrize("causal", [1, 0])
def test_score_with_lse_matches_oracle_and_two_pass(A, causal):
    cfg = get_config(1, n_items=2)
    lens = [700, 2048]
    items = [gen_item(cfg, i, seqlen=lens[i]) for i in range(2)]
    G = cfg.group
    q = bf16_tensor(np.concatenate([it["q_win"].reshape(-1) for it in items]))
    k = bf16_tensor(np.concatenate([it["k"].reshape(-1) for it in items]))
    lse = np.stack([window_lse(bf16_bits_to_f64(it["q_win"]), bf16_bits_to_f64(it["k"]), G, bool(causal)) for it in items])
    p = A.Params(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.window, pool_kernel=cfg.pool_kernel, causal=causal)
    s_lse = A.score(p, q, k, lens, lse=torch.from_numpy(lse.astype(np.float32)).cuda()).cpu().numpy()
    s_two = A.score(p, q, k, lens).cpu().numpy()
    off = 0
    for it, L in zip(items, lens):
        ref = O.score(bf16_bits_to_f64(it["q_win"]), bf16_bits_to_f64(it["k"]), pool_kernel=cfg.pool_kernel, causal=bool(causal))
        for h in range(cfg.n_kv_heads):
            assert rel_err(s_lse[off:off + L], ref[h]) <= SCORE_RTOL
            assert rel_err(s_lse[off:off + L], s_two[off:off + L]) <= 1e-4
            off += L


def test_evict_with_lse_keeps_the_same_tokens(A):
    cfg = get_config(1, n_items=2)
    items = [gen_item(cfg, i) for i in range(2)]
    L = cfg.seqlen
    q = bf16_tensor(np.concatenate([it["q_win"].reshape(-1) for it in items]))
    k = bf16_tensor(np.concatenate([it["k"].reshape(-1) for it in items]))
    v = bf16_tensor(np.concatenate([it["v"].reshape(-1) for it in items]))
    w = torch.from_numpy(gen_weights(cfg)).cuda()
    lse = np.stack([window_lse(bf16_bits_to_f64(it["q_win"]), bf16_bits_to_f64(it["k"]), cfg.group) for it in items])
    p = A.Params(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.window, pool_kernel=cfg.pool_kernel, floor_frac=cfg.floor_frac)
    a = A.evict(p, q, k, v, w, [L, L], cfg.ratio, cfg.cutoff, cfg.alpha, alloc_scope=A.SCOPE_GLOBAL)
    b = A.evict(p, q, k, v, w, [L, L], cfg.ratio, cfg.cutoff, cfg.alpha, alloc_scope=A.SCOPE_GLOBAL,
                lse=torch.from_numpy(lse.astype(np.float32)).cuda())
    torch.cuda.synchronize()
    assert torch.equal(a["budgets"], b["budgets"])
    cu = a["cu_budgets"].cpu().numpy()
    ia, ib = a["indices"].cpu().numpy(), b["indices"].cpu().numpy()
    agree = [len(np.intersect1d(ia[cu[g]:cu[g + 1]], ib[cu[g]:cu[g + 1]])) / (cu[g + 1] - cu[g]) for g in range(len(cu) - 1)]
    assert np.mean(agree) >= 0.999, agree
    # against the oracle, head by head
    bud = a["budgets"].cpu().numpy()
    for g in range(len(bud)):
        it, h = items[g // cfg.n_kv_heads], g % cfg.n_kv_heads
        s = O.score(bf16_bits_to_f64(it["q_win"][h * cfg.group:(h + 1) * cfg.group]), bf16_bits_to_f64(it["k"][h:h + 1]),
                    pool_kernel=cfg.pool_kernel)[0]
        s_hat = O.smooth(s, cfg.cutoff, cfg.alpha)
        ref = O.select(s_hat, int(bud[g]), cfg.window)
        mine = ib[cu[g]:cu[g + 1]]
        diff = np.setxor1d(mine, ref)
        if len(diff):
            thr = np.sort(s_hat[:L - cfg.window])[::-1][int(bud[g]) - cfg.window - 1]
            assert np.all(np.abs(s_hat[diff] - thr) <= SCORE_RTOL * np.abs(s_hat).max())
    with pytest.raises(A.AudioKVError):
        A.binding._check(A.binding._lib.audiokv_score_lse(None, None, None, None, None, None, 0, None, None, 0, None))
