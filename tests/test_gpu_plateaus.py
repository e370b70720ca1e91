"""Masks that leave an exact plateau or the input itself (paper Sec. 3.3, Eqs. 17-19: with only the DC bin kept the
inverse transform is the mean at every position; with every bin kept it is the input). The selection that follows
breaks ties by index, so these cases must come out of the kernels as exact plateaus / exact copies at every length
(powers of two, and lengths that go through the chirp-z transform), not as a constant plus rounding noise."""
import numpy as np
import pytest
import torch

from oracle import audiokv_oracle as O
from workloads import bf16_bits_to_f64, gen_item, gen_weights, get_config

from gpu_util import SCORE_RTOL, bf16_tensor

pytestmark = pytest.mark.gpu

LENGTHS = [64, 777, 2048, 3000, 18, 19, 30000]      # 3000 and 30000 take the multi-workgroup chirp-z path otherwise


@pytest.fixture(scope="module")
def A():
    import paper_2604_06694_amd as A
    return A


def _scores(rng, H, L):
    return (0.02 + 0.01 * rng.random((H, L)) + (rng.random((H, L)) < 0.01) * rng.random((H, L))).astype(np.float32)


@pytest.mark.parametrize("L", LENGTHS)
@pytest.mark.parametrize("alpha", [1.0, 0.5])
def test_dc_only_mask_gives_an_exact_plateau(A, L, alpha):
    rng = np.random.default_rng(L)
    H = 3
    s = _scores(rng, H, L)
    p = A.Params(H, H, 128, 1)
    out = A.smooth(p, torch.from_numpy(s.reshape(-1)).cuda(), [L], 0.0, alpha).cpu().numpy().reshape(H, L)
    for h in range(H):
        ref = O.smooth(s[h].astype(np.float64), 0.0, alpha)
        assert np.abs(out[h] - ref).max() <= 1e-6 * np.abs(ref).max()
        if alpha == 1.0:
            assert np.all(out[h] == out[h][0]), "not one value"      # bitwise plateau
            assert np.all(ref == ref[0])                             # and so is the definition's


@pytest.mark.parametrize("L", LENGTHS)
def test_energy_rule_that_keeps_only_dc_gives_an_exact_plateau(A, L):
    # non-negative scores: the DC bin alone holds most of the energy, so Eqs. 15-16 taken literally give k* = 0
    rng = np.random.default_rng(100 + L)
    H = 2
    s = (0.02 + 0.01 * rng.random((H, L))).astype(np.float32)
    p = A.Params(H, H, 128, 1, cutoff_mode=A.CUTOFF_ENERGY)
    x = torch.from_numpy(s.reshape(-1)).cuda()
    ks = A.smooth_cutoffs(p, x, [L], 0.5).cpu().numpy()
    out = A.smooth(p, x, [L], 0.5, 1.0).cpu().numpy().reshape(H, L)
    for h in range(H):
        assert ks[h] == 0 == O.energy_cutoff_bin(O.rdft(s[h].astype(np.float64)), 0.5, False)
        assert np.all(out[h] == out[h][0])
        assert abs(out[h][0] - s[h].astype(np.float64).mean()) <= 1e-6 * s[h].mean()


@pytest.mark.parametrize("L", LENGTHS)
@pytest.mark.parametrize("alpha", [1.0, 0.25])
def test_all_bins_kept_is_a_bitwise_copy(A, L, alpha):
    rng = np.random.default_rng(200 + L)
    H = 3
    s = _scores(rng, H, L)
    s[:, : L // 3] = s[:, :1]                        # a run of exactly equal values, as max pooling makes them
    p = A.Params(H, H, 128, 1)
    out = A.smooth(p, torch.from_numpy(s.reshape(-1)).cuda(), [L], 1.0, alpha).cpu().numpy().reshape(H, L)
    assert np.array_equal(out.view(np.uint32), s.view(np.uint32))
    # the taper does not matter once k* is the last bin
    pt = A.Params(H, H, 128, 1, taper_bins=5)
    out = A.smooth(pt, torch.from_numpy(s.reshape(-1)).cuda(), [L], 1.0, alpha).cpu().numpy().reshape(H, L)
    assert np.array_equal(out.view(np.uint32), s.view(np.uint32))


def _evict_small(A, L, *, cutoff, pool_mode=0, alpha=1.0, cutoff_mode=0, ratio=0.4):
    cfg = get_config(1, seqlen=L, n_items=2, n_spikes=8)
    items = [gen_item(cfg, i, seqlen=L) for i in range(cfg.n_items)]
    q = bf16_tensor(np.concatenate([it["q_win"].reshape(-1) for it in items]))
    k = bf16_tensor(np.concatenate([it["k"].reshape(-1) for it in items]))
    v = bf16_tensor(np.concatenate([it["v"].reshape(-1) for it in items]))
    w = gen_weights(cfg)
    p = A.Params(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.window, pool_kernel=cfg.pool_kernel, pool_mode=pool_mode,
                 floor_frac=cfg.floor_frac, cutoff_mode=cutoff_mode)
    out = A.evict(p, q, k, v, torch.from_numpy(w).cuda(), [L] * cfg.n_items, ratio, cutoff, alpha, alloc_scope=A.SCOPE_GLOBAL)
    torch.cuda.synchronize()
    b = out["budgets"].cpu().numpy(); cu_b = out["cu_budgets"].cpu().numpy(); idx = out["indices"].cpu().numpy()
    return cfg, items, p, (q, k), b, cu_b, idx


@pytest.mark.parametrize("L", [2048, 3000, 1100])
@pytest.mark.parametrize("cutoff_mode,cutoff", [(0, 0.0), (1, 1e-3)])   # a small energy ratio is reached by the DC bin alone
def test_evict_on_a_plateau_keeps_the_lowest_indices(A, L, cutoff_mode, cutoff):
    """k* = 0: every score of a head is the same value, so the index decides: the kept set is the first b - W
    positions plus the window, exactly what the oracle's full sort gives, on a power-of-two length and on
    chirp-z lengths alike."""
    cfg, items, p, _, b, cu_b, idx = _evict_small(A, L, cutoff=cutoff, cutoff_mode=cutoff_mode)
    W = cfg.window
    for g in range(len(b)):
        it, h = items[g // cfg.n_kv_heads], g % cfg.n_kv_heads
        s = O.score(bf16_bits_to_f64(it["q_win"][h * cfg.group:(h + 1) * cfg.group]), bf16_bits_to_f64(it["k"][h:h + 1]),
                    pool_kernel=cfg.pool_kernel)[0]
        s_hat = O.smooth(s, cutoff, 1.0) if cutoff_mode == 0 else O.smooth(s, 0.0, 1.0, energy_rho=cutoff)
        ref = O.select(s_hat, int(b[g]), W)
        assert np.array_equal(ref, np.concatenate([np.arange(b[g] - W), np.arange(L - W, L)]))
        assert np.array_equal(idx[cu_b[g]:cu_b[g + 1]], ref), g


@pytest.mark.parametrize("L", [2048, 3000])
def test_evict_max_pool_with_every_bin_kept(A, L):
    """Max pooling makes runs of exactly equal scores and cutoff = 1 keeps every bin: the filter is the identity,
    so the fused call must select exactly what audiokv_select makes of the pooled scores (bit for bit), and against
    the oracle's pooled scores any difference must sit at the threshold."""
    cfg, items, p, (q, k), b, cu_b, idx = _evict_small(A, L, cutoff=1.0, pool_mode=1)
    W = cfg.window
    lens = [L] * cfg.n_items
    s = A.score(p, q, k, lens)
    own = A.select(p, s, torch.from_numpy(b).cuda(), torch.from_numpy(cu_b).cuda(), lens, int(cu_b[-1])).cpu().numpy()
    assert np.array_equal(own, idx[:int(cu_b[-1])])
    agree = []
    for g in range(len(b)):
        it, h = items[g // cfg.n_kv_heads], g % cfg.n_kv_heads
        so = O.score(bf16_bits_to_f64(it["q_win"][h * cfg.group:(h + 1) * cfg.group]), bf16_bits_to_f64(it["k"][h:h + 1]),
                     pool_kernel=cfg.pool_kernel, pool_mode="max")[0]
        ref = O.select(so, int(b[g]), W)              # Eq. 19 with every weight 1 returns s itself
        mine = idx[cu_b[g]:cu_b[g + 1]]
        agree.append(len(np.intersect1d(mine, ref)) / len(ref))
        diff = np.setxor1d(mine, ref)
        if len(diff):
            thr = np.sort(so[:L - W])[::-1][int(b[g]) - W - 1]
            floor = 1e-3 * np.abs(so).max()
            tol = SCORE_RTOL * (np.maximum(np.abs(so[diff]), floor) + max(abs(thr), floor))
            assert np.all(np.abs(so[diff] - thr) <= tol), g
    assert np.mean(agree) >= 0.99, agree
