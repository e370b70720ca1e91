"""Per-stage GPU-vs-oracle parity through the C ABI (ctypes binding).

Integer/byte stages (allocate, select, compact) are bit-exact; floating stages
(score, smooth) meet the 2e-3 floored relative tolerance."""
import numpy as np
import pytest
import torch

from oracle import audiokv_oracle as O
from workloads import bf16_bits_to_f64, f64_to_bf16_bits, gen_item, gen_weights, get_config

from gpu_util import SCORE_RTOL, bf16_bits, bf16_tensor, pack_items_head_major, pack_items_token_major, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    import paper_2604_06694_amd as A
    return A


def _rand_items(rng, H_q, H_kv, W, d, lens, k_scale=1.0):
    items = []
    for L in lens:
        items.append({
            "q_win": f64_to_bf16_bits(rng.standard_normal((H_q, W, d))),
            "k": f64_to_bf16_bits(rng.standard_normal((H_kv, L, d)) * k_scale),
            "v": f64_to_bf16_bits(rng.standard_normal((H_kv, L, d))),
            "seqlen": L,
        })
    return items


# ------------------------------------------------------------------ compact

@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("layout", [0, 1])
def test_compact_bit_exact(A, d, layout):
    rng = np.random.default_rng(d + layout)
    H_kv, lens = 3, [37, 300, 1]
    items = _rand_items(rng, H_kv, H_kv, 1, d, lens)
    p = A.Params(H_kv, H_kv, d, 1, kv_layout=layout)
    idx_lists, budgets = [], []
    for it in items:
        for h in range(H_kv):
            b = int(rng.integers(1, it["seqlen"] + 1))
            idx_lists.append(np.sort(rng.choice(it["seqlen"], size=b, replace=False)))
            budgets.append(b)
    cu_b = np.concatenate([[0], np.cumsum(budgets)]).astype(np.int32)
    total = int(cu_b[-1])
    pack = pack_items_head_major if layout == 0 else pack_items_token_major
    k = bf16_tensor(pack(items, "k")); v = bf16_tensor(pack(items, "v"))
    idx = torch.from_numpy(np.concatenate(idx_lists).astype(np.int32)).cuda()
    ko, vo = A.compact(p, k, v, idx, torch.from_numpy(cu_b).cuda(), lens, total)
    torch.cuda.synchronize()
    ref_k, ref_v = [], []
    for i, it in enumerate(items):
        rk, rv = O.compact(it["k"], it["v"], idx_lists[i * H_kv:(i + 1) * H_kv])
        ref_k.append(rk); ref_v.append(rv)
    assert np.array_equal(bf16_bits(ko), np.concatenate(ref_k))
    assert np.array_equal(bf16_bits(vo), np.concatenate(ref_v))


# ----------------------------------------------------------------- allocate

def _alloc_case(A, S, n_seg, hps, lens, ratio, W, beta, group=1):
    p = A.Params(4 * group, 4, 128, W, floor_frac=beta)
    w = torch.from_numpy(np.asarray(S, dtype=np.float32)).cuda()
    b, cu = A.allocate(p, w, n_seg, hps, lens, ratio, weight_group=group)
    torch.cuda.synchronize()
    b, cu = b.cpu().numpy(), cu.cpu().numpy()
    S32 = np.asarray(S, dtype=np.float32).astype(np.float64).reshape(n_seg, hps * group)
    ref_b = []
    for s in range(n_seg):
        rb, _ = O.allocate(S32[s], lens[s], ratio, window=W, floor_frac=float(np.float32(beta)), group=group)
        ref_b.append(rb)
    ref_b = np.concatenate(ref_b)
    assert np.array_equal(b, ref_b)
    assert np.array_equal(cu, np.concatenate([[0], np.cumsum(ref_b)]))
    return b


@pytest.mark.parametrize("cfg_idx", [1, 2, 3, 4, 5])
def test_allocate_configs_bit_exact(A, cfg_idx):
    from workloads import gen_lengths
    cfg = get_config(cfg_idx)
    S = gen_weights(cfg)
    lens = [int(x) for x in gen_lengths(cfg)]
    if cfg.alloc_scope == "global":
        b = _alloc_case(A, S, 1, cfg.n_items * cfg.n_kv_heads, lens[:1], cfg.ratio, cfg.window, cfg.floor_frac)
        assert int(b.sum()) == O.n_keep_of(cfg.ratio, lens[0]) * len(S)
    else:
        _alloc_case(A, S, cfg.n_items, cfg.n_kv_heads, lens, cfg.ratio, cfg.window, cfg.floor_frac)


def test_allocate_random_and_edge_cases(A):
    rng = np.random.default_rng(77)
    for _ in range(40):
        n = int(rng.integers(1, 300))
        L = int(rng.integers(64, 40000))
        W = int(rng.integers(0, 33))
        ratio = float(rng.uniform(0.05, 1.0))
        if O.n_keep_of(ratio, L) < W:
            continue
        a = float(rng.choice([0.05, 0.2, 1.0, 5.0]))
        S = rng.gamma(a, size=n)
        S = S / S.sum() if S.sum() > 0 else S
        _alloc_case(A, S, 1, n, [L], ratio, W, float(rng.choice([0.0, 0.1, 0.5, 1.0])))
    _alloc_case(A, np.zeros(9), 1, 9, [500], 0.4, 8, 0.1)                  # all-zero weights
    _alloc_case(A, np.ones(28), 1, 28, [8192], 0.4, 32, 0.1)               # uniform
    _alloc_case(A, [0.97, 0.01, 0.01, 0.01], 1, 4, [1000], 0.5, 10, 0.0)   # cap + re-spread
    _alloc_case(A, [0.6, 0.35, 0.03, 0.02], 1, 4, [100], 0.7, 0, 0.0)      # two rounds of capping
    _alloc_case(A, np.ones(4), 1, 4, [10], 0.25, 0, 0.0)                   # ties in the remainders
    _alloc_case(A, rng.gamma(1.0, size=56), 2, 4, [2048, 777], 0.4, 32, 0.1, group=7)   # query-head weights


# ------------------------------------------------------------------- select

def _select_case(A, scores_per_head, lens, H_kv, budgets, W):
    p = A.Params(H_kv, H_kv, 128, W)
    flat = np.concatenate([np.asarray(s, dtype=np.float32) for s in scores_per_head])
    cu_b = np.concatenate([[0], np.cumsum(budgets)]).astype(np.int32)
    total = int(cu_b[-1])
    idx = A.select(p, torch.from_numpy(flat).cuda(), torch.tensor(budgets, dtype=torch.int32).cuda(),
                   torch.from_numpy(cu_b).cuda(), lens, total)
    torch.cuda.synchronize()
    idx = idx.cpu().numpy()
    for g, s in enumerate(scores_per_head):
        ref = O.select(np.asarray(s, dtype=np.float32), budgets[g], W)
        got = idx[cu_b[g]:cu_b[g + 1]]
        assert np.array_equal(got, ref), f"head {g}"


def test_select_bit_exact_random_and_ties(A):
    rng = np.random.default_rng(5)
    for L, W in [(8, 2), (33, 1), (64, 8), (1000, 32), (2048, 32), (5000, 0), (32768, 64)]:
        H_kv = 3
        heads, budgets = [], []
        for h in range(H_kv):
            s = rng.standard_normal(L).astype(np.float32)
            if h == 1:
                s = np.round(s * 4) / 4           # heavy ties
            if h == 2:
                s[: L // 2] = 0.0
                s[::7] = -0.0                      # signed zeros
            heads.append(s)
            budgets.append(int(rng.integers(max(W, 1), L + 1)))
        _select_case(A, heads, [L], H_kv, budgets, W)


def test_select_adversarial(A):
    L, W = 4096, 32
    const = np.full(L, 1.25, dtype=np.float32)
    ramp = np.arange(L, dtype=np.float32)
    neg = -np.abs(np.random.default_rng(1).standard_normal(L)).astype(np.float32)
    _select_case(A, [const, ramp, neg, const], [L], 4, [1000, 1000, 1000, L], W)       # pure tie-break; b = L
    _select_case(A, [const, ramp, neg, ramp[::-1].copy()], [L], 4, [W, W + 1, L - 1, 77], W)   # b = W: window only


@pytest.mark.parametrize("L,W", [(12352, 64), (16384, 32), (30000, 1), (32768, 64)])
def test_select_long_heads_every_distribution(A, L, W):
    """Long heads bracket the threshold between two pivots taken from a sample of the keys; the result must not depend
    on how good the sample is. Distributions that defeat it (sorted, periodic in the register layout, alternating with
    the sampled threads, plateaus, few distinct values, a narrow range, half zeros) and budgets at both extremes."""
    rng = np.random.default_rng(L + W)
    x = rng.standard_normal(L)
    t = np.arange(L)
    dists = [x, np.exp(3 * x), np.sort(x), np.sort(x)[::-1], np.round(x * 2) / 2, np.full(L, 0.5),
             np.sin(t * 2 * np.pi / 1024) + 1e-3 * x, (t % 2) * 100.0 + x, 1.0 + 1e-5 * x,
             np.where(rng.random(L) < 0.5, 0.0, np.abs(x)), -np.exp(x)]
    heads = [np.ascontiguousarray(s, dtype=np.float32) for s in dists]
    lo = max(W, 1)
    for budgets in ([int(rng.integers(lo, L + 1)) for _ in heads], [int(0.4 * L)] * len(heads),
                    [lo + 3] * len(heads), [L - 5] * len(heads)):
        _select_case(A, heads, [L], len(heads), budgets, W)


def test_select_ragged_items(A):
    rng = np.random.default_rng(9)
    lens = [100, 2500, 33]
    H_kv = 2
    heads, budgets = [], []
    for L in lens:
        for h in range(H_kv):
            heads.append(rng.standard_normal(L).astype(np.float32))
            budgets.append(int(rng.integers(8, L + 1)))
    _select_case(A, heads, lens, H_kv, budgets, 8)


# ------------------------------------------------------------------- smooth

@pytest.mark.parametrize("L", [4, 8, 64, 256, 2048, 8192])
@pytest.mark.parametrize("c,alpha", [(0.125, 1.0), (0.25, 0.5), (1.0, 1.0), (0.0, 1.0), (0.0625, 0.0)])
def test_smooth_parity(A, L, c, alpha):
    rng = np.random.default_rng(L)
    H_kv = 3
    p = A.Params(H_kv, H_kv, 128, 1)
    s = (np.abs(rng.standard_normal((H_kv, L))) + 0.1 * rng.standard_normal((H_kv, L))).astype(np.float32)
    out = A.smooth(p, torch.from_numpy(s.reshape(-1)).cuda(), [L], c, alpha)
    torch.cuda.synchronize()
    out = out.cpu().numpy().reshape(H_kv, L)
    for h in range(H_kv):
        ref = O.smooth(s[h].astype(np.float64), c, alpha)
        assert rel_err(out[h], ref) <= SCORE_RTOL
        if alpha == 0.0:
            assert np.array_equal(out[h], s[h])            # bitwise copy
    # the kernel is far more accurate than the tolerance: guard against silent degradation
    if alpha > 0:
        ref = O.smooth(s[0].astype(np.float64), c, alpha)
        assert np.abs(out[0] - ref).max() <= 2e-5 * np.abs(ref).max()


def test_smooth_L32768_and_in_place(A):
    rng = np.random.default_rng(3)
    L, H_kv = 32768, 2
    p = A.Params(H_kv, H_kv, 128, 1)
    s = np.abs(rng.standard_normal((H_kv, L))).astype(np.float32)
    t = torch.from_numpy(s.reshape(-1)).cuda()
    out = A.smooth(p, t, [L], 1.0 / 16, 1.0, out=t)        # in place
    torch.cuda.synchronize()
    out = out.cpu().numpy().reshape(H_kv, L)
    ref = O.smooth(s[1].astype(np.float64), 1.0 / 16, 1.0)
    assert rel_err(out[1], ref) <= SCORE_RTOL


@pytest.mark.parametrize("L", [5, 33, 100, 1000, 2049, 5003, 12345, 20000, 32767])
def test_smooth_arbitrary_length(A, L):
    # transform length is exactly L (no zero padding): chirp-z path
    rng = np.random.default_rng(L)
    H_kv = 2
    p = A.Params(H_kv, H_kv, 128, 1)
    s = (np.abs(rng.standard_normal((H_kv, L))) + 0.05 * rng.standard_normal((H_kv, L))).astype(np.float32)
    for c, alpha in [(0.125, 1.0), (0.3, 0.5)]:
        out = A.smooth(p, torch.from_numpy(s.reshape(-1)).cuda(), [L], c, alpha)
        torch.cuda.synchronize()
        out = out.cpu().numpy().reshape(H_kv, L)
        for h in range(H_kv):
            ref = O.smooth(s[h].astype(np.float64), c, alpha)
            assert rel_err(out[h], ref) <= SCORE_RTOL
            assert np.abs(out[h] - ref).max() <= 1e-4 * np.abs(ref).max()


def test_smooth_mixed_lengths_in_one_call(A):
    rng = np.random.default_rng(12)
    lens = [1024, 777, 4096, 3001]
    H_kv = 2
    p = A.Params(H_kv, H_kv, 128, 1)
    parts = [np.abs(rng.standard_normal((H_kv, L))).astype(np.float32) for L in lens]
    flat = np.concatenate([x.reshape(-1) for x in parts])
    out = A.smooth(p, torch.from_numpy(flat).cuda(), lens, 0.125, 1.0).cpu().numpy()
    off = 0
    for x, L in zip(parts, lens):
        for h in range(H_kv):
            ref = O.smooth(x[h].astype(np.float64), 0.125, 1.0)
            assert rel_err(out[off:off + L], ref) <= SCORE_RTOL
            off += L


# -------------------------------------------------------------------- score

def _score_case(A, H_q, H_kv, W, d, lens, *, causal=1, layout=0, pool_kernel=7, pool_mode=0, k_scale=1.0, seed=0):
    rng = np.random.default_rng(seed)
    items = _rand_items(rng, H_q, H_kv, W, d, lens, k_scale)
    p = A.Params(H_q, H_kv, d, W, pool_kernel=pool_kernel, pool_mode=pool_mode, causal=causal, kv_layout=layout)
    pack = pack_items_head_major if layout == 0 else pack_items_token_major
    q = bf16_tensor(np.concatenate([it["q_win"].reshape(-1) for it in items]))
    k = bf16_tensor(pack(items, "k"))
    s = A.score(p, q, k, lens)
    torch.cuda.synchronize()
    s = s.cpu().numpy()
    off = 0
    worst = 0.0
    for it in items:
        L = it["seqlen"]
        ref = O.score(bf16_bits_to_f64(it["q_win"]), bf16_bits_to_f64(it["k"]), pool_kernel=pool_kernel,
                      pool_mode="avg" if pool_mode == 0 else "max", causal=bool(causal))
        got = s[off:off + H_kv * L].reshape(H_kv, L)
        off += H_kv * L
        for h in range(H_kv):
            worst = max(worst, rel_err(got[h], ref[h]))
    assert worst <= SCORE_RTOL, worst
    return worst


@pytest.mark.parametrize("H_q,H_kv,W,d", [(28, 4, 32, 128), (32, 4, 32, 128), (8, 2, 32, 256), (4, 2, 8, 64),
                                          (14, 2, 64, 128), (2, 2, 16, 128), (3, 1, 5, 64),
                                          (16, 2, 64, 128), (16, 2, 64, 64), (9, 1, 32, 128), (8, 1, 33, 64),
                                          (8, 1, 32, 256), (9, 1, 64, 128), (15, 1, 32, 64)])
def test_score_parity_shapes(A, H_q, H_kv, W, d):
    _score_case(A, H_q, H_kv, W, d, [1000], seed=H_q + W)


@pytest.mark.parametrize("L", [32, 33, 64, 129, 257, 2048])
def test_score_parity_lengths(A, L):
    _score_case(A, 28, 4, 32, 128, [L], seed=L)


def test_score_ragged_batch_and_layouts(A):
    _score_case(A, 8, 2, 32, 256, [2100, 40, 777], seed=1)
    _score_case(A, 8, 2, 16, 128, [300, 1025], layout=1, seed=2)


def test_score_variants(A):
    _score_case(A, 8, 2, 16, 128, [500], causal=0, seed=3)
    _score_case(A, 8, 2, 16, 128, [500], pool_kernel=1, seed=4)
    _score_case(A, 8, 2, 16, 128, [500], pool_kernel=5, pool_mode=1, seed=5)
    _score_case(A, 8, 2, 16, 128, [500], k_scale=6.0, seed=6)      # peaky softmax: large logits


@pytest.mark.parametrize("shape", ["ramp", "step", "descent"])
def test_score_logits_far_from_first_block(A, shape):
    """Logits that climb (or fall) by far more than 64 binary orders after the first keys of a row: the row sums
    are kept relative to a reference taken from the first block a lane meets, and this is the case in which that
    reference has to be raised (ramp: several times; step: a single jump that overflows exp2; descent: never)."""
    rng = np.random.default_rng(11)
    H_q, H_kv, W, d, L = 14, 2, 32, 128, 3000
    t = {"ramp": np.linspace(-4.0, 4.0, L), "step": np.where(np.arange(L) < L // 2, -4.0, 4.0),
         "descent": np.linspace(4.0, -4.0, L)}[shape]
    kk = t[None, :, None] * np.ones((H_kv, 1, d)) + 0.25 * rng.standard_normal((H_kv, L, d))
    qq = rng.uniform(0.5, 2.0, size=(H_q, W, 1)) * np.ones((1, 1, d)) + 0.25 * rng.standard_normal((H_q, W, d))
    qq[1::3] *= -1.0                                   # some query heads see the ramp the other way round
    item = {"q_win": f64_to_bf16_bits(qq), "k": f64_to_bf16_bits(kk), "seqlen": L}
    p = A.Params(H_q, H_kv, d, W)
    s = A.score(p, bf16_tensor(item["q_win"].reshape(-1)), bf16_tensor(item["k"].reshape(-1)), [L])
    torch.cuda.synchronize()
    s = s.cpu().numpy().reshape(H_kv, L)
    assert np.isfinite(s).all()
    ref = O.score(bf16_bits_to_f64(item["q_win"]), bf16_bits_to_f64(item["k"]))
    for h in range(H_kv):
        assert rel_err(s[h], ref[h]) <= SCORE_RTOL, (shape, h, rel_err(s[h], ref[h]))


def test_score_config1_workload(A):
    cfg = get_config(1)
    it = gen_item(cfg, 0)
    p = A.Params(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.window)
    s = A.score(p, bf16_tensor(it["q_win"].reshape(-1)), bf16_tensor(it["k"].reshape(-1)), [cfg.seqlen])
    torch.cuda.synchronize()
    s = s.cpu().numpy().reshape(cfg.n_kv_heads, cfg.seqlen)
    ref = O.score(bf16_bits_to_f64(it["q_win"]), bf16_bits_to_f64(it["k"]))
    for h in range(cfg.n_kv_heads):
        assert rel_err(s[h], ref[h]) <= SCORE_RTOL
