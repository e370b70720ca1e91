"""Heads longer than 32768 tokens: selection streams the scores instead of holding the keys in registers, and the
spectral smoothing runs its chirp-z transforms (up to 262144 points) on global memory. Same parity bars as the
short-sequence tests; the limit (131072 tokens for smoothing) is an error code, not a crash."""
import numpy as np
import pytest
import torch

from oracle import audiokv_oracle as O
from workloads import bf16_bits_to_f64, f64_to_bf16_bits

from gpu_util import SCORE_RTOL, bf16_bits, bf16_tensor, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    import paper_2604_06694_amd as A
    return A


def _select(A, heads, lens, H_kv, budgets, W):
    p = A.Params(H_kv, H_kv, 128, W)
    flat = np.concatenate([np.asarray(s, dtype=np.float32) for s in heads])
    cu_b = np.concatenate([[0], np.cumsum(budgets)]).astype(np.int32)
    idx = A.select(p, torch.from_numpy(flat).cuda(), torch.tensor(budgets, dtype=torch.int32).cuda(),
                   torch.from_numpy(cu_b).cuda(), lens, int(cu_b[-1]))
    torch.cuda.synchronize()
    idx = idx.cpu().numpy()
    for g, s in enumerate(heads):
        ref = O.select(np.asarray(s, dtype=np.float32), budgets[g], W)
        assert np.array_equal(idx[cu_b[g]:cu_b[g + 1]], ref), f"head {g}"


def test_select_long_heads_bit_exact(A):
    rng = np.random.default_rng(21)
    L, W = 100003, 64
    a = rng.standard_normal(L).astype(np.float32)
    ties = (np.round(rng.standard_normal(L) * 3) / 3).astype(np.float32)        # long runs of equal keys
    zeros = np.zeros(L, dtype=np.float32); zeros[::5] = -0.0; zeros[L // 3:L // 3 + 10] = 1.0
    const = np.full(L, -2.5, dtype=np.float32)
    _select(A, [a, ties, zeros, const], [L], 4, [40000, 33333, 50000, 70001], W)
    _select(A, [a, ties, zeros, const], [L], 4, [W, W + 1, L, L - 1], W)        # window only, one more, everything


def test_select_long_and_short_heads_in_one_call(A):
    rng = np.random.default_rng(22)
    lens = [3000, 70000, 40]
    heads, budgets = [], []
    for L in lens:
        for h in range(2):
            heads.append(rng.standard_normal(L).astype(np.float32))
            budgets.append(int(rng.integers(8, L + 1)))
    _select(A, heads, lens, 2, budgets, 8)


@pytest.mark.parametrize("L,c", [(40000, 0.125), (65536, 0.0625), (100003, 0.05), (131072, 0.03125)])
def test_smooth_long_lengths(A, L, c):
    rng = np.random.default_rng(L)
    p = A.Params(1, 1, 128, 1)
    s = (np.abs(rng.standard_normal(L)) + 0.05 * rng.standard_normal(L)).astype(np.float32)
    for alpha in (1.0, 0.5):
        out = A.smooth(p, torch.from_numpy(s).cuda(), [L], c, alpha)
        torch.cuda.synchronize()
        out = out.cpu().numpy()
        ref = O.smooth(s.astype(np.float64), c, alpha)
        assert rel_err(out, ref) <= SCORE_RTOL
        assert np.abs(out - ref).max() <= 1e-4 * np.abs(ref).max()


def test_smooth_long_with_energy_cutoff_and_mixed_batch(A):
    """All bins are wanted when the cutoff comes from the spectrum: the largest transform for the length. A short
    head of the ordinary multi-workgroup size rides in the same call."""
    rng = np.random.default_rng(31)
    lens = [50000, 6000]
    p = A.Params(1, 1, 128, 1, cutoff_mode=A.CUTOFF_ENERGY_NO_DC)
    parts = [(np.abs(rng.standard_normal(L)) + 0.05 * rng.standard_normal(L)).astype(np.float32) for L in lens]
    flat = torch.from_numpy(np.concatenate(parts)).cuda()
    ks = A.smooth_cutoffs(p, flat, lens, 0.6).cpu().numpy()
    out = A.smooth(p, flat, lens, 0.6, 1.0).cpu().numpy()
    off = 0
    for i, L in enumerate(lens):
        ref = O.smooth(parts[i].astype(np.float64), 0.0, 1.0, k_star=int(ks[i]))
        assert rel_err(out[off:off + L], ref) <= SCORE_RTOL
        F = np.fft.rfft(parts[i].astype(np.float64))
        k_ref = O.energy_cutoff_bin(F, 0.6, True)
        assert abs(int(ks[i]) - k_ref) <= 1        # fp32 spectrum against float64 at a flat crossing
        off += L
    p2 = A.Params(1, 1, 128, 1)
    out2 = A.smooth(p2, flat, lens, 0.1, 1.0).cpu().numpy()
    off = 0
    for i, L in enumerate(lens):
        assert rel_err(out2[off:off + L], O.smooth(parts[i].astype(np.float64), 0.1, 1.0)) <= SCORE_RTOL
        off += L


def test_evict_long_sequence_end_to_end(A):
    H_q, H_kv, d, W, L, ratio, c = 4, 2, 64, 16, 50001, 0.3, 0.125
    rng = np.random.default_rng(77)
    qb = f64_to_bf16_bits(rng.standard_normal((H_q, W, d)))
    kb = f64_to_bf16_bits(rng.standard_normal((H_kv, L, d)) * 1.5)
    vb = f64_to_bf16_bits(rng.standard_normal((H_kv, L, d)))
    w = np.array([0.7, 0.3], dtype=np.float32)
    p = A.Params(H_q, H_kv, d, W)
    out = A.evict(p, bf16_tensor(qb.reshape(-1)), bf16_tensor(kb.reshape(-1)), bf16_tensor(vb.reshape(-1)),
                  torch.from_numpy(w).cuda(), [L], ratio, c, 1.0, alloc_scope=0)
    torch.cuda.synchronize()
    budgets = out["budgets"].cpu().numpy(); cu_b = out["cu_budgets"].cpu().numpy(); idx = out["indices"].cpu().numpy()
    ref_b, _ = O.allocate(w.astype(np.float64), L, ratio, window=W, floor_frac=float(np.float32(0.1)))
    assert np.array_equal(budgets, ref_b)
    ko, vo = bf16_bits(out["k_out"]), bf16_bits(out["v_out"])
    G = H_q // H_kv
    for h in range(H_kv):
        mine = idx[cu_b[h]:cu_b[h + 1]]
        assert np.array_equal(ko[cu_b[h]:cu_b[h + 1]], kb[h][mine]) and np.array_equal(vo[cu_b[h]:cu_b[h + 1]], vb[h][mine])
        s = O.score(bf16_bits_to_f64(qb[h * G:(h + 1) * G]), bf16_bits_to_f64(kb[h:h + 1]), pool_kernel=7)[0]
        s_hat = O.smooth(s, c, 1.0)
        ref = O.select(s_hat, int(ref_b[h]), W)
        agree = len(np.intersect1d(mine, ref)) / len(ref)
        assert agree >= 0.999, agree
        diff = np.setxor1d(mine, ref)
        if len(diff):
            thr = np.sort(s_hat[:L - W])[::-1][int(ref_b[h]) - W - 1]
            assert np.all(np.abs(s_hat[diff] - thr) <= SCORE_RTOL * np.abs(s_hat).max())


def test_length_beyond_the_smoothing_limit_is_refused(A):
    p = A.Params(1, 1, 128, 1)
    with pytest.raises(A.AudioKVError) as e:
        A.smooth(p, torch.zeros(131073, device="cuda"), [131073], 0.125, 1.0)
    assert e.value.code == -2
