"""GPU parity of the spectral-smoothing variants: adaptive energy cutoff
(paper Sec. 3.3, Eqs. 14-16) and the cosine transition band after Eq. 17.

The energy rule lets floating point decide an integer (k*). The kernel's
spectrum is fp32, the oracle's float64, so where the cumulative energy passes
the target within the fp32 error of the spectrum both neighbours are valid
answers: the tests check that the kernel's k* satisfies the defining
inequalities up to that error, that it equals the oracle's k* whenever the
oracle's margin is clear, and then compare the filtered scores against the
oracle run with the kernel's k*.
"""
import numpy as np
import pytest
import torch

from oracle import audiokv_oracle as O
from workloads import bf16_bits_to_f64, gen_item, gen_weights, get_config

from gpu_util import SCORE_RTOL, bf16_tensor, rel_err

pytestmark = pytest.mark.gpu

ENERGY_RTOL = 2e-5      # fp32 spectrum: relative error of a cumulative energy


@pytest.fixture(scope="module")
def A():
    import paper_2604_06694_amd as A
    return A


def score_like(rng, H, L):
    """Positive, slowly varying importance profile plus spikes and noise, like pooled attention mass."""
    t = np.arange(L) / L
    out = np.empty((H, L), dtype=np.float32)
    for h in range(H):
        base = 0.02 + 0.01 * np.sin(2 * np.pi * (2 + h) * t + h) + 0.005 * np.cos(2 * np.pi * 17 * t)
        spikes = np.zeros(L)
        spikes[rng.integers(0, L, size=max(1, L // 200))] = rng.uniform(0.05, 0.5, size=max(1, L // 200))
        out[h] = (base + spikes + 0.004 * np.abs(rng.standard_normal(L))).astype(np.float32)
    return out


def check_kstar(F, rho, skip_dc, k_gpu):
    m2 = np.abs(F) ** 2
    first = 1 if skip_dc else 0
    if skip_dc:
        m2 = m2.copy(); m2[0] = 0.0
    E = np.cumsum(m2)
    target, tol = rho * E[-1], ENERGY_RTOL * E[-1]
    assert first <= k_gpu < len(F)
    assert E[k_gpu] >= target - tol, (k_gpu, E[k_gpu], target)
    if k_gpu > first:
        assert E[k_gpu - 1] < target + tol, (k_gpu, E[k_gpu - 1], target)
    k_ref = O.energy_cutoff_bin(F, rho, skip_dc)
    lo = E[k_ref - 1] if k_ref > first else -np.inf
    clear = (E[k_ref] - target > tol) and (target - lo > tol)
    if clear:
        assert k_gpu == k_ref
    return k_ref, clear


@pytest.mark.parametrize("T", [0, 1, 8, 100])
@pytest.mark.parametrize("L", [256, 1000, 2048, 8192])
def test_taper_parity(A, L, T):
    rng = np.random.default_rng(100 + L + T)
    H = 2
    s = score_like(rng, H, L)
    p = A.Params(H, H, 128, 1, taper_bins=T)
    for c, alpha in [(0.125, 1.0), (0.25, 0.5), (0.99, 1.0)]:
        out = A.smooth(p, torch.from_numpy(s.reshape(-1)).cuda(), [L], c, alpha).cpu().numpy().reshape(H, L)
        for h in range(H):
            ref = O.smooth(s[h].astype(np.float64), c, alpha, taper_bins=T)
            assert rel_err(out[h], ref) <= SCORE_RTOL
            assert np.abs(out[h] - ref).max() <= 1e-4 * np.abs(ref).max()
    if T == 0:      # the hard mask is the default path
        p0 = A.Params(H, H, 128, 1)
        a = A.smooth(p, torch.from_numpy(s.reshape(-1)).cuda(), [L], 0.125, 1.0)
        b = A.smooth(p0, torch.from_numpy(s.reshape(-1)).cuda(), [L], 0.125, 1.0)
        assert torch.equal(a, b)


def test_energy_cutoff_closed_form_spectrum(A):
    # DC of amplitude 1 plus cosines of amplitude 2 (bin 3) and 1 (bin 10): one-sided energies L^2, L^2, L^2/4
    for L in (64, 96):                      # LDS path and chirp-z path
        n = np.arange(L)
        s = (1.0 + 2.0 * np.cos(2 * np.pi * 3 * n / L) + 1.0 * np.cos(2 * np.pi * 10 * n / L)).astype(np.float32)
        t = torch.from_numpy(s).cuda()
        for mode, rho, want in [(A.CUTOFF_ENERGY, 0.40, 0), (A.CUTOFF_ENERGY, 0.50, 3), (A.CUTOFF_ENERGY, 0.88, 3),
                                (A.CUTOFF_ENERGY, 0.95, 10), (A.CUTOFF_ENERGY_NO_DC, 0.5, 3),
                                (A.CUTOFF_ENERGY_NO_DC, 0.9, 10)]:
            p = A.Params(1, 1, 128, 1, cutoff_mode=mode)
            ks = A.smooth_cutoffs(p, t, [L], rho).cpu().numpy()
            assert ks[0] == want, (L, mode, rho, ks)
        # fixed-fraction mode reports the fixed bin
        assert A.smooth_cutoffs(A.Params(1, 1, 128, 1), t, [L], 0.25).cpu().numpy()[0] == int(0.25 * (L // 2))
        # energy mode end to end: rho = 0.6 keeps DC and bin 3 only
        p = A.Params(1, 1, 128, 1, cutoff_mode=A.CUTOFF_ENERGY)
        out = A.smooth(p, t, [L], 0.6, 1.0).cpu().numpy()
        np.testing.assert_allclose(out, 1.0 + 2.0 * np.cos(2 * np.pi * 3 * n / L), atol=2e-5)


@pytest.mark.parametrize("L", [512, 1000, 4096, 5003, 8192])
def test_energy_cutoff_parity(A, L):
    rng = np.random.default_rng(200 + L)
    H = 3
    s = score_like(rng, H, L)
    t = torch.from_numpy(s.reshape(-1)).cuda()
    F = [O.rdft(s[h].astype(np.float64)) for h in range(H)]
    n_clear = n_total = 0
    for mode, skip, rhos in [(A.CUTOFF_ENERGY, False, (0.5, 0.9, 0.99, 0.999, 1.0)),
                             (A.CUTOFF_ENERGY_NO_DC, True, (0.3, 0.6, 0.9, 0.99))]:
        for rho in rhos:
            p = A.Params(H, H, 128, 1, cutoff_mode=mode, taper_bins=3 if rho == 0.9 else 0)
            ks = A.smooth_cutoffs(p, t, [L], rho).cpu().numpy()
            out = A.smooth(p, t, [L], rho, 1.0).cpu().numpy().reshape(H, L)
            for h in range(H):
                _, clear = check_kstar(F[h], rho, skip, int(ks[h]))
                if rho < 1.0:                 # at rho = 1 the target is the total itself: never clear
                    n_clear += clear; n_total += 1
                ref = O.smooth(s[h].astype(np.float64), 0.0, 1.0, k_star=int(ks[h]), taper_bins=p.taper_bins)
                assert rel_err(out[h], ref) <= SCORE_RTOL
    assert n_clear >= 0.75 * n_total         # the exact comparison is the rule, the tolerance the exception


def test_energy_cutoff_L32768_mixed_batch(A):
    rng = np.random.default_rng(9)
    lens = [32768, 3000]
    H = 2
    parts = [score_like(rng, H, L) for L in lens]
    flat = torch.from_numpy(np.concatenate([x.reshape(-1) for x in parts])).cuda()
    p = A.Params(H, H, 128, 1, cutoff_mode=A.CUTOFF_ENERGY_NO_DC, taper_bins=16)
    ks = A.smooth_cutoffs(p, flat, lens, 0.9).cpu().numpy()
    out = A.smooth(p, flat, lens, 0.9, 0.5).cpu().numpy()
    off = 0
    for i, (x, L) in enumerate(zip(parts, lens)):
        for h in range(H):
            if L <= 4096 or h == 0:          # the float64 spectrum of the long head costs seconds: one is enough
                check_kstar(O.rdft(x[h].astype(np.float64)), 0.9, True, int(ks[i * H + h]))
                ref = O.smooth(x[h].astype(np.float64), 0.0, 0.5, k_star=int(ks[i * H + h]), taper_bins=16)
                assert rel_err(out[off:off + L], ref) <= SCORE_RTOL
            off += L


def test_evict_with_energy_cutoff_and_taper_equals_composed(A):
    cfg = get_config(1)
    item = gen_item(cfg, 0)
    L = cfg.seqlen
    q = bf16_tensor(item["q_win"].reshape(-1)); k = bf16_tensor(item["k"].reshape(-1)); v = bf16_tensor(item["v"].reshape(-1))
    w = torch.from_numpy(gen_weights(cfg)).cuda()
    p = A.Params(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.window, pool_kernel=cfg.pool_kernel,
                 floor_frac=cfg.floor_frac, cutoff_mode=A.CUTOFF_ENERGY_NO_DC, taper_bins=4)
    rho = 0.9
    out = A.evict(p, q, k, v, w, [L], cfg.ratio, rho, 1.0, alloc_scope=A.SCOPE_GLOBAL)
    s = A.score(p, q, k, [L])
    b, cu = A.allocate(p, w, 1, cfg.n_kv_heads, [L], cfg.ratio)
    sh = A.smooth(p, s, [L], rho, 1.0)
    ks = A.smooth_cutoffs(p, s, [L], rho).cpu().numpy()
    idx = A.select(p, sh, b, cu, [L], out["total_rows"])
    ko, vo = A.compact(p, k, v, idx, cu, [L], out["total_rows"])
    torch.cuda.synchronize()
    assert torch.equal(idx, out["indices"][:out["total_rows"]])
    assert torch.equal(ko.view(torch.int16), out["k_out"][:out["total_rows"]].view(torch.int16))
    assert torch.equal(vo.view(torch.int16), out["v_out"][:out["total_rows"]].view(torch.int16))
    # the smoothed scores against the oracle's whole chain, cutoff forced to the kernel's (valid, checked) choice
    G = cfg.group
    sh_host = sh.cpu().numpy().reshape(cfg.n_kv_heads, L)
    for h in range(cfg.n_kv_heads):
        so = O.score(bf16_bits_to_f64(item["q_win"][h * G:(h + 1) * G]), bf16_bits_to_f64(item["k"][h:h + 1]),
                     pool_kernel=cfg.pool_kernel)[0]
        check_kstar(O.rdft(so), rho, True, int(ks[h]))
        ref = O.smooth(so, 0.0, 1.0, k_star=int(ks[h]), taper_bins=4)
        assert rel_err(sh_host[h], ref) <= SCORE_RTOL


def test_cutoff_argument_validation(A):
    t = torch.ones(64, device="cuda")
    with pytest.raises(A.AudioKVError) as e:
        A.smooth(A.Params(1, 1, 128, 1, cutoff_mode=A.CUTOFF_ENERGY), t, [64], 0.0, 1.0)      # rho must be > 0
    assert e.value.code == -1
    with pytest.raises(A.AudioKVError) as e:
        A.smooth(A.Params(1, 1, 128, 1, cutoff_mode=7), t, [64], 0.5, 1.0)
    assert e.value.code == -1
    with pytest.raises(A.AudioKVError) as e:
        A.smooth(A.Params(1, 1, 128, 1, taper_bins=-1), t, [64], 0.5, 1.0)
    assert e.value.code == -1
    # a constant signal has no energy outside DC: the variant without DC settles on its first bin
    ks = A.smooth_cutoffs(A.Params(1, 1, 128, 1, cutoff_mode=A.CUTOFF_ENERGY_NO_DC), t, [64], 0.9).cpu().numpy()
    assert 1 <= ks[0] <= 32


def test_alpha_zero_is_a_bitwise_copy_at_any_length(A):
    rng = np.random.default_rng(31)
    lens = [1000, 512, 37]
    H = 2
    flat = np.concatenate([score_like(rng, H, L).reshape(-1) for L in lens])
    t = torch.from_numpy(flat).cuda()
    for mode in (A.CUTOFF_FRACTION, A.CUTOFF_ENERGY):
        out = A.smooth(A.Params(H, H, 128, 1, cutoff_mode=mode, taper_bins=2), t, lens, 0.5, 0.0)
        assert torch.equal(out, t)


def test_evict_energy_cutoff_on_ragged_lengths(A):
    # lengths that are not powers of two, cutoff found from the spectrum: the filters are prepared beside the
    # score kernels for all bins; fused must equal composed
    rng = np.random.default_rng(32)
    H_q, H_kv, d, W = 8, 2, 64, 16
    lens = [700, 1024, 333]
    from workloads import f64_to_bf16_bits
    q = bf16_tensor(np.concatenate([f64_to_bf16_bits(rng.standard_normal((H_q, W, d))).reshape(-1) for _ in lens]))
    k = bf16_tensor(np.concatenate([f64_to_bf16_bits(rng.standard_normal((H_kv, L, d))).reshape(-1) for L in lens]))
    v = bf16_tensor(np.concatenate([f64_to_bf16_bits(rng.standard_normal((H_kv, L, d))).reshape(-1) for L in lens]))
    w = torch.rand(len(lens) * H_kv, device="cuda") + 0.1
    p = A.Params(H_q, H_kv, d, W, cutoff_mode=A.CUTOFF_ENERGY_NO_DC, taper_bins=3)
    out = A.evict(p, q, k, v, w, lens, 0.5, 0.8, 1.0, alloc_scope=A.SCOPE_ITEM)
    s = A.score(p, q, k, lens)
    b, cu = A.allocate(p, w, len(lens), H_kv, lens, 0.5)
    sh = A.smooth(p, s, lens, 0.8, 1.0)
    idx = A.select(p, sh, b, cu, lens, out["total_rows"])
    torch.cuda.synchronize()
    assert torch.equal(b, out["budgets"])
    assert torch.equal(idx, out["indices"][:out["total_rows"]])
    # and the smoothed scores against the oracle with the kernel's own (checked) cutoffs
    ks = A.smooth_cutoffs(p, s, lens, 0.8).cpu().numpy()
    s_host, sh_host = s.cpu().numpy(), sh.cpu().numpy()
    off = 0
    for i, L in enumerate(lens):
        for h in range(H_kv):
            x = s_host[off:off + L].astype(np.float64)
            check_kstar(O.rdft(x), 0.8, True, int(ks[i * H_kv + h]))
            ref = O.smooth(x, 0.0, 1.0, k_star=int(ks[i * H_kv + h]), taper_bins=3)
            assert rel_err(sh_host[off:off + L], ref) <= SCORE_RTOL
            off += L


@pytest.mark.parametrize("L", [4096, 16384, 32768])      # the few-heads path starts at 16384: below, both calls take one workgroup per head
@pytest.mark.parametrize("cutoff,alpha,T", [(0.125, 1.0, 0), (0.25, 0.5, 0), (0.0625, 1.0, 9), (0.9, 1.0, 0), (0.0, 1.0, 0)])
def test_few_heads_path_matches_one_workgroup_per_head_and_the_oracle(A, L, cutoff, alpha, T):
    """A call with few heads spreads every power-of-two head over several workgroups (interleaved sub-sequences);
    a call with many heads keeps one workgroup per head. Same definition, different order of the butterflies: the
    two agree to fp32 rounding, and both meet the oracle (the few-heads path also in place and with pooling fused
    into its loads, as audiokv_evict uses it)."""
    rng = np.random.default_rng(L + T)
    H = 4
    s = score_like(rng, H, L)
    p = A.Params(H, H, 128, 1, taper_bins=T)
    x = torch.from_numpy(s.reshape(-1)).cuda()
    few = A.smooth(p, x, [L], cutoff, alpha).cpu().numpy().reshape(H, L)
    n_rep = 20                                         # 80 heads: beyond the few-heads limit
    many = A.smooth(p, x.repeat(n_rep), [L] * n_rep, cutoff, alpha).cpu().numpy().reshape(n_rep, H, L)
    assert np.array_equal(many[0], many[-1])
    for h in range(H):
        ref = O.smooth(s[h].astype(np.float64), cutoff, alpha, taper_bins=T)
        scale = np.abs(ref).max()
        assert np.abs(few[h] - many[0][h]).max() <= 4e-6 * scale, (h, np.abs(few[h] - many[0][h]).max() / scale)
        assert rel_err(few[h], ref) <= SCORE_RTOL and np.abs(few[h] - ref).max() <= 2e-5 * scale
        assert rel_err(many[0][h], ref) <= SCORE_RTOL and np.abs(many[0][h] - ref).max() <= 2e-5 * scale
    inplace = x.clone()
    A.smooth(p, inplace, [L], cutoff, alpha, out=inplace)
    assert np.array_equal(inplace.cpu().numpy().reshape(H, L), few)
