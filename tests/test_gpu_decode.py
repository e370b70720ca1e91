"""GPU parity of the decode-side consumer (single-query attention over the
packed, per-head-ragged compacted cache) against the float64 oracle, through
the C ABI. Tolerance: the floored relative error used for the scores (2e-3),
plus a much tighter absolute guard, since the arithmetic is fp32 throughout."""
import numpy as np
import pytest
import torch

from oracle import audiokv_oracle as O
from workloads import bf16_bits_to_f64, f64_to_bf16_bits, gen_item, gen_weights, get_config

from gpu_util import SCORE_RTOL, bf16_bits, bf16_tensor, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    import paper_2604_06694_amd as A
    return A


def run_case(A, rng, H_q, H_kv, d, budgets, n_items, *, k_scale=1.0, total_rows=None, scale=0.0):
    n_heads = n_items * H_kv
    assert len(budgets) == n_heads
    cu = np.concatenate([[0], np.cumsum(budgets)]).astype(np.int32)
    rows = int(cu[-1])
    kb = f64_to_bf16_bits(k_scale * rng.standard_normal((rows, d)))
    vb = f64_to_bf16_bits(rng.standard_normal((rows, d)))
    qb = f64_to_bf16_bits(rng.standard_normal((n_items, H_q, d)))
    p = A.Params(H_q, H_kv, d, 1, softmax_scale=scale)
    tr = rows if total_rows is None else total_rows
    out = A.decode_attend(p, bf16_tensor(qb.reshape(-1)), bf16_tensor(kb.reshape(-1)), bf16_tensor(vb.reshape(-1)),
                          torch.from_numpy(cu).cuda(), n_items, tr)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    kf, vf, qf = bf16_bits_to_f64(kb), bf16_bits_to_f64(vb), bf16_bits_to_f64(qb)
    sc = None if scale == 0.0 else float(np.float32(scale))
    for i in range(n_items):
        kr = [kf[cu[i * H_kv + h]:min(cu[i * H_kv + h + 1], tr)] for h in range(H_kv)]
        vr = [vf[cu[i * H_kv + h]:min(cu[i * H_kv + h + 1], tr)] for h in range(H_kv)]
        ref = O.decode_attend(qf[i], kr, vr, scale=sc)
        assert rel_err(out[i], ref) <= SCORE_RTOL, (i, rel_err(out[i], ref))
        assert np.abs(out[i] - ref).max() <= 1e-4 * max(np.abs(ref).max(), 1e-3)
    return out


@pytest.mark.parametrize("H_q,H_kv,d", [(28, 4, 128), (8, 8, 64), (8, 2, 256), (32, 2, 128), (32, 4, 128), (6, 2, 64),
                                         (32, 2, 256)])
def test_decode_ragged_budgets(A, H_q, H_kv, d):
    rng = np.random.default_rng(H_q * 1000 + d)
    n_items = 2
    pool = [1, 5, 16, 17, 511, 512, 513, 1500, 64, 1024]
    budgets = [int(pool[(3 * g + H_q) % len(pool)]) for g in range(n_items * H_kv)]
    run_case(A, rng, H_q, H_kv, d, budgets, n_items)


def test_decode_long_heads_and_peaked_softmax(A):
    rng = np.random.default_rng(5)
    # many chunks per head; large keys make the softmax sharp (logits up to ~ +-60)
    run_case(A, rng, 28, 4, 128, [32768, 13107, 6554, 700], 1, k_scale=4.0)
    run_case(A, rng, 8, 2, 256, [9000, 3000], 1, k_scale=0.05, scale=0.5)


def test_decode_one_very_long_head(A):
    # more chunks than the merge kernel's on-chip table holds: the path that sums straight from memory
    rng = np.random.default_rng(8)
    run_case(A, rng, 1, 1, 64, [1024 * 256 + 300], 1, k_scale=0.5)
    run_case(A, rng, 9, 1, 64, [512 * 256 + 7], 1, k_scale=0.5)          # 16-wide group padding: 512-row chunks


def test_decode_total_rows_bounds_the_reads_and_errors(A):
    rng = np.random.default_rng(6)
    run_case(A, rng, 8, 2, 128, [2000, 300], 1, total_rows=2100)      # rows at or past total_rows are not read
    p = A.Params(8, 2, 128, 1)
    q = torch.zeros(8 * 128, dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros(10 * 128, dtype=torch.bfloat16, device="cuda")
    cu = torch.tensor([0, 5, 10], dtype=torch.int32, device="cuda")
    with pytest.raises(A.AudioKVError) as e:
        A.decode_attend(p, q, kv, kv, cu, 1, 10, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -3
    with pytest.raises(A.AudioKVError) as e:
        A.decode_attend(A.Params(34, 2, 128, 1), q, kv, kv, cu, 1, 10)
    assert e.value.code == -2
    with pytest.raises(A.AudioKVError) as e:
        A.decode_attend(p, q, kv, kv, cu, 1, -1)
    assert e.value.code == -1
    # zero query: the mean of the retained rows; an empty head gives zeros
    v = torch.arange(10 * 128, dtype=torch.float32, device="cuda").remainder(7).to(torch.bfloat16)
    cu0 = torch.tensor([0, 10, 10], dtype=torch.int32, device="cuda")
    out = A.decode_attend(p, q, kv, v, cu0, 1, 10).cpu().numpy()
    want = v.float().view(10, 128).mean(0).cpu().numpy()
    np.testing.assert_allclose(out[0, :4], np.tile(want, (4, 1)), rtol=1e-6)
    assert np.all(out[0, 4:] == 0.0)


def test_decode_consumes_the_output_of_evict(A):
    cfg = get_config(1, n_items=2)
    items = [gen_item(cfg, i) for i in range(cfg.n_items)]
    L = cfg.seqlen
    q = bf16_tensor(np.concatenate([it["q_win"].reshape(-1) for it in items]))
    k = bf16_tensor(np.concatenate([it["k"].reshape(-1) for it in items]))
    v = bf16_tensor(np.concatenate([it["v"].reshape(-1) for it in items]))
    w = torch.from_numpy(gen_weights(cfg)).cuda()
    p = A.Params(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.window, pool_kernel=cfg.pool_kernel,
                 floor_frac=cfg.floor_frac)
    ev = A.evict(p, q, k, v, w, [L] * cfg.n_items, cfg.ratio, cfg.cutoff, cfg.alpha, alloc_scope=A.SCOPE_GLOBAL)
    # the next query: the last window row of every query head stands in for the first generated token's query
    qn_bits = np.stack([it["q_win"][:, -1, :] for it in items])              # [items, H_q, d]
    out = A.decode_attend(p, bf16_tensor(qn_bits.reshape(-1)), ev["k_out"], ev["v_out"], ev["cu_budgets"],
                          cfg.n_items, ev["total_rows"])
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    cu = ev["cu_budgets"].cpu().numpy(); idx = ev["indices"].cpu().numpy()
    for i, it in enumerate(items):
        kr, vr = [], []
        for h in range(cfg.n_kv_heads):
            g = i * cfg.n_kv_heads + h
            mine = idx[cu[g]:cu[g + 1]]
            kr.append(bf16_bits_to_f64(it["k"][h][mine])); vr.append(bf16_bits_to_f64(it["v"][h][mine]))
        ref = O.decode_attend(bf16_bits_to_f64(qn_bits[i]), kr, vr)
        assert rel_err(out[i], ref) <= SCORE_RTOL
        assert np.abs(out[i] - ref).max() <= 1e-4 * np.abs(ref).max()
