"""K/V passed by explicit strides (audiokv_params.kv_stride_*): a padded prefill cache [B][H_kv][L_max][d], and a
token-major slab with extra heads between the ones used, against the same data in the packed default layout.
Score values match bit for bit, and so do budgets, indices and the compacted rows of the fused call: the strides
change where a row is read from and nothing else."""
import dataclasses

import numpy as np
import pytest
import torch

from workloads import f64_to_bf16_bits

from gpu_util import bf16_tensor

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    import paper_2604_06694_amd as A
    return A


def _packed_and_padded(rng, H_q, H_kv, d, W, lens, L_max, *, token_major=False, extra_heads=0, row_pad=0):
    q = bf16_tensor(np.concatenate([f64_to_bf16_bits(rng.standard_normal((H_q, W, d))).reshape(-1) for _ in lens]))
    ks = [f64_to_bf16_bits(rng.standard_normal((H_kv, L, d)) * 1.5) for L in lens]
    vs = [f64_to_bf16_bits(rng.standard_normal((H_kv, L, d))) for L in lens]
    packed_k = bf16_tensor(np.concatenate([x.reshape(-1) for x in ks]))
    packed_v = bf16_tensor(np.concatenate([x.reshape(-1) for x in vs]))
    B, Hs, ds = len(lens), H_kv + extra_heads, d + row_pad
    junk = lambda shape: f64_to_bf16_bits(rng.standard_normal(shape) * 50.0)      # padding that must never be read
    if token_major:
        big_k, big_v = junk((B, L_max, Hs, ds)), junk((B, L_max, Hs, ds))
        for i, L in enumerate(lens):
            big_k[i, :L, :H_kv, :d] = ks[i].transpose(1, 0, 2)
            big_v[i, :L, :H_kv, :d] = vs[i].transpose(1, 0, 2)
        strides = dict(kv_stride_item=L_max * Hs * ds, kv_stride_head=ds, kv_stride_tok=Hs * ds)
    else:
        big_k, big_v = junk((B, Hs, L_max, ds)), junk((B, Hs, L_max, ds))
        for i, L in enumerate(lens):
            big_k[i, :H_kv, :L, :d] = ks[i]
            big_v[i, :H_kv, :L, :d] = vs[i]
        strides = dict(kv_stride_item=Hs * L_max * ds, kv_stride_head=L_max * ds, kv_stride_tok=ds)
    return q, packed_k, packed_v, bf16_tensor(big_k.reshape(-1)), bf16_tensor(big_v.reshape(-1)), strides


@pytest.mark.parametrize("case", [
    dict(H_q=28, H_kv=4, d=128, W=32, lens=[1500, 4096, 700], L_max=4096),                                  # padded [B][H][L_max][d]
    dict(H_q=8, H_kv=2, d=256, W=32, lens=[2048, 900], L_max=2304, token_major=True, extra_heads=1),        # heads interleaved per token
    dict(H_q=8, H_kv=2, d=64, W=16, lens=[1000], L_max=1000, row_pad=8),                                    # rows 16 bytes apart beyond d
])
def test_strided_cache_matches_packed(A, case):
    rng = np.random.default_rng(len(case["lens"]) + case["d"])
    H_q, H_kv, d, W, lens = case["H_q"], case["H_kv"], case["d"], case["W"], case["lens"]
    q, pk, pv, bk, bv, strides = _packed_and_padded(rng, H_q, H_kv, d, W, lens, case["L_max"],
                                                    token_major=case.get("token_major", False),
                                                    extra_heads=case.get("extra_heads", 0), row_pad=case.get("row_pad", 0))
    p = A.Params(H_q, H_kv, d, W)
    ps = dataclasses.replace(p, **strides)
    s_ref = A.score(p, q, pk, lens)
    s_str = A.score(ps, q, bk, lens)
    torch.cuda.synchronize()
    assert torch.equal(s_ref.view(torch.int32), s_str.view(torch.int32))
    w = torch.from_numpy(rng.gamma(1.0, size=len(lens) * H_kv).astype(np.float32)).cuda()
    ref = A.evict(p, q, pk, pv, w, lens, 0.4, 0.125, 1.0, alloc_scope=A.SCOPE_ITEM)
    out = A.evict(ps, q, bk, bv, w, lens, 0.4, 0.125, 1.0, alloc_scope=A.SCOPE_ITEM)
    torch.cuda.synchronize()
    rows = ref["total_rows"]
    for name in ("budgets", "cu_budgets"):
        assert torch.equal(out[name], ref[name]), name
    assert torch.equal(out["indices"][:rows], ref["indices"][:rows])
    assert torch.equal(out["k_out"][:rows].view(torch.int16), ref["k_out"][:rows].view(torch.int16))
    assert torch.equal(out["v_out"][:rows].view(torch.int16), ref["v_out"][:rows].view(torch.int16))
    # the stand-alone gather, too
    ko, vo = A.compact(ps, bk, bv, ref["indices"][:rows], ref["cu_budgets"], lens, rows)
    torch.cuda.synchronize()
    assert torch.equal(ko.view(torch.int16), ref["k_out"][:rows].view(torch.int16))
    assert torch.equal(vo.view(torch.int16), ref["v_out"][:rows].view(torch.int16))
