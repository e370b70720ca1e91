#!/usr/bin/env python3
"""Benchmark of the fused AudioKV eviction path (audiokv_evict) on one MI355X.

A "step" is one pass of the whole hot path (allocate, score, smooth, select,
compact) over one batch of synthetic audio-shaped input: all layers of one
configuration in one call. Inputs are resident in HBM before the timed region.
Prints one JSON line:
  value     = layer-tokens evicted per second: sum_items (L_i - n_keep_i) / step time
  roofline  = the dominant kernel's algorithmic rate against its bound, with the
              kernel duration measured by HIP events on the launch stream
  cpu_baseline = the float64 oracle timed on this host on one layer of the same workload
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (default 3: 28 layers x L=32768, W=64)")
    ap.add_argument("--ratio", type=float, default=None)
    ap.add_argument("--cutoff", type=float, default=None)
    ap.add_argument("--seqlen", type=int, default=None,
                    help="replace the sequence length of a fixed-length workload (e.g. 30000: a length that is not a power of two)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-layer", action="store_true", help="skip the one-launch-per-layer timing")
    ap.add_argument("--no-lse", action="store_true", help="skip the timing of the variant that is given the window's log-sum-exp")
    ap.add_argument("--no-decode", action="store_true", help="skip the timing of the decode-side consumer")
    ap.add_argument("--no-data-probe", action="store_true", help="skip the timing of the score kernels on all-zero keys")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the short runs of the other workloads")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (a kernel of known HBM traffic) so that a "
                         "rocprofv3 --pmc run of this command can scale FETCH_SIZE / WRITE_SIZE")
    return ap.parse_args()


def algorithmic_bytes(cfg, lens, ratio):
    """Bytes the method must move per step (one read of K for scoring, gather read + packed write of
    kept K/V rows, one write + one read of the score vector and of the indices)."""
    H, d = cfg.n_kv_heads, cfg.head_dim
    from paper_2604_06694_amd import n_keep
    per = {"score_read_k": 0, "compact": 0, "scores_rw": 0, "indices_rw": 0}
    for L in lens:
        nk = n_keep(ratio, L)
        per["score_read_k"] += L * H * d * 2
        per["compact"] += 4 * nk * H * d * 2
        per["scores_rw"] += 2 * 4 * L * H
        per["indices_rw"] += 2 * 4 * nk * H
    per["total"] = sum(per.values())
    return per


def measured_traffic(workload: str) -> dict:
    """HBM bytes per launch measured with rocprofv3 --pmc for this workload's default settings, as recorded
    (already scaled by the copy-kernel calibration) in profiles/<workload>_hbm_traffic.md; {} if absent."""
    short = {"cfg3_long_audio_L32768": "evict_cfg3_L32768_hbm_traffic.md",
             "cfg2_qwen25_omni_7b_L8192": "evict_cfg2_L8192_hbm_traffic.md",
             "cfg4_qwen3_omni_30b_L16384": "evict_cfg4_L16384_hbm_traffic.md"}.get(workload)
    path = os.path.join(ROOT, "profiles", short) if short else None
    out = {}
    if path and os.path.exists(path):
        for line in open(path):
            parts = line.split()
            if len(parts) == 4 and parts[0] == "traffic" and parts[2] == "=":
                out[parts[1]] = float(parts[3])
    return out


def cpu_baseline(cfg, sample_items, w, ratio, cutoff, alpha, budget_s=12.0):
    """The oracle as it stands, layer after layer of the same workload (all KV heads of each) until about
    `budget_s` seconds of CPU work are spent or the sample runs out."""
    import numpy as np
    from oracle import audiokv_oracle as O
    from workloads import bf16_bits_to_f64
    t0 = time.perf_counter()
    done, evicted = 0, 0
    for i, it in enumerate(sample_items):
        L = it["seqlen"]
        b, _ = O.allocate(w[i * cfg.n_kv_heads:(i + 1) * cfg.n_kv_heads].astype(np.float64), L, ratio, window=cfg.window,
                          floor_frac=float(np.float32(cfg.floor_frac)))
        _, _, idx = O.evict_item(bf16_bits_to_f64(it["q_win"]), bf16_bits_to_f64(it["k"]), b, window=cfg.window,
                                 pool_kernel=cfg.pool_kernel, cutoff_frac=cutoff, alpha=alpha)
        O.compact(it["k"], it["v"], idx)
        done += 1
        evicted += L - O.n_keep_of(ratio, L)
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([int(x.get("num_threads", 1)) for x in threadpool_info()] or [1])
    except Exception:
        blas_threads = None
    return {"value": evicted / dt, "unit": "layer-tokens evicted/s", "cores": len(os.sched_getaffinity(0)),
            "blas_threads": blas_threads, "kind": "oracle", "seconds": dt,
            "sample": f"{done} of {cfg.n_items} items of the same workload (all {cfg.n_kv_heads} KV heads of each, "
                      f"per-item budget pools); float64 numpy, BLAS threads as configured by the host"}


def load_workload(cfg, dev):
    """Synthetic inputs of one workload, resident on the device; the first items are kept on the host for the oracle."""
    import numpy as np
    import torch
    from workloads import gen_item, gen_lengths, gen_weights
    lens = [int(x) for x in gen_lengths(cfg)]
    with cf.ThreadPoolExecutor(max_workers=8) as ex:
        items = list(ex.map(lambda i: gen_item(cfg, i, seqlen=lens[i]), range(cfg.n_items)))

    def to_dev(key):
        flat = np.concatenate([it[key].reshape(-1) for it in items])
        return torch.from_numpy(flat.view(np.int16)).to(dev).view(torch.bfloat16)

    q, k, v = to_dev("q_win"), to_dev("k"), to_dev("v")
    w_host = gen_weights(cfg)
    return {"lens": lens, "q": q, "k": k, "v": v, "w_host": w_host, "w": torch.from_numpy(w_host).to(dev),
            "sample_items": items[:8]}


def time_config(A, cfg, data, steps, warmup, dev):
    """Step time of the fused call on one workload, the duration of each of its kernels (HIP events recorded by the
    library on the launch stream), the algorithmic rates and the dominant kernel against its bound."""
    import numpy as np
    import torch
    lens, q, k, v, w = data["lens"], data["q"], data["k"], data["v"], data["w"]
    p = A.Params(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.window, pool_kernel=cfg.pool_kernel,
                 floor_frac=cfg.floor_frac)
    scope = A.SCOPE_GLOBAL if cfg.alloc_scope == "global" else A.SCOPE_ITEM
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device=dev)
    ws = torch.empty(A.workspace_bytes(p, lens), dtype=torch.uint8, device=dev)
    outs: dict = {}

    def step():
        A.evict(p, q, k, v, w, lens, cfg.ratio, cfg.cutoff, cfg.alpha, alloc_scope=scope, cu_seqlens=cu,
                workspace=ws, outputs=outs)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps

    # the same steps again with HIP events recorded between the kernels on the launch stream
    A.profile_enable(True)
    acc = {n: 0.0 for n in A.PROFILE_STAGES}
    n_prof = max(3, min(steps, 10))
    for _ in range(n_prof):
        # the events of the last of three back-to-back steps are read: a step that follows an idle GPU runs at a
        # higher clock than one inside a stream of steps, which is what the timed loop above and a profiler see
        step()
        step()
        step()
        for n, ms in A.profile_read().items():
            acc[n] += ms
    A.profile_enable(False)
    stage_ms = {n: acc[n] / n_prof for n in acc}

    tokens = sum(lens)
    kept = sum(A.n_keep(cfg.ratio, L) for L in lens)
    ab = algorithmic_bytes(cfg, lens, cfg.ratio)
    score_flops = sum(2.0 * cfg.n_q_heads * cfg.window * L * cfg.head_dim for L in lens)
    dominant = max(stage_ms, key=stage_ms.get)
    dom_s = stage_ms[dominant] * 1e-3
    if dominant in ("score_sweep1", "score_sweep2"):
        # each sweep performs the whole contraction once
        roof = {"bound": "mfma", "achieved": score_flops / dom_s / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "kernel": dominant, "kernel_ms": stage_ms[dominant], "traffic": None,
                "hbm_GBs_of_this_kernel": ab["score_read_k"] / dom_s / 1e9}
    else:
        key = {"compact": "compact", "pool_smooth": "scores_rw", "select": "indices_rw", "allocate": "indices_rw"}[dominant]
        roof = {"bound": "hbm", "achieved": ab[key] / dom_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "kernel": dominant, "kernel_ms": stage_ms[dominant], "traffic": None}
        if dominant != "compact":
            roof["note"] = ("a chain of small per-head kernels, bound by launch and barrier latency rather than by bandwidth; "
                            "with stage timing on, work that otherwise runs beside the score sweeps on the helper stream "
                            "(chirp-z filter preparation for lengths that are not powers of two) is in line and counted here")
    roof["frac"] = roof["achieved"] / roof["peak"]
    return {"dt": dt, "stage_ms": stage_ms, "tokens": tokens, "kept": kept, "ab": ab, "score_flops": score_flops,
            "roof": roof, "p": p, "scope": scope, "cu": cu, "ws": ws, "outs": outs, "step": step}


def other_config_line(A, index, steps, warmup, dev, **over):
    """Compact record of another workload: the same measurement, fewer fields."""
    import torch
    from workloads import get_config
    cfg = get_config(index, **over)
    data = load_workload(cfg, dev)
    m = time_config(A, cfg, data, steps, warmup, dev)
    line = {"workload": cfg.name, "ratio": cfg.ratio, "ms_per_step": m["dt"] * 1e3,
            "value": (m["tokens"] - m["kept"]) / m["dt"], "hbm_frac": m["ab"]["total"] / m["dt"] / 1e9 / HBM_PEAK_GBS,
            "stage_ms": {n: round(x, 4) for n, x in m["stage_ms"].items()},
            "dominant": {"kernel": m["roof"]["kernel"], "bound": m["roof"]["bound"], "frac": m["roof"]["frac"],
                         "hbm_GBs_of_this_kernel": m["roof"].get("hbm_GBs_of_this_kernel")}}
    if "note" in m["roof"]:
        line["dominant"]["note"] = m["roof"]["note"]
    del data, m
    torch.cuda.empty_cache()
    return line


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2604_06694_amd as A
    from workloads import get_config

    over = {}
    if args.ratio is not None:
        over["ratio"] = args.ratio
    if args.cutoff is not None:
        over["cutoff"] = args.cutoff
    if args.seqlen is not None:
        over["seqlen"] = args.seqlen
    cfg = get_config(args.config, **over)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    data = load_workload(cfg, dev)
    lens, q, k, v, w, w_host, sample_items = (data["lens"], data["q"], data["k"], data["v"], data["w"], data["w_host"],
                                              data["sample_items"])

    if args.pmc_calibration:
        cal_src = torch.empty(256 * 2**20, dtype=torch.uint8, device=dev).fill_(1)
        cal_dst = torch.empty_like(cal_src)
        cal_dst.copy_(cal_src)
        torch.cuda.synchronize()
        del cal_src, cal_dst

    m = time_config(A, cfg, data, args.steps, args.warmup, dev)
    dt, stage_ms, p, scope, cu, ws, outs, step = (m["dt"], m["stage_ms"], m["p"], m["scope"], m["cu"], m["ws"], m["outs"],
                                                  m["step"])
    tokens, kept, ab, score_flops, roof = m["tokens"], m["kept"], m["ab"], m["score_flops"], m["roof"]
    evicted = tokens - kept
    score_exps = sum(float(cfg.n_q_heads * cfg.window * L) for L in lens)
    if args.ratio is None and args.cutoff is None and args.seqlen is None:
        roof["traffic"] = measured_traffic(cfg.name).get(roof["kernel"])

    res = {
        "metric": "prefill KV tokens evicted/sec per layer (1 GPU) + achieved HBM GB/s fraction",
        "value": evicted / dt,
        "unit": "layer-tokens evicted/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": dt * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": cfg.name, "n_items": cfg.n_items, "n_q_heads": cfg.n_q_heads,
                   "n_kv_heads": cfg.n_kv_heads, "head_dim": cfg.head_dim, "window": cfg.window,
                   "seqlen": lens[0] if len(set(lens)) == 1 else lens, "ratio": cfg.ratio, "cutoff": cfg.cutoff,
                   "alpha": cfg.alpha, "pool_kernel": cfg.pool_kernel, "alloc_scope": cfg.alloc_scope},
        "tokens_processed_per_s": tokens / dt,
        "whole_path": {"algorithmic_bytes": ab["total"], "GBs": ab["total"] / dt / 1e9,
                       "hbm_frac": ab["total"] / dt / 1e9 / HBM_PEAK_GBS, "us_per_layer": dt * 1e6 / cfg.n_items},
        "stage_ms": stage_ms,
        "score": {"TFLOPs_both_sweeps": 2 * score_flops / ((stage_ms["score_sweep1"] + stage_ms["score_sweep2"]) * 1e-3) / 1e12,
                  "exp_per_s_both_sweeps": 2 * score_exps / ((stage_ms["score_sweep1"] + stage_ms["score_sweep2"]) * 1e-3)},
        "compact_GBs": ab["compact"] / (stage_ms["compact"] * 1e-3) / 1e9,
        "roofline": roof,
    }
    # the same work as one launch per layer (28 calls, each layer its own budget pool): what a framework that evicts
    # layer by layer during prefill would issue; `value` above is the all-layers-batched call
    if cfg.seqlen is not None and cfg.n_items > 1 and not args.no_per_layer:
        L0 = lens[0]
        per_q = cfg.n_q_heads * cfg.window * cfg.head_dim
        per_kv = cfg.n_kv_heads * L0 * cfg.head_dim
        rows1 = A.n_keep(cfg.ratio, L0) * cfg.n_kv_heads
        ws1 = torch.empty(A.workspace_bytes(p, [L0]), dtype=torch.uint8, device=dev)
        cu1 = torch.tensor([0, L0], dtype=torch.int32, device=dev)
        o1 = {"k_out": outs["k_out"][:rows1], "v_out": outs["v_out"][:rows1], "indices": outs["indices"][:rows1],
              "budgets": outs["budgets"][:cfg.n_kv_heads], "cu_budgets": outs["cu_budgets"][:cfg.n_kv_heads + 1]}

        def layer_steps():
            for i in range(cfg.n_items):
                A.evict(p, q[i * per_q:(i + 1) * per_q], k[i * per_kv:(i + 1) * per_kv], v[i * per_kv:(i + 1) * per_kv],
                        w[i * cfg.n_kv_heads:(i + 1) * cfg.n_kv_heads], [L0], cfg.ratio, cfg.cutoff, cfg.alpha,
                        alloc_scope=A.SCOPE_ITEM, cu_seqlens=cu1, workspace=ws1, outputs=o1)
        layer_steps()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n_rep = max(2, args.steps // 4)
        for _ in range(n_rep):
            layer_steps()
        torch.cuda.synchronize()
        dt_layer = (time.perf_counter() - t0) / n_rep
        res["one_launch_per_layer"] = {"ms_per_step": dt_layer * 1e3, "value": evicted / dt_layer,
                                       "note": "28 audiokv_evict calls of one layer each, per-layer budget pools; "
                                               "outputs of every layer written to the same buffers"}
        # the same 28 calls issued round-robin on three streams (own workspace and output buffers per stream):
        # the one-workgroup-per-head stages of one layer then overlap the score kernels of the next
        n_str = 3
        streams = [torch.cuda.Stream() for _ in range(n_str)]
        slot_ws = [torch.empty_like(ws1) for _ in range(n_str)]
        slot_out = [{key: torch.empty_like(val) for key, val in o1.items() if torch.is_tensor(val) and key != "workspace"}
                    for _ in range(n_str)]

        def layer_steps_streams():
            for i in range(cfg.n_items):
                j = i % n_str
                with torch.cuda.stream(streams[j]):
                    A.evict(p, q[i * per_q:(i + 1) * per_q], k[i * per_kv:(i + 1) * per_kv], v[i * per_kv:(i + 1) * per_kv],
                            w[i * cfg.n_kv_heads:(i + 1) * cfg.n_kv_heads], [L0], cfg.ratio, cfg.cutoff, cfg.alpha,
                            alloc_scope=A.SCOPE_ITEM, cu_seqlens=cu1, workspace=slot_ws[j], outputs=slot_out[j])
        torch.cuda.synchronize()
        layer_steps_streams()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_rep):
            layer_steps_streams()
        torch.cuda.synchronize()
        dt_ls = (time.perf_counter() - t0) / n_rep
        res["one_launch_per_layer"]["three_streams_ms_per_step"] = dt_ls * 1e3
        res["one_launch_per_layer"]["three_streams_value"] = evicted / dt_ls
        # the last layers of the one-stream run and of the three-stream run must agree bit for bit
        last = (cfg.n_items - 1) % n_str
        res["one_launch_per_layer"]["streams_match"] = bool(torch.equal(slot_out[last]["indices"], o1["indices"]))
        del slot_ws, slot_out
        step()                                   # restore the batched outputs for what follows
        torch.cuda.synchronize()
    if not args.no_lse:
        # variant, never `value`: the window rows' log-sum-exp handed over by the prefill attention kernel (made here
        # with torch outside the timed region), so that the first pass over K is not needed
        lse_parts = []
        off_q = off_k = 0
        scale = 1.0 / (cfg.head_dim ** 0.5)
        for L_i in lens:
            qi = q[off_q:off_q + cfg.n_q_heads * cfg.window * cfg.head_dim].view(cfg.n_kv_heads, cfg.group * cfg.window, cfg.head_dim).float()
            ki = k[off_k:off_k + cfg.n_kv_heads * L_i * cfg.head_dim].view(cfg.n_kv_heads, L_i, cfg.head_dim).float()
            z = torch.bmm(qi, ki.transpose(1, 2)) * scale                                  # [H_kv, G*W, L]
            pos = torch.arange(L_i, device=dev)[None, None, :]
            last = (L_i - cfg.window + torch.arange(cfg.window, device=dev)).repeat(cfg.group)[None, :, None]
            z = z.masked_fill(pos > last, float("-inf"))
            lse_parts.append(torch.logsumexp(z, dim=2).reshape(-1))
            del qi, ki, z
            off_q += cfg.n_q_heads * cfg.window * cfg.head_dim
            off_k += cfg.n_kv_heads * L_i * cfg.head_dim
        lse = torch.cat(lse_parts).contiguous()

        def lstep():
            A.evict(p, q, k, v, w, lens, cfg.ratio, cfg.cutoff, cfg.alpha, alloc_scope=scope, cu_seqlens=cu,
                    workspace=ws, outputs=outs, lse=lse)
        for _ in range(3):
            lstep()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            lstep()
        torch.cuda.synchronize()
        dt_lse = (time.perf_counter() - t0) / args.steps
        res["with_prefill_lse"] = {"ms_per_step": dt_lse * 1e3, "value": evicted / dt_lse,
                                   "hbm_frac": ab["total"] / dt_lse / 1e9 / HBM_PEAK_GBS,
                                   "note": "audiokv_evict_lse: softmax denominators of the window rows supplied by the "
                                           "caller, one pass over K instead of two; a variant, not the headline path"}
        step()
        torch.cuda.synchronize()
    if not args.no_decode:
        # the step after the path: one decoding step (one new query per head) over the compacted cache just written
        qd = torch.randn(cfg.n_items * cfg.n_q_heads * cfg.head_dim, device=dev).to(torch.bfloat16)
        n_rows = kept * cfg.n_kv_heads
        dws = torch.empty(A.decode_workspace_bytes(p, cfg.n_items, n_rows), dtype=torch.uint8, device=dev)
        dout = torch.empty((cfg.n_items, cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device=dev)

        def dstep():
            A.decode_attend(p, qd, outs["k_out"], outs["v_out"], outs["cu_budgets"], cfg.n_items, n_rows,
                            out=dout, workspace=dws)
        for _ in range(3):
            dstep()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            dstep()
        e1.record()
        torch.cuda.synchronize()
        d_ms = e0.elapsed_time(e1) / args.steps
        d_bytes = 2 * kept * cfg.n_kv_heads * cfg.head_dim * 2          # every retained K and V row once
        res["decode_consumer"] = {"ms_per_step": d_ms, "algorithmic_bytes": d_bytes, "GBs": d_bytes / d_ms / 1e6,
                                  "hbm_frac": d_bytes / d_ms / 1e6 / HBM_PEAK_GBS,
                                  "what": "single-query attention of all query heads over the compacted cache of all layers"}
    if not args.no_data_probe:
        # The score sweeps run the same instruction stream whatever the key values are; their duration is not the
        # same: with all-zero keys (nothing toggles in the multipliers) they finish sooner. The ratio says how far the
        # kernel time on real data is set by the chip's power management rather than by issue slots.
        probe_out = torch.empty(sum(lens) * cfg.n_kv_heads, dtype=torch.float32, device=dev)

        def timed_score(kk):
            for _ in range(3):
                A.score(p, q, kk, lens, cu_seqlens=cu, workspace=ws, out=probe_out)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                A.score(p, q, kk, lens, cu_seqlens=cu, workspace=ws, out=probe_out)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / 10
        real_ms = timed_score(k)
        kz = torch.zeros_like(k)
        zero_ms = timed_score(kz)
        del kz, probe_out
        res["score_time_vs_key_data"] = {"real_keys_ms": real_ms, "all_zero_keys_ms": zero_ms, "ratio": zero_ms / real_ms,
                                         "what": "audiokv_score (both sweeps + pooling) on the workload's keys and on "
                                                 "all-zero keys: identical instruction streams, different data"}
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg, sample_items, w_host, cfg.ratio, cfg.cutoff, cfg.alpha)
    if not args.no_other_configs and args.config == 3 and not over:
        # every other workload, measured the same way in the same process (fewer steps); `value` stays on cfg 3
        n_s, n_w = max(5, args.steps // 2), 3
        res["other_configs"] = {
            "cfg3_ratio0.2": other_config_line(A, 3, n_s, n_w, dev, ratio=0.2),
            "cfg1": other_config_line(A, 1, n_s, n_w, dev),
            "cfg2": other_config_line(A, 2, n_s, n_w, dev),
            "cfg4": other_config_line(A, 4, n_s, n_w, dev),
            "cfg5": other_config_line(A, 5, n_s, n_w, dev),
        }
    print(json.dumps(res))


if __name__ == "__main__":
    main()
