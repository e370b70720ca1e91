"""Writes oracle_tiny.json: the oracle's outputs on one tiny seeded case. Calls only oracle/ and workloads/."""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import audiokv_oracle as O  # noqa: E402
from workloads import bf16_bits_to_f64, gen_item, gen_weights, get_config  # noqa: E402


def compute():
    cfg = get_config(1, seqlen=96, window=8, n_spikes=4)
    it = gen_item(cfg, 0)
    w = gen_weights(cfg)
    b, cu = O.allocate(w.astype(np.float64), 96, cfg.ratio, window=8, floor_frac=float(np.float32(cfg.floor_frac)))
    s, s_hat, idx = O.evict_item(bf16_bits_to_f64(it["q_win"]), bf16_bits_to_f64(it["k"]), b, window=8,
                                 cutoff_frac=cfg.cutoff, alpha=cfg.alpha)
    return {
        "budgets": [int(x) for x in b],
        "score_head0_first8": [float(x) for x in s[0, :8]],
        "smoothed_head0_first8": [float(x) for x in s_hat[0, :8]],
        "score_sums": [float(x) for x in s.sum(axis=1)],
        "indices_head0": [int(x) for x in idx[0]],
    }


if __name__ == "__main__":
    with open(os.path.join(HERE, "oracle_tiny.json"), "w") as f:
        json.dump(compute(), f, indent=1)
