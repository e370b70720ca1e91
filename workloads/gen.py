"""Seeded generators for the five synthetic audio-prefill workloads.

The paper evaluates on real audio-language-model prefills (speech recognition
and translation sets); neither those datasets nor the trained models are
available here, so every tensor is synthetic with the statistics that matter
for the eviction path:

* keys of an audio span follow an AR(1) process along the token axis
  (temporally continuous, like acoustic frames), optionally with a few
  "spike" tokens whose key vector is scaled up (heavy hitters);
* keys of a text span are i.i.d. N(0, 1);
* window queries and values are i.i.d. N(0, 1);
* per-KV-head criticality weights are Dirichlet draws (concentrated for the
  "few audio-critical heads" case).

Everything is drawn in float64 from numpy's PCG64 and then rounded to bf16
(round to nearest even); the bf16 bit patterns are what both the CPU oracle
and the GPU path consume, so parity isolates arithmetic, not input rounding.

Nothing in this file computes any part of the eviction method.
"""

from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass
from typing import Dict, Optional, Tuple

import numpy as np
from scipy.signal import lfilter


# --------------------------------------------------------------------------
# bf16 <-> float helpers (input preparation only)
# --------------------------------------------------------------------------

def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round finite float64 values to bf16 (nearest even); returns uint16 bit patterns."""
    u = np.array(x, dtype=np.float32).view(np.uint32)      # private copy, modified in place
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    u += lsb
    u += np.uint32(0x7FFF)                                  # finite inputs: cannot wrap
    u >>= np.uint32(16)
    return u.astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) exactly to float64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return u.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# Workload descriptions
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class Workload:
    """One synthetic configuration. An "item" is one (sequence, layer) pair."""

    index: int                      # 1-based configuration number
    name: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    window: int                     # W: observation window (last W queries)
    n_items: int                    # layers of one sequence, or sequences
    seqlen: Optional[int]           # uniform L; None when lengths are ragged
    len_range: Optional[Tuple[int, int]] = None   # ragged: log-uniform range
    ratio: float = 0.4              # retained-token ratio
    cutoff: float = 0.125           # SSS cutoff, fraction of spectrum bins
    alpha: float = 1.0              # SSS mixing coefficient
    pool_kernel: int = 7
    floor_frac: float = 0.1         # uniform floor r as a fraction (allocation)
    ar_rho: Optional[float] = 0.95  # None: per KV head ~ U(0.8, 0.99)
    n_spikes: int = 0
    spike_gain: float = 4.0
    text_tail: int = 0              # trailing tokens that are a text span
    text_frac_range: Optional[Tuple[float, float]] = None  # ragged text spans
    dirichlet_alpha: float = 1.0
    alloc_scope: str = "global"     # "global": one budget pool over all items
                                    # "item": each item (sequence) has its own
    repeats: int = 1                # how many times the batch is repeated

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def seed_tensors(self) -> int:
        return 1000 + self.index

    @property
    def seed_weights(self) -> int:
        return 2000 + self.index

    @property
    def seed_lengths(self) -> int:
        return 3000 + self.index


CONFIGS: Dict[int, Workload] = {
    1: Workload(index=1, name="cfg1_single_layer_L2048",
                n_q_heads=28, n_kv_heads=4, head_dim=128, window=32,
                n_items=1, seqlen=2048, n_spikes=16),
    2: Workload(index=2, name="cfg2_qwen25_omni_7b_L8192",
                n_q_heads=28, n_kv_heads=4, head_dim=128, window=32,
                n_items=28, seqlen=8192, n_spikes=16, text_tail=256),
    3: Workload(index=3, name="cfg3_long_audio_L32768",
                n_q_heads=28, n_kv_heads=4, head_dim=128, window=64,
                n_items=28, seqlen=32768, ar_rho=None),
    4: Workload(index=4, name="cfg4_qwen3_omni_30b_L16384",
                n_q_heads=32, n_kv_heads=4, head_dim=128, window=32,
                n_items=48, seqlen=16384, n_spikes=16, dirichlet_alpha=0.2),
    5: Workload(index=5, name="cfg5_ragged_batch8",
                n_q_heads=8, n_kv_heads=2, head_dim=256, window=32,
                n_items=8, seqlen=None, len_range=(2048, 32768), ratio=0.3,
                text_frac_range=(0.05, 0.3), alloc_scope="item", repeats=30),
}


def get_config(index: int, **overrides) -> Workload:
    """Return configuration `index` (1..5), optionally with fields replaced
    (tests shrink `seqlen` / `n_items`; the long-audio config sweeps `ratio`
    and `cutoff`)."""
    return dataclasses.replace(CONFIGS[index], **overrides)


# --------------------------------------------------------------------------
# Generators
# --------------------------------------------------------------------------

def _rng(*words: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(words))))


def gen_lengths(cfg: Workload) -> np.ndarray:
    """Per-item sequence lengths (int64). Ragged: floor(exp(U(ln lo, ln hi)))."""
    if cfg.seqlen is not None:
        return np.full(cfg.n_items, cfg.seqlen, dtype=np.int64)
    lo, hi = cfg.len_range
    u = _rng(cfg.seed_lengths).uniform(math.log(lo), math.log(hi), size=cfg.n_items)
    return np.floor(np.exp(u)).astype(np.int64)


def gen_weights(cfg: Workload) -> np.ndarray:
    """Per-KV-head criticality weights over all items, float32 [n_items*H_kv].

    Dirichlet(alpha) via normalised Gamma draws. With alloc_scope == "item"
    each item's heads are an independent Dirichlet draw."""
    rng = _rng(cfg.seed_weights)
    n = cfg.n_items * cfg.n_kv_heads
    if cfg.alloc_scope == "global":
        g = rng.gamma(cfg.dirichlet_alpha, size=n)
        w = g / g.sum()
    else:
        g = rng.gamma(cfg.dirichlet_alpha, size=(cfg.n_items, cfg.n_kv_heads))
        w = (g / g.sum(axis=1, keepdims=True)).reshape(n)
    return w.astype(np.float32)


def _ar1(rng: np.random.Generator, rho: np.ndarray, shape: Tuple[int, int, int]) -> np.ndarray:
    """AR(1) along axis 1 of [H, L, d]; rho has shape [H]. Stationary start."""
    H, L, d = shape
    eps = rng.standard_normal(shape)
    out = np.empty(shape, dtype=np.float64)
    for h in range(H):
        r = float(rho[h])
        e = eps[h]
        e[0] *= 1.0 / math.sqrt(1.0 - r * r)      # k_0 ~ N(0, 1/(1-rho^2))
        out[h] = lfilter([1.0], [1.0, -r], e, axis=0)
    return out


def gen_item(cfg: Workload, item: int, seqlen: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Tensors of one item, as bf16 bit patterns (uint16).

    Returns q_win [H_q, W, d], k [H_kv, L, d], v [H_kv, L, d].
    Each item has its own seed stream, so items can be generated independently.
    """
    L = int(seqlen if seqlen is not None else gen_lengths(cfg)[item])
    H, d, W = cfg.n_kv_heads, cfg.head_dim, cfg.window
    rng = _rng(cfg.seed_tensors, item)

    if cfg.ar_rho is None:
        rho = rng.uniform(0.8, 0.99, size=H)
    else:
        rho = np.full(H, cfg.ar_rho)
    k = _ar1(rng, rho, (H, L, d))

    if cfg.n_spikes > 0 and L - W > 0:
        n_sp = min(cfg.n_spikes, L - W)
        pos = rng.choice(L - W, size=n_sp, replace=False)
        k[:, pos, :] *= cfg.spike_gain

    n_text = 0
    if cfg.text_tail > 0:
        n_text = min(cfg.text_tail, L)
    elif cfg.text_frac_range is not None:
        lo, hi = cfg.text_frac_range
        n_text = int(math.floor(rng.uniform(lo, hi) * L))
    if n_text > 0:
        k[:, L - n_text:, :] = rng.standard_normal((H, n_text, d))

    q = rng.standard_normal((cfg.n_q_heads, W, d))
    v = rng.standard_normal((H, L, d))
    return {
        "q_win": f64_to_bf16_bits(q),
        "k": f64_to_bf16_bits(k),
        "v": f64_to_bf16_bits(v),
        "seqlen": L,
    }
