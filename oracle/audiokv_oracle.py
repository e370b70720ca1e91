"""Float64 CPU oracle for the AudioKV prefill-time KV-cache eviction path.

TEST INFRASTRUCTURE ONLY. This module is the slow, plain reference that the
HIP kernels are checked against. It shares no code with the GPU path, is never
imported by the product package, and must only be used from tests, the smoke
check and the CPU-baseline leg of the benchmark.

What it computes (paper: AudioKV, Sec. 3):

  score     observation-window importance: the last W queries of every query
            head attend to all L keys of their KV head; row softmax; sum over
            window rows and over the query heads of the GQA group; local
            pooling. (Sec. 3.3: the per-head importance sequence s in R^L,
            given there as attention averaged over a window of recent
            queries; Sec. 1/2: local pooling of SnapKV-style scores.)
  allocate  head-wise budgets b = w + r + B_score * S / sum(S)  (Sec. 3.1,
            Eq. 1) with the floor of Sec. 3.2, Eq. 12, made to sum exactly to
            the total by a largest-remainder top-up.
  smooth    Spectral Score Smoothing (Sec. 3.3, Eqs. 13, 17-20): real DFT,
            hard low-pass mask at bin k*, inverse real DFT of length L,
            residual mix with coefficient alpha. Optional adaptive
            energy-based cutoff (Eqs. 14-16).
  select    keep the b_h highest-scoring tokens of each head (top-K selection,
            Sec. 1, Solution 2), forced observation window included, ties to
            the lower index, indices ascending.
  compact   gather the retained K/V rows into a packed cache (Sec. 1: the
            cache keeps only salient tokens; Sec. 4.6: memory follows the
            retention ratio).
  decode_attend  what the next decoding step does with that cache: each query
            head attends to the retained rows of its KV head only (plain
            scaled-dot-product attention over b_h rows; the definition itself).

The method is a heuristic pipeline rather than a fast route to a textbook
quantity, so each function takes the steps in the paper's order, in float64
(decode_attend alone has a plain definition, and is that definition).
The DFTs are written as direct sums (no FFT library); because every bin above
k* is zeroed, the direct sums cost only O(L * k*).

Readings taken where the paper is silent (each also listed in the design
notes): softmax scale 1/sqrt(d); causal mask inside the window; *sum* (not
mean) over window and group; average pooling with zero padding and divisor k;
fixed-fraction cutoff k* = floor(c * (n_bins - 1)); unnormalised forward DFT
and 1/L inverse; floor r = floor(beta * (n_keep - W)); water-filling cap at L
tokens per head; largest-remainder integerisation; n_keep = floor(ratio*L+.5).

Parity status: no function here can be pinned to a number printed in the
paper (it prints none for this path). They are pinned by closed forms,
invariants, brute force on tiny inputs and library cross-checks in
tests/test_oracle_*.py. The value of the uniform floor fraction beta, and the
shape and width of the cosine taper, are "parity unpinned".
"""

from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

__all__ = [
    "window_attention",
    "pool",
    "score",
    "n_keep_of",
    "allocate",
    "cutoff_bin",
    "energy_cutoff_bin",
    "rdft",
    "irdft",
    "smooth",
    "select",
    "compact",
    "decode_attend",
    "evict_item",
]


# ---------------------------------------------------------------------------
# Stage 1: observation-window importance score
# ---------------------------------------------------------------------------

def window_attention(q_win: np.ndarray, k: np.ndarray, *, causal: bool = True,
                     scale: Optional[float] = None) -> np.ndarray:
    """Summed window attention per KV head (Sec. 3.3, the sequence s before pooling).

    q_win [H_q, W, d]: queries of the last W prompt positions (position of row
                       i is L - W + i).
    k     [H_kv, L, d]
    returns raw [H_kv, L]:  raw[h, j] = sum over query heads q of group(h) and
    window rows i of softmax_j(scale * <q_win[q, i], k[h, j]>), where with
    `causal` a row only sees keys j <= L - W + i.
    """
    q_win = np.asarray(q_win, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    H_q, W, d = q_win.shape
    H_kv, L, d2 = k.shape
    assert d == d2 and H_q % H_kv == 0 and 1 <= W <= L
    G = H_q // H_kv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    raw = np.zeros((H_kv, L), dtype=np.float64)
    cols = np.arange(L)
    for h in range(H_kv):
        for g in range(G):
            qh = q_win[h * G + g]                      # [W, d]
            z = (qh @ k[h].T) * scale                  # [W, L]
            if causal:
                last_visible = (L - W) + np.arange(W)  # per row
                z = np.where(cols[None, :] <= last_visible[:, None], z, -np.inf)
            z = z - z.max(axis=1, keepdims=True)
            e = np.exp(z)
            p = e / e.sum(axis=1, keepdims=True)       # rows sum to 1
            raw[h] += p.sum(axis=0)
    return raw


def pool(x: np.ndarray, kernel: int, mode: str = "avg") -> np.ndarray:
    """Local pooling along the last axis, stride 1, centred odd kernel.

    avg: zeros outside [0, L), divisor always `kernel`.
    max: -inf outside [0, L).
    """
    x = np.asarray(x, dtype=np.float64)
    assert kernel >= 1 and kernel % 2 == 1
    if kernel == 1:
        return x.copy()
    half = kernel // 2
    L = x.shape[-1]
    pad_val = 0.0 if mode == "avg" else -np.inf
    pad = [(0, 0)] * (x.ndim - 1) + [(half, half)]
    xp = np.pad(x, pad, constant_values=pad_val)
    if mode == "avg":
        acc = np.zeros_like(x)
        for t in range(kernel):
            acc = acc + xp[..., t:t + L]
        return acc / kernel
    if mode == "max":
        acc = np.full_like(x, -np.inf)
        for t in range(kernel):
            acc = np.maximum(acc, xp[..., t:t + L])
        return acc
    raise ValueError(mode)


def score(q_win: np.ndarray, k: np.ndarray, *, pool_kernel: int = 7,
          pool_mode: str = "avg", causal: bool = True,
          scale: Optional[float] = None) -> np.ndarray:
    """Stage 1 complete: pooled window-attention importance, [H_kv, L]."""
    return pool(window_attention(q_win, k, causal=causal, scale=scale),
                pool_kernel, pool_mode)


# ---------------------------------------------------------------------------
# Stage 2: head-wise budget allocation
# ---------------------------------------------------------------------------

def n_keep_of(ratio: float, L: int) -> int:
    """Tokens kept per head on average: round-half-up of ratio * L in float64."""
    return int(math.floor(float(ratio) * float(L) + 0.5))


def allocate(weights: Sequence[float], L: int, ratio: float, *, window: int,
             floor_frac: float = 0.1, group: int = 1) -> Tuple[np.ndarray, np.ndarray]:
    """Per-head integer budgets (Sec. 3.1 Eq. 1; Sec. 3.2 Eq. 12).

    weights: criticality S >= 0; if group > 1 they are per query head and are
             summed inside each GQA group first (the cache is per KV head).
    Returns (b [n], cu_b [n+1]) with sum(b) == n_keep * n exactly,
    window + r <= b_h <= L, where
        n_keep = round(ratio * L), r = floor(floor_frac * (n_keep - window)),
        b_h = window + r + (share of B_score = n*(n_keep - window - r)
              proportional to S_h, capped so b_h <= L, floored, leftover units
              handed out by largest fractional part, ties to the lower index).
    """
    S = np.asarray(weights, dtype=np.float64)
    if group > 1:
        S = S.reshape(-1, group)
        Ssum = np.zeros(S.shape[0], dtype=np.float64)
        for g in range(group):                 # index order, like any plain loop
            Ssum = Ssum + S[:, g]
        S = Ssum
    n = S.shape[0]
    assert n >= 1 and np.all(S >= 0.0)
    nk = n_keep_of(ratio, L)
    assert window <= nk <= L
    r = int(math.floor(float(floor_frac) * float(nk - window)))
    f = window + r                              # w + r of Eq. 1
    B_score = n * (nk - f)                      # what is left to share out
    cap = L - f                                 # a head cannot keep more than L

    capped = np.zeros(n, dtype=bool)
    x = np.zeros(n, dtype=np.float64)
    while True:
        free = [h for h in range(n) if not capped[h]]
        T = float(B_score - int(capped.sum()) * cap)
        tot = 0.0
        for h in free:
            tot += S[h]
        for h in free:
            x[h] = (T * S[h]) / tot if tot > 0.0 else T / float(len(free))
        over = [h for h in free if x[h] > float(cap)]
        if not over:
            break
        for h in over:
            capped[h] = True
            x[h] = float(cap)

    e = np.zeros(n, dtype=np.int64)
    frac = np.zeros(n, dtype=np.float64)
    for h in range(n):
        if capped[h]:
            e[h] = cap
        else:
            e[h] = int(math.floor(x[h]))
            frac[h] = x[h] - float(e[h])
    leftover = B_score - int(e.sum())
    free = [h for h in range(n) if not capped[h]]
    order = sorted(free, key=lambda h: (-frac[h], h))       # largest remainder first
    while leftover > 0:
        progressed = False
        for h in order:
            if leftover > 0 and e[h] < cap:
                e[h] += 1
                leftover -= 1
                progressed = True
        assert progressed
    # floating-point safety net: floors of rounded shares overshoot by a unit
    rev = sorted(free, key=lambda h: (frac[h], -h))
    while leftover < 0:
        progressed = False
        for h in rev:
            if leftover < 0 and e[h] > 0:
                e[h] -= 1
                leftover += 1
                progressed = True
        assert progressed

    b = e + f
    cu = np.zeros(n + 1, dtype=np.int64)
    cu[1:] = np.cumsum(b)
    return b, cu


# ---------------------------------------------------------------------------
# Stage 3: Spectral Score Smoothing
# ---------------------------------------------------------------------------

def _twiddle_table(L: int) -> np.ndarray:
    """exp(+2*pi*i*m/L) for m = 0..L-1, float64, from exactly reduced angles."""
    m = np.arange(L, dtype=np.float64)
    ang = 2.0 * np.pi * (m / float(L))
    return np.cos(ang) + 1j * np.sin(ang)


def rdft(s: np.ndarray, k_max: Optional[int] = None) -> np.ndarray:
    """Bins 0..k_max of the unnormalised real DFT (Sec. 3.3, Eq. 13):
    F_k = sum_n s_n exp(-2*pi*i*k*n/L). Default k_max = floor(L/2) (all bins)."""
    s = np.asarray(s, dtype=np.float64)
    L = s.shape[0]
    if k_max is None:
        k_max = L // 2
    tw = np.conj(_twiddle_table(L))
    n = np.arange(L, dtype=np.int64)
    F = np.empty(k_max + 1, dtype=np.complex128)
    step = max(1, (1 << 21) // max(L, 1))
    for k0 in range(0, k_max + 1, step):
        kk = np.arange(k0, min(k0 + step, k_max + 1), dtype=np.int64)
        idx = (kk[:, None] * n[None, :]) % L            # k*n reduced in integers
        F[k0:k0 + len(kk)] = tw[idx] @ s
    return F


def irdft(F: np.ndarray, L: int) -> np.ndarray:
    """Inverse real DFT of length L (Sec. 3.3, Eq. 19) from bins 0..len(F)-1;
    missing higher bins are zero. s_n = (1/L) sum_k g_k Re(F_k exp(+2*pi*i*k*n/L)),
    g_k = 1 for k = 0 and for k = L/2 (L even), else 2."""
    F = np.asarray(F, dtype=np.complex128)
    nb = F.shape[0]
    assert nb <= L // 2 + 1
    tw = _twiddle_table(L)
    n = np.arange(L, dtype=np.int64)
    g = np.full(nb, 2.0)
    g[0] = 1.0
    if L % 2 == 0 and nb == L // 2 + 1:
        g[-1] = 1.0
    out = np.zeros(L, dtype=np.float64)
    step = max(1, (1 << 21) // max(L, 1))
    for k0 in range(0, nb, step):
        kk = np.arange(k0, min(k0 + step, nb), dtype=np.int64)
        idx = (kk[:, None] * n[None, :]) % L
        out += ((g[kk] * F[kk]) @ tw[idx]).real
    return out / float(L)


def cutoff_bin(L: int, cutoff_frac: float) -> int:
    """Fixed-fraction cutoff: k* = floor(c * (n_bins - 1)), n_bins = floor(L/2) + 1."""
    return int(math.floor(float(cutoff_frac) * float(L // 2)))


def energy_cutoff_bin(F: np.ndarray, rho: float, skip_dc: bool = False) -> int:
    """Adaptive cutoff (Sec. 3.3, Eqs. 14-16): smallest k* with
    E(k*) >= rho * E(last bin), E(k) = sum_{i<=k} |F_i|^2 over the one-sided
    spectrum, DC included as the equations are written. `skip_dc` is the
    variant whose sums start at bin 1 (the DC bin of a non-negative score
    sequence otherwise holds nearly all the energy); then k* >= 1."""
    m2 = np.abs(np.asarray(F, dtype=np.complex128)) ** 2
    if skip_dc and m2.shape[0] > 1:
        m2 = m2.copy()
        m2[0] = 0.0
        E = np.cumsum(m2)
        target = float(rho) * E[-1]
        return max(1, int(np.argmax(E >= target)))
    E = np.cumsum(m2)
    target = float(rho) * E[-1]
    return int(np.argmax(E >= target))


def mask_weights(k_star: int, taper_bins: int, n_bins: int) -> np.ndarray:
    """Frequency mask of Eqs. 17-18 with the cosine transition band that the
    text after Eq. 17 asks for: w_i = 1 for i <= k*, then `taper_bins` bins of
    a half-cosine roll-off, w_i = (1 + cos(pi (i - k*) / (T + 1))) / 2 for
    k* < i <= k* + T, and 0 beyond. T = 0 is the hard mask of Eq. 17. (The paper
    gives neither width nor exact shape of the band: this form is a reading.)"""
    i = np.arange(n_bins, dtype=np.float64)
    w = np.where(i <= k_star, 1.0, 0.0)
    T = int(taper_bins)
    if T > 0:
        band = (i > k_star) & (i <= k_star + T)
        w = np.where(band, 0.5 * (1.0 + np.cos(np.pi * (i - k_star) / float(T + 1))), w)
    return w


def smooth(s: np.ndarray, cutoff_frac: float, alpha: float, *,
           energy_rho: Optional[float] = None, skip_dc: bool = False,
           taper_bins: int = 0, k_star: Optional[int] = None) -> np.ndarray:
    """Spectral Score Smoothing of one head's sequence (Sec. 3.3, Eqs. 13-20).

    F = RDFT(s); F~ = F * w with the mask of Eqs. 17-18 (bins i <= k* kept,
    optional cosine roll-off over the next `taper_bins` bins);
    s~ = IRDFT(F~, L) (Eq. 19); return (1 - alpha) s + alpha s~ (Eq. 20).
    k* is the fixed fraction `cutoff_frac` of the bins, or, when `energy_rho`
    is given, the energy-based cutoff of Eqs. 15-16, or `k_star` when forced.
    """
    s = np.asarray(s, dtype=np.float64)
    L = s.shape[0]
    n_bins = L // 2 + 1
    if k_star is not None:
        ks = int(k_star)
    elif energy_rho is None:
        ks = cutoff_bin(L, cutoff_frac)
    else:
        ks = energy_cutoff_bin(rdft(s), energy_rho, skip_dc)
    k_top = min(ks + int(taper_bins), n_bins - 1)
    F = rdft(s, k_top) * mask_weights(ks, taper_bins, n_bins)[:k_top + 1]
    s_tilde = irdft(F, L)
    return (1.0 - float(alpha)) * s + float(alpha) * s_tilde


# ---------------------------------------------------------------------------
# Stage 4: per-head top-k selection
# ---------------------------------------------------------------------------

def select(s_hat: np.ndarray, budget: int, window: int) -> np.ndarray:
    """Indices kept for one head, ascending (int64).

    The last `window` positions are always kept (w of Eq. 1); the other
    budget - window slots go to the highest scores among positions
    [0, L - window), equal scores resolved in favour of the lower index
    (-0.0 and +0.0 are equal). Scores are assumed finite.
    """
    s_hat = np.asarray(s_hat)
    L = s_hat.shape[0]
    assert window <= budget <= L
    n_cand = L - window
    want = budget - window
    cand = list(range(n_cand))
    cand.sort(key=lambda j: (-float(s_hat[j]), j))        # full sort: score desc, index asc
    kept = sorted(cand[:want]) + list(range(n_cand, L))
    return np.asarray(kept, dtype=np.int64)


# ---------------------------------------------------------------------------
# Stage 5: K/V compaction
# ---------------------------------------------------------------------------

def compact(k: np.ndarray, v: np.ndarray, indices: List[np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    """Gather retained rows: k, v are [H_kv, L, d] (any dtype, copied bit for
    bit); indices[h] are head h's kept token indices. Output rows are packed
    head after head: [sum_h b_h, d]."""
    ko = [k[h][np.asarray(ix, dtype=np.int64)] for h, ix in enumerate(indices)]
    vo = [v[h][np.asarray(ix, dtype=np.int64)] for h, ix in enumerate(indices)]
    return np.concatenate(ko, axis=0), np.concatenate(vo, axis=0)


# ---------------------------------------------------------------------------
# After the path: one decoding step on the compacted cache
# ---------------------------------------------------------------------------

def decode_attend(q: np.ndarray, k_rows: Sequence[np.ndarray], v_rows: Sequence[np.ndarray], *,
                  scale: Optional[float] = None) -> np.ndarray:
    """Single-query attention of every query head over the retained rows of its
    KV head (Sec. 1 / Sec. 4.6: decoding runs on the compressed cache).
    q: [H_q, d]; k_rows[h], v_rows[h]: [b_h, d] for KV head h (b_h >= 1);
    query head j reads KV head j // (H_q / H_kv). Returns [H_q, d] float64:
    out_j = sum_t softmax_t(scale * <q_j, K_h[t]>) * V_h[t]."""
    q = np.asarray(q, dtype=np.float64)
    H_q, d = q.shape
    H_kv = len(k_rows)
    assert H_q % H_kv == 0 and len(v_rows) == H_kv
    G = H_q // H_kv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.empty((H_q, d), dtype=np.float64)
    for j in range(H_q):
        K = np.asarray(k_rows[j // G], dtype=np.float64)
        V = np.asarray(v_rows[j // G], dtype=np.float64)
        z = scale * (K @ q[j])
        z = z - z.max()
        e = np.exp(z)
        out[j] = (e / e.sum()) @ V
    return out


# ---------------------------------------------------------------------------
# The whole path for one item
# ---------------------------------------------------------------------------

def evict_item(q_win: np.ndarray, k: np.ndarray, budgets: Sequence[int], *, window: int,
               pool_kernel: int = 7, pool_mode: str = "avg", causal: bool = True,
               scale: Optional[float] = None, cutoff_frac: float = 0.125,
               alpha: float = 1.0):
    """score -> smooth -> select for one item whose per-head budgets are given
    (allocation is global over items, so it is done by the caller).
    Returns (s [H_kv, L], s_hat [H_kv, L], [indices per head])."""
    s = score(q_win, k, pool_kernel=pool_kernel, pool_mode=pool_mode, causal=causal, scale=scale)
    s_hat = np.stack([smooth(s[h], cutoff_frac, alpha) for h in range(s.shape[0])])
    idx = [select(s_hat[h], int(budgets[h]), window) for h in range(s.shape[0])]
    return s, s_hat, idx
