"""ctypes binding of libaudiokv.so. Same names as the C entry points (without
the audiokv_ prefix); every function only marshals arguments. Tensors must be
contiguous CUDA(HIP) tensors of the documented dtype; outputs are allocated
here with torch and returned."""
from __future__ import annotations

import ctypes as C
import dataclasses
import os
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libaudiokv.so")

POOL_AVG, POOL_MAX = 0, 1
LAYOUT_HEAD_MAJOR, LAYOUT_TOKEN_MAJOR = 0, 1
SCOPE_ITEM, SCOPE_GLOBAL = 0, 1
CUTOFF_FRACTION, CUTOFF_ENERGY, CUTOFF_ENERGY_NO_DC = 0, 1, 2


class AudioKVError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"audiokv error {code}: {msg}")
        self.code = code


class _CParams(C.Structure):
    _fields_ = [
        ("size", C.c_uint32),
        ("n_q_heads", C.c_int32),
        ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32),
        ("window", C.c_int32),
        ("pool_kernel", C.c_int32),
        ("pool_mode", C.c_int32),
        ("causal", C.c_int32),
        ("kv_layout", C.c_int32),
        ("softmax_scale", C.c_float),
        ("floor_frac", C.c_float),
        ("cutoff_mode", C.c_int32),
        ("taper_bins", C.c_int32),
        ("kv_stride_item", C.c_int64),
        ("kv_stride_head", C.c_int64),
        ("kv_stride_tok", C.c_int64),
    ]


@dataclass
class Params:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    window: int
    pool_kernel: int = 7
    pool_mode: int = POOL_AVG
    causal: int = 1
    kv_layout: int = LAYOUT_HEAD_MAJOR
    softmax_scale: float = 0.0
    floor_frac: float = 0.1
    cutoff_mode: int = CUTOFF_FRACTION
    taper_bins: int = 0
    kv_stride_item: int = 0       # explicit K/V strides in elements; all 0: the packed layout of kv_layout
    kv_stride_head: int = 0
    kv_stride_tok: int = 0

    def key(self) -> tuple:
        return (self.n_q_heads, self.n_kv_heads, self.head_dim, self.window, self.pool_kernel, self.pool_mode,
                self.causal, self.kv_layout, self.softmax_scale, self.floor_frac, self.cutoff_mode, self.taper_bins,
                self.kv_stride_item, self.kv_stride_head, self.kv_stride_tok)

    def c(self) -> _CParams:
        return _CParams(C.sizeof(_CParams), self.n_q_heads, self.n_kv_heads, self.head_dim, self.window,
                        self.pool_kernel, self.pool_mode, self.causal, self.kv_layout,
                        self.softmax_scale, self.floor_frac, self.cutoff_mode, self.taper_bins,
                        self.kv_stride_item, self.kv_stride_head, self.kv_stride_tok)


def lib_path() -> str:
    return _LIB_PATH


def _load() -> C.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2604_06694_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_double
    pp = C.POINTER(_CParams)
    lib.audiokv_version.restype = i32
    lib.audiokv_last_error.restype = C.c_char_p
    lib.audiokv_n_keep.restype = i32
    lib.audiokv_n_keep.argtypes = [f64, i32]
    lib.audiokv_total_kept.argtypes = [pp, i32, vp, f64, C.POINTER(i64)]
    lib.audiokv_workspace_bytes.argtypes = [pp, i32, vp, C.POINTER(C.c_size_t)]
    lib.audiokv_score.argtypes = [pp, vp, vp, vp, vp, i32, vp, vp, C.c_size_t, vp]
    lib.audiokv_score_lse.argtypes = [pp, vp, vp, vp, vp, vp, i32, vp, vp, C.c_size_t, vp]
    lib.audiokv_allocate.argtypes = [pp, vp, i32, i32, i32, vp, vp, f64, vp, vp, vp]
    lib.audiokv_smooth.argtypes = [pp, vp, vp, vp, i32, f64, f64, vp, vp, C.c_size_t, vp]
    lib.audiokv_smooth_cutoffs.argtypes = [pp, vp, vp, vp, i32, f64, vp, vp, C.c_size_t, vp]
    lib.audiokv_select.argtypes = [pp, vp, vp, vp, vp, vp, i32, vp, vp, C.c_size_t, vp]
    lib.audiokv_compact.argtypes = [pp, vp, vp, vp, vp, vp, vp, i32, i64, vp, vp, vp]
    lib.audiokv_evict.argtypes = [pp, vp, vp, vp, vp, i32, vp, vp, i32, f64, f64, f64,
                                  vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.audiokv_evict_lse.argtypes = [pp, vp, vp, vp, vp, vp, i32, vp, vp, i32, f64, f64, f64,
                                  vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.audiokv_evict_noalloc.argtypes = [pp, vp, vp, vp, vp, i32, vp, vp, i32, f64, f64, f64,
                                          vp, vp, vp, vp, vp, vp]
    lib.audiokv_decode_workspace_bytes.argtypes = [pp, i32, i64, C.POINTER(C.c_size_t)]
    lib.audiokv_decode_attend.argtypes = [pp, vp, vp, vp, vp, i32, i64, vp, vp, C.c_size_t, vp]
    lib.audiokv_profile_enable.argtypes = [i32]
    lib.audiokv_profile_enable.restype = i32
    lib.audiokv_profile_read.argtypes = [C.POINTER(C.c_float)]
    lib.audiokv_profile_read.restype = i32
    for name in ("total_kept", "workspace_bytes", "score", "allocate", "smooth", "smooth_cutoffs", "select", "compact", "evict",
                 "decode_workspace_bytes", "decode_attend", "score_lse", "evict_lse", "evict_noalloc"):
        getattr(lib, "audiokv_" + name).restype = i32
    return lib


_lib = _load()


def _check(rc: int) -> None:
    if rc != 0:
        raise AudioKVError(rc, _lib.audiokv_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


_LENS_CACHE: dict = {}


def _host_lens(seqlens: Sequence[int]):
    """ctypes int32 array of the lengths; the arrays of recent length lists are kept (a serving loop passes the
    same few lists over and over, and building the array costs more than the rest of the marshalling)."""
    key = tuple(seqlens)
    arr = _LENS_CACHE.get(key)
    if arr is None:
        if len(_LENS_CACHE) > 256:
            _LENS_CACHE.clear()
        arr = _LENS_CACHE[key] = (C.c_int32 * len(key))(*[int(x) for x in key])
    return arr


def _cu(seqlens: Sequence[int], device) -> torch.Tensor:
    cu = [0]
    for L in seqlens:
        cu.append(cu[-1] + int(L))
    return torch.tensor(cu, dtype=torch.int32, device=device)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _need(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor of dtype {dtype}")
    return t


def version() -> int:
    return _lib.audiokv_version()


def n_keep(ratio: float, L: int) -> int:
    return _lib.audiokv_n_keep(float(ratio), int(L))


_SIZE_CACHE: dict = {}


def _cached(key, compute):
    v = _SIZE_CACHE.get(key)
    if v is None:
        if len(_SIZE_CACHE) > 1024:
            _SIZE_CACHE.clear()
        v = _SIZE_CACHE[key] = compute()
    return v


def total_kept(p: Params, seqlens: Sequence[int], ratio: float) -> int:
    def compute():
        out = C.c_int64(0)
        cp = p.c()
        _check(_lib.audiokv_total_kept(C.byref(cp), len(seqlens), _host_lens(seqlens), float(ratio), C.byref(out)))
        return out.value
    return _cached(("rows", p.key(), tuple(seqlens), float(ratio)), compute)


def workspace_bytes(p: Params, seqlens: Sequence[int]) -> int:
    def compute():
        out = C.c_size_t(0)
        cp = p.c()
        _check(_lib.audiokv_workspace_bytes(C.byref(cp), len(seqlens), _host_lens(seqlens), C.byref(out)))
        return out.value
    return _cached(("ws", p.key(), tuple(seqlens)), compute)


def _workspace(p: Params, seqlens: Sequence[int], device, workspace: Optional[torch.Tensor]) -> torch.Tensor:
    need = workspace_bytes(p, seqlens)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace


def score(p: Params, q_win: torch.Tensor, k: torch.Tensor, seqlens: Sequence[int], *,
          cu_seqlens: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
          workspace: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None) -> torch.Tensor:
    """`lse` (fp32 [n_items, n_q_heads, window], natural-log softmax denominators of the window rows) selects
    audiokv_score_lse."""
    _need(q_win, torch.bfloat16, "q_win"); _need(k, torch.bfloat16, "k")
    dev = k.device
    cu = cu_seqlens if cu_seqlens is not None else _cu(seqlens, dev)
    total = sum(int(x) for x in seqlens) * p.n_kv_heads
    if out is None:
        out = torch.empty(total, dtype=torch.float32, device=dev)
    ws = _workspace(p, seqlens, dev, workspace)
    cp = p.c()
    if lse is not None:
        _need(lse, torch.float32, "lse")
        _check(_lib.audiokv_score_lse(C.byref(cp), _ptr(q_win), _ptr(k), _ptr(lse), _ptr(cu), _host_lens(seqlens),
                                      len(seqlens), _ptr(out), _ptr(ws), ws.numel(), _stream()))
        return out
    _check(_lib.audiokv_score(C.byref(cp), _ptr(q_win), _ptr(k), _ptr(cu), _host_lens(seqlens), len(seqlens),
                              _ptr(out), _ptr(ws), ws.numel(), _stream()))
    return out


def allocate(p: Params, weights: torch.Tensor, n_segments: int, heads_per_segment: int, seqlens: Sequence[int],
             ratio: float, *, weight_group: int = 1, cu_seqlens: Optional[torch.Tensor] = None
             ) -> Tuple[torch.Tensor, torch.Tensor]:
    _need(weights, torch.float32, "weights")
    dev = weights.device
    cu = cu_seqlens if cu_seqlens is not None else _cu(seqlens, dev)
    n = n_segments * heads_per_segment
    budgets = torch.empty(n, dtype=torch.int32, device=dev)
    cu_b = torch.empty(n + 1, dtype=torch.int32, device=dev)
    cp = p.c()
    _check(_lib.audiokv_allocate(C.byref(cp), _ptr(weights), n_segments, heads_per_segment, weight_group, _ptr(cu),
                                 _host_lens(seqlens), float(ratio), _ptr(budgets), _ptr(cu_b), _stream()))
    return budgets, cu_b


def smooth(p: Params, scores: torch.Tensor, seqlens: Sequence[int], cutoff_frac: float, alpha: float, *,
           cu_seqlens: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
           workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    _need(scores, torch.float32, "scores")
    dev = scores.device
    cu = cu_seqlens if cu_seqlens is not None else _cu(seqlens, dev)
    if out is None:
        out = torch.empty_like(scores)
    ws = _workspace(dataclasses.replace(p, window=0), seqlens, dev, workspace)
    cp = p.c()
    _check(_lib.audiokv_smooth(C.byref(cp), _ptr(scores), _ptr(cu), _host_lens(seqlens), len(seqlens),
                               float(cutoff_frac), float(alpha), _ptr(out), _ptr(ws), ws.numel(), _stream()))
    return out


def smooth_cutoffs(p: Params, scores: torch.Tensor, seqlens: Sequence[int], cutoff_frac: float, *,
                   cu_seqlens: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The cutoff bin k* of every head (int32 [n_items * n_kv_heads])."""
    _need(scores, torch.float32, "scores")
    dev = scores.device
    cu = cu_seqlens if cu_seqlens is not None else _cu(seqlens, dev)
    out = torch.empty(len(seqlens) * p.n_kv_heads, dtype=torch.int32, device=dev)
    ws = _workspace(dataclasses.replace(p, window=0), seqlens, dev, workspace)
    cp = p.c()
    _check(_lib.audiokv_smooth_cutoffs(C.byref(cp), _ptr(scores), _ptr(cu), _host_lens(seqlens), len(seqlens),
                                       float(cutoff_frac), _ptr(out), _ptr(ws), ws.numel(), _stream()))
    return out


def select(p: Params, scores: torch.Tensor, budgets: torch.Tensor, cu_budgets: torch.Tensor,
           seqlens: Sequence[int], total_rows: int, *, cu_seqlens: Optional[torch.Tensor] = None) -> torch.Tensor:
    _need(scores, torch.float32, "scores"); _need(budgets, torch.int32, "budgets"); _need(cu_budgets, torch.int32, "cu_budgets")
    dev = scores.device
    cu = cu_seqlens if cu_seqlens is not None else _cu(seqlens, dev)
    idx = torch.empty(max(int(total_rows), 1), dtype=torch.int32, device=dev)
    cp = p.c()
    _check(_lib.audiokv_select(C.byref(cp), _ptr(scores), _ptr(budgets), _ptr(cu_budgets), _ptr(cu),
                               _host_lens(seqlens), len(seqlens), _ptr(idx), None, 0, _stream()))
    return idx[:int(total_rows)]


def compact(p: Params, k: torch.Tensor, v: torch.Tensor, indices: torch.Tensor, cu_budgets: torch.Tensor,
            seqlens: Sequence[int], total_rows: int, *, cu_seqlens: Optional[torch.Tensor] = None
            ) -> Tuple[torch.Tensor, torch.Tensor]:
    _need(k, torch.bfloat16, "k"); _need(v, torch.bfloat16, "v"); _need(indices, torch.int32, "indices")
    dev = k.device
    cu = cu_seqlens if cu_seqlens is not None else _cu(seqlens, dev)
    k_out = torch.empty((max(int(total_rows), 1), p.head_dim), dtype=torch.bfloat16, device=dev)
    v_out = torch.empty_like(k_out)
    cp = p.c()
    _check(_lib.audiokv_compact(C.byref(cp), _ptr(k), _ptr(v), _ptr(indices), _ptr(cu_budgets), _ptr(cu),
                                _host_lens(seqlens), len(seqlens), int(total_rows), _ptr(k_out), _ptr(v_out),
                                _stream()))
    return k_out[:int(total_rows)], v_out[:int(total_rows)]


def evict(p: Params, q_win: torch.Tensor, k: torch.Tensor, v: torch.Tensor, weights: torch.Tensor,
          seqlens: Sequence[int], ratio: float, cutoff_frac: float, alpha: float, *,
          alloc_scope: int = SCOPE_GLOBAL, cu_seqlens: Optional[torch.Tensor] = None,
          workspace: Optional[torch.Tensor] = None, outputs: Optional[dict] = None,
          lse: Optional[torch.Tensor] = None) -> dict:
    """Runs the fused path (audiokv_evict_lse when `lse` is given). `outputs` may carry preallocated k_out, v_out, indices, budgets, cu_budgets
    (used by the benchmark so that the timed region allocates nothing)."""
    _need(q_win, torch.bfloat16, "q_win"); _need(k, torch.bfloat16, "k"); _need(v, torch.bfloat16, "v")
    _need(weights, torch.float32, "weights")
    dev = k.device
    cu = cu_seqlens if cu_seqlens is not None else _cu(seqlens, dev)
    n_heads = len(seqlens) * p.n_kv_heads
    rows = total_kept(p, seqlens, ratio)
    o = outputs if outputs is not None else {}
    if "k_out" not in o:
        o["k_out"] = torch.empty((max(rows, 1), p.head_dim), dtype=torch.bfloat16, device=dev)
        o["v_out"] = torch.empty_like(o["k_out"])
        o["indices"] = torch.empty(max(rows, 1), dtype=torch.int32, device=dev)
        o["budgets"] = torch.empty(n_heads, dtype=torch.int32, device=dev)
        o["cu_budgets"] = torch.empty(n_heads + 1, dtype=torch.int32, device=dev)
    ws = _workspace(p, seqlens, dev, workspace)
    cp = p.c()
    if lse is not None:
        _need(lse, torch.float32, "lse")
        _check(_lib.audiokv_evict_lse(C.byref(cp), _ptr(q_win), _ptr(k), _ptr(v), _ptr(lse), _ptr(weights),
                                      int(alloc_scope), _ptr(cu), _host_lens(seqlens), len(seqlens), float(ratio),
                                      float(cutoff_frac), float(alpha), _ptr(o["k_out"]), _ptr(o["v_out"]),
                                      _ptr(o["indices"]), _ptr(o["budgets"]), _ptr(o["cu_budgets"]), _ptr(ws),
                                      ws.numel(), _stream()))
        o["total_rows"] = rows
        o["workspace"] = ws
        return o
    _check(_lib.audiokv_evict(C.byref(cp), _ptr(q_win), _ptr(k), _ptr(v), _ptr(weights), int(alloc_scope), _ptr(cu),
                              _host_lens(seqlens), len(seqlens), float(ratio), float(cutoff_frac), float(alpha),
                              _ptr(o["k_out"]), _ptr(o["v_out"]), _ptr(o["indices"]), _ptr(o["budgets"]),
                              _ptr(o["cu_budgets"]), _ptr(ws), ws.numel(), _stream()))
    o["total_rows"] = rows
    o["workspace"] = ws
    return o


NOALLOC_SCRATCH_BYTES = 8 << 20


def evict_noalloc(p: Params, q_win: torch.Tensor, k: torch.Tensor, v: torch.Tensor, weights: torch.Tensor,
                  seqlens: Sequence[int], ratio: float, cutoff_frac: float, alpha: float, outputs: dict, *,
                  alloc_scope: int = SCOPE_GLOBAL, cu_seqlens: torch.Tensor) -> dict:
    """audiokv_evict_noalloc: the caller brings every buffer (`outputs` with k_out, v_out, indices, budgets,
    cu_budgets; `cu_seqlens` on the device); neither this function nor the library allocates device memory."""
    cp = p.c()
    o = outputs
    _check(_lib.audiokv_evict_noalloc(C.byref(cp), _ptr(q_win), _ptr(k), _ptr(v), _ptr(weights), int(alloc_scope),
                                      _ptr(cu_seqlens), _host_lens(seqlens), len(seqlens), float(ratio),
                                      float(cutoff_frac), float(alpha), _ptr(o["k_out"]), _ptr(o["v_out"]),
                                      _ptr(o["indices"]), _ptr(o["budgets"]), _ptr(o["cu_budgets"]), _stream()))
    return o


def decode_workspace_bytes(p: Params, n_items: int, total_rows: int) -> int:
    out = C.c_size_t(0)
    cp = p.c()
    _check(_lib.audiokv_decode_workspace_bytes(C.byref(cp), int(n_items), int(total_rows), C.byref(out)))
    return out.value


def decode_attend(p: Params, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                  cu_budgets: torch.Tensor, n_items: int, total_rows: int, *,
                  out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """One decoding step on the compacted cache: fp32 [n_items, n_q_heads, head_dim]."""
    _need(q, torch.bfloat16, "q"); _need(k_cache, torch.bfloat16, "k_cache"); _need(v_cache, torch.bfloat16, "v_cache")
    _need(cu_budgets, torch.int32, "cu_budgets")
    dev = q.device
    if out is None:
        out = torch.empty((n_items, p.n_q_heads, p.head_dim), dtype=torch.float32, device=dev)
    need = decode_workspace_bytes(p, n_items, total_rows)
    ws = workspace if workspace is not None else torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    cp = p.c()
    _check(_lib.audiokv_decode_attend(C.byref(cp), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(cu_budgets),
                                      int(n_items), int(total_rows), _ptr(out), _ptr(ws), ws.numel(), _stream()))
    return out


PROFILE_STAGES = ("allocate", "score_sweep1", "score_sweep2", "pool_smooth", "select", "compact")


def profile_enable(on: bool) -> None:
    _check(_lib.audiokv_profile_enable(1 if on else 0))


def profile_read() -> dict:
    """Milliseconds of each kernel of the most recent evict() issued while profiling was enabled."""
    buf = (C.c_float * len(PROFILE_STAGES))()
    _check(_lib.audiokv_profile_read(buf))
    return {n: float(buf[i]) for i, n in enumerate(PROFILE_STAGES)}
