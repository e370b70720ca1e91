"""Helpers shared by the GPU parity tests: tensor marshalling and the tolerance rule."""
from __future__ import annotations

import numpy as np
import torch


def bf16_tensor(bits: np.ndarray, device="cuda") -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on the device (no value change)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device)
    return t.view(torch.bfloat16)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def rel_err(gpu: np.ndarray, ref: np.ndarray, floor_frac: float = 1e-3) -> float:
    """max |g - o| / max(|o|, floor_frac * max|o|) over one head's sequence: the
    relative error with a floor, because smoothed scores cross zero."""
    ref = np.asarray(ref, dtype=np.float64)
    gpu = np.asarray(gpu, dtype=np.float64)
    den = np.maximum(np.abs(ref), floor_frac * np.abs(ref).max())
    return float((np.abs(gpu - ref) / den).max())


SCORE_RTOL = 2e-3     # pre-selection and smoothed scores: fp32 accumulation on bf16 inputs


def pack_items_head_major(items, key):
    """Concatenate per-item [H, L, d] blocks into the packed 1-D layout of the C ABI."""
    return np.concatenate([it[key].reshape(-1) for it in items])


def pack_items_token_major(items, key):
    return np.concatenate([np.ascontiguousarray(it[key].transpose(1, 0, 2)).reshape(-1) for it in items])
