"""Helpers shared by the GPU parity tests: numpy <-> device tensors, the error measure, step drivers."""
from __future__ import annotations

import numpy as np
import torch

TOL = {"bf16": 2e-2, "f32": 1e-5}


def to_dev(x: np.ndarray) -> torch.Tensor:
    """uint16 arrays are bfloat16 bit patterns; everything else keeps its dtype."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def to_host_bits(t: torch.Tensor) -> np.ndarray:
    """Raw storage back on the host as unsigned integers (uint16 for bfloat16, uint32 for float32),
    so that comparisons are bitwise (NaN poison included)."""
    if t.dtype == torch.bfloat16:
        return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.detach().view(torch.int32).cpu().numpy().view(np.uint32)
    return t.detach().cpu().numpy()


def bits(a: np.ndarray) -> np.ndarray:
    """Host array as unsigned integers of the same width (bitwise comparison)."""
    if a.dtype == np.float32:
        return a.view(np.uint32)
    return a


def row_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max over rows (last axis) of max|got - ref| / max|ref|."""
    got = np.asarray(got, np.float64).reshape(-1, got.shape[-1])
    ref = np.asarray(ref, np.float64).reshape(-1, ref.shape[-1])
    num = np.abs(got - ref).max(axis=1)
    den = np.maximum(np.abs(ref).max(axis=1), 1e-30)
    return float((num / den).max())


def poison_tail(cache: np.ndarray, prefix_len: np.ndarray) -> np.ndarray:
    """Copy of a [..., B, Hkv, Lcap, D] cache whose rows >= prefix_len[b] hold NaN (f32) / 0x7fc0 (bf16)."""
    out = cache.copy()
    B = prefix_len.shape[0]
    bad = np.uint16(0x7FC0) if out.dtype == np.uint16 else np.float32(np.nan)
    for b in range(B):
        out[..., b, :, int(prefix_len[b]):, :] = bad
    return out
