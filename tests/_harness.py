"""Helpers shared by the GPU parity tests: numpy <-> device tensors, the error measure, step drivers."""
from __future__ import annotations

import numpy as np
import torch

# The bound the target states: relative error per output row, max|got - ref| / max|ref|.
TOL = {"bf16": 2e-2, "f32": 1e-5}

# Bounds derived from the arithmetic, asserted beside the stated one (all relative to the row maximum):
#   "logits"  fp32 logits from the same bf16 bits, fp32 accumulation over d <= 16384 terms in a blocked
#             order: the sum's rounding error is ~1e-6 of the row scale; 1e-4 leaves two orders of slack.
#   "resid"   logits behind the residual block: SiLU(W1 h) + h is rounded to bf16 on both sides, and the
#             fp32 / fp64 values of it straddle a rounding boundary in about one element per 2000, each
#             moving a logit by ~2^-8 |w r|: a few 1e-5 of the row maximum at d = 4096; bound 5e-4.
#   "rounded" outputs stored in bf16 (attention, block operators): half an ulp of the result (2^-9)
#             plus bf16 probabilities in the second product and fp16 split partials: bound 2^-7.
#   "rounded2" the same when the reference is itself rounded to bf16 (operators of the block): the two
#             sides may round a value to neighbouring bf16 numbers, one ulp = up to 2^-7 of the value
#             apart, on top of the above: bound 2^-6.
BOUND = {"bf16": {"logits": 1e-4, "resid": 5e-4, "rounded": 2.0 ** -7, "rounded2": 2.0 ** -6},
         "f32": {"logits": 1e-5, "resid": 1e-5, "rounded": 1e-5, "rounded2": 1e-5}}

_ACHIEVED = {}


def record(case: str, stage: str, err: float) -> None:
    """Keep the largest error seen per (case, stage) and mirror the table to gpurun_out/parity_achieved.json."""
    import json
    import os
    key = f"{case} | {stage}"
    _ACHIEVED[key] = max(_ACHIEVED.get(key, 0.0), float(err))
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    try:
        os.makedirs(os.path.join(root, "gpurun_out"), exist_ok=True)
        path = os.path.join(root, "gpurun_out", "parity_achieved.json")
        old = {}
        if os.path.exists(path):
            with open(path) as f:
                old = json.load(f)
        old.update(_ACHIEVED)
        with open(path, "w") as f:
            json.dump(old, f, indent=1, sort_keys=True)
    except OSError:
        pass


def resid_bound(dtype: str, d: int) -> float:
    """Derived bound for logits behind the residual block at hidden size d: a storage rounding that falls the
    other way moves a logit by 2^-8 |w r|, which is about 2^-8 / sqrt(d) of a row whose d terms add up at
    random, and a row maximum sits about four such deviations out; a handful of such roundings per row."""
    return BOUND[dtype]["resid"] if dtype != "bf16" else max(BOUND[dtype]["resid"], 1e-4 + 2.0 ** -8 * 4.0 / d ** 0.5)


def check_close(case: str, stage: str, got, ref, dtype: str, kind: str = None, rounded_output: bool = False,
                bound: float = None) -> float:
    """Assert the stated bound and the derived one, and record the achieved error."""
    kind = kind or ("rounded" if rounded_output else ("resid" if stage == "heads" else "logits"))
    bound = BOUND[dtype][kind] if bound is None else bound
    err = row_rel_err(got, ref)
    record(case, stage, err)
    assert err <= TOL[dtype], f"{case} {stage}: {err:.3e} exceeds the stated bound {TOL[dtype]:.0e}"
    assert err <= bound, f"{case} {stage}: {err:.3e} exceeds the derived bound {bound:.1e} ({kind})"
    return err


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
