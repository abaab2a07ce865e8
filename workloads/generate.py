"""Seeded tensor generators shared by the oracle's tests and the HIP path's tests.

Every tensor is a pure function of (seed, tensor id, shape, std, dtype): it is
drawn in fixed-size chunks, chunk c from the stream
``SeedSequence([seed, tensor_id, c])``, so the bytes do not depend on how many
worker threads filled it.  bf16 tensors are float32 draws rounded once
(round-to-nearest-even) and handed out as raw ``uint16`` bit patterns.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Iterable, Optional, Sequence

import numpy as np

from .configs import StepConfig

# Stable ids: changing one changes that tensor's bytes.
TENSOR_IDS = {
    "h_last": 0,        # [B, d]            hidden state the Medusa heads read
    "hidden_tree": 1,   # [B, T, d]         backbone output rows for the tree tokens
    "w1": 2,            # [K, d, d]         residual-block weights, out x in
    "w2": 3,            # [K, V, d]         vocabulary projections, out x in
    "w_lm": 4,          # [V, d]            original LM head, out x in
    "q": 5,             # [B, Hq, T, D]
    "k_tree": 6,        # [NL, B, Hkv, T, D]
    "v_tree": 7,        # [NL, B, Hkv, T, D]
    "k_cache": 8,       # [NL, B, Hkv, Lcap, D]
    "v_cache": 9,       # [NL, B, Hkv, Lcap, D]
    "prefix_len": 10,   # [B] int32
}

_CHUNK = 1 << 22


def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns, round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def f32_from_bf16_bits(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns -> the float32 values they denote (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _n_threads() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def draw_normal(seed: int, tensor_id: int, shape: Sequence[int], std: float, dtype: str) -> np.ndarray:
    """N(0, std^2) tensor; float32 array for "f32", uint16 bit patterns for "bf16"."""
    if dtype not in ("f32", "bf16"):
        raise ValueError(f"unknown dtype {dtype!r}")
    n = int(np.prod(shape, dtype=np.int64))
    out = np.empty(n, dtype=np.float32 if dtype == "f32" else np.uint16)
    n_chunks = (n + _CHUNK - 1) // _CHUNK

    def fill(c: int) -> None:
        lo, hi = c * _CHUNK, min(n, (c + 1) * _CHUNK)
        rng = np.random.default_rng(np.random.SeedSequence([seed, tensor_id, c]))
        x = rng.standard_normal(hi - lo, dtype=np.float32)
        if std != 1.0:
            x *= np.float32(std)
        out[lo:hi] = x if dtype == "f32" else bf16_bits_from_f32(x)

    if n_chunks <= 1:
        for c in range(n_chunks):
            fill(c)
    else:
        with ThreadPoolExecutor(_n_threads()) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out.reshape(tuple(shape))


def draw_prefix_len(cfg: StepConfig) -> np.ndarray:
    """Per-sequence prefix KV lengths, uniform integers in [L_min, L_max]."""
    rng = np.random.default_rng(np.random.SeedSequence([cfg.seed, TENSOR_IDS["prefix_len"], 0]))
    return rng.integers(cfg.L_min, cfg.L_max + 1, size=cfg.B).astype(np.int32)


def tensor_shapes(cfg: StepConfig, nl: Optional[int] = None) -> Dict[str, tuple]:
    NL = cfg.NL if nl is None else nl
    return {
        "h_last": (cfg.B, cfg.d),
        "hidden_tree": (cfg.B, cfg.T, cfg.d),
        "w1": (cfg.K, cfg.d, cfg.d),
        "w2": (cfg.K, cfg.V, cfg.d),
        "w_lm": (cfg.V, cfg.d),
        "q": (cfg.B, cfg.Hq, cfg.T, cfg.D),
        "k_tree": (NL, cfg.B, cfg.Hkv, cfg.T, cfg.D),
        "v_tree": (NL, cfg.B, cfg.Hkv, cfg.T, cfg.D),
        "k_cache": (NL, cfg.B, cfg.Hkv, cfg.Lcap, cfg.D),
        "v_cache": (NL, cfg.B, cfg.Hkv, cfg.Lcap, cfg.D),
    }


_WEIGHTS = ("w1", "w2", "w_lm")


def make_step_inputs(cfg: StepConfig, names: Optional[Iterable[str]] = None,
                     nl: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Draw the named input tensors of one step (all of them by default).

    Activations and KV are N(0,1), weights N(0, 0.02^2).  ``nl`` overrides the
    number of KV layers drawn (layer l of a tensor is the same bytes whatever
    ``nl`` is only when the tensor is drawn whole; tests that compare two sides
    always pass both sides the same arrays).
    """
    shapes = tensor_shapes(cfg, nl)
    wanted = list(shapes) + ["prefix_len"] if names is None else list(names)
    out: Dict[str, np.ndarray] = {}
    for name in wanted:
        if name == "prefix_len":
            out[name] = draw_prefix_len(cfg)
            continue
        std = 0.02 if name in _WEIGHTS else 1.0
        out[name] = draw_normal(cfg.seed, TENSOR_IDS[name], shapes[name], std, cfg.dtype)
    return out
