"""Analytical model of the appendix "Exploration and Modeling of Hardware Constraints": operational
intensity of the block's operators under parallel decoding with q candidate tokens, the logarithmic
fit of the acceleration rate, and the simulated speedup of a simplified decoder block.

Closed forms only (host arithmetic on a handful of numbers).  The operator latencies the model
consumes are either roofline estimates from a machine's peak rates or the latencies measured on
the GPU by ``bench.py --speed-model``."""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Callable, Dict, Iterable, List, Sequence

ACC_RATE_COEFF = 0.477      # appendix, "Predicting Medusa performance": acc_rate = 0.477 log(num_candidate)


def attention_intensity(q: int, s: int, d: int) -> float:
    """Operator table, parallel-decoding rows Q K^T and P V, per head: 4 q s d flops over 2-byte
    operands Q (q d), K and V (2 s d) and the score matrix written and read back (2 s q), i.e.
    q s d / (q d + s d + s q) flops per byte (batch and head count cancel)."""
    return q * s * d / (q * d + s * d + s * q)


def linear_intensity(m: int, h: int, i: int) -> float:
    """Operator table, rows X W_u / X W_g / X W_d with m = batch * q token rows: 2 m h i flops over
    2-byte input, output (m (h + i)) and weights (h i): m h i / (m (h + i) + h i) flops per byte."""
    return m * h * i / (m * (h + i) + h * i)


def acceleration_rate(num_candidates: int) -> float:
    """Tokens accepted per step as fitted in the appendix: 0.477 log2(candidates).  The base is not
    printed; base 2 gives 2.86 at 64 candidates, in line with the about three tokens per step the
    experiments report (the natural logarithm would give 1.98)."""
    return ACC_RATE_COEFF * math.log2(num_candidates) if num_candidates > 1 else 0.0


@dataclass(frozen=True)
class BlockShape:
    """Simplified decoder block of the latency model: X W_Q, X W_K, X W_V, Q K^T, P V, X W_u, X W_g, X W_d."""
    h: int          # hidden size
    inter: int      # feed-forward width
    n_heads: int
    n_kv_heads: int
    d: int          # head dimension

    def operators(self, b: int, q: int, s: int, elem: int = 2) -> Dict[str, Dict[str, float]]:
        """flops and bytes of every operator for batch b, q candidate tokens, s cached tokens.
        Attention is counted fused (scores never leave the chip), which is how this library runs
        it; the appendix's unfused count is `attention_intensity`."""
        m = b * q
        lin = lambda n_in, n_out: {"flops": 2.0 * m * n_in * n_out, "bytes": float(elem) * (m * (n_in + n_out) + n_in * n_out)}
        kv = self.n_kv_heads * self.d
        ops = {
            "X W_Q": lin(self.h, self.n_heads * self.d),
            "X W_K": lin(self.h, kv),
            "X W_V": lin(self.h, kv),
            "QK^T, PV": {"flops": 4.0 * b * self.n_heads * q * (s + q) * self.d,
                         "bytes": float(elem) * b * (2 * self.n_kv_heads * (s + q) * self.d + 2 * self.n_heads * q * self.d)},
            "X W_u": lin(self.n_heads * self.d, self.inter),
            "X W_g": lin(self.n_heads * self.d, self.inter),
            "X W_d": lin(self.inter, self.h),
        }
        return ops


LLAMA_7B = BlockShape(h=4096, inter=11008, n_heads=32, n_kv_heads=32, d=128)
LLAMA_13B = BlockShape(h=5120, inter=13824, n_heads=40, n_kv_heads=40, d=128)
LLAMA_33B = BlockShape(h=6656, inter=17920, n_heads=52, n_kv_heads=52, d=128)


def roofline_latency(shape: BlockShape, b: int, q: int, s: int, peak_flops: float, peak_bytes: float) -> float:
    """Seconds for one block if every operator ran at the roofline of a machine with the given
    peak FLOP/s and bytes/s: sum over operators of max(flops / peak_flops, bytes / peak_bytes)."""
    return sum(max(o["flops"] / peak_flops, o["bytes"] / peak_bytes) for o in shape.operators(b, q, s).values())


def simulate_speedup(latency: Callable[[int], float], candidates: Sequence[int]) -> List[Dict[str, float]]:
    """The appendix's prediction: decoding with q candidates accepts acceleration_rate(q) tokens per
    step at latency(q) per block, against one token per latency(1) for plain decoding, so
    speedup(q) = acceleration_rate(q) * latency(1) / latency(q).  Returns one row per q."""
    base = latency(1)
    rows = []
    for q in candidates:
        lat = latency(q)
        rows.append({"candidates": q, "acc_rate": acceleration_rate(q), "latency": lat, "normalized_latency": lat / base,
                     "speedup": acceleration_rate(q) * base / lat})
    return rows


def best_candidates(rows: Iterable[Dict[str, float]]) -> int:
    return int(max(rows, key=lambda r: r["speedup"])["candidates"])
