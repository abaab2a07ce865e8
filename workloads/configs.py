"""Shape tables of the five synthetic verification-step workloads.

Pure data: sizes, dtypes, seeds and acceptance hyper-parameters.  Nothing here
computes anything the method computes.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Tuple


@dataclass(frozen=True)
class StepConfig:
    name: str
    dtype: str                 # "f32" or "bf16": storage type of activations, weights and KV
    B: int                     # sequences in the batch
    d: int                     # hidden size
    Hq: int                    # query heads
    Hkv: int                   # key/value heads
    D: int                     # head dimension
    V: int                     # vocabulary size
    branching: Tuple[int, ...]  # s_1..s_K of the Cartesian candidate tree
    L_min: int                 # prefix KV length range (inclusive); equal => fixed length
    L_max: int
    Lcap: int                  # allocated cache rows per sequence (>= L_max + K + 1)
    NL: int                    # layers whose KV is committed
    accept: str                # "greedy" or "typical"
    temperature: float
    eps: float
    delta: float
    seed: int

    @property
    def K(self) -> int:
        return len(self.branching)

    @property
    def N(self) -> int:
        """Candidate nodes: sum over levels of the running product of s_k."""
        n, p = 0, 1
        for s in self.branching:
            p *= s
            n += p
        return n

    @property
    def T(self) -> int:
        """Tree tokens entering attention: candidates plus the root."""
        return self.N + 1


CONFIGS = {
    # Tiny fp32 step, batch 1.
    "C1": StepConfig("C1", "f32", 1, 256, 4, 4, 64, 1000, (3, 2), 128, 128, 160, 1,
                     "greedy", 1.0, 0.0, 0.0, 0),
    # 7B-shaped bf16 step, batch 1, prefix 1024, 32 layers committed.
    "C2": StepConfig("C2", "bf16", 1, 4096, 32, 32, 128, 32000, (4, 3, 2, 1), 1024, 1024, 1152, 32,
                     "greedy", 1.0, 0.0, 0.0, 1),
    # Long-context 7B-shaped step, typical acceptance.  Three cache layers are
    # allocated (one layer's KV is 136 MB), enough to rotate the attended layer.
    "C3": StepConfig("C3", "bf16", 1, 4096, 32, 32, 128, 32000, (4, 3, 2, 1), 8192, 8192, 8320, 3,
                     "typical", 0.7, 0.09, 0.3, 2),
    # 13B-shaped step, batch 4, ragged prefixes.
    "C4": StepConfig("C4", "bf16", 4, 5120, 40, 40, 128, 32000, (4, 3, 2, 1, 1), 512, 2048, 2176, 40,
                     "greedy", 1.0, 0.0, 0.0, 3),
    # GQA 7B-shaped step, batch 16, ragged prefixes, typical acceptance.
    "C5": StepConfig("C5", "bf16", 16, 4096, 32, 8, 128, 32000, (4, 3, 2, 1), 256, 4096, 4224, 32,
                     "typical", 0.7, 0.09, 0.3, 4),
}


def get_config(name: str) -> StepConfig:
    return CONFIGS[name]


def scaled_config(name: str, **overrides) -> StepConfig:
    """A named config with some sizes replaced (used for CPU-sized parity cases)."""
    return replace(CONFIGS[name], **overrides)


def synthetic_accuracy_table(K: int, S: int):
    """Stand-in for the calibration statistics of Sec. 2.3.3 (top-i accuracy of every head measured
    on a calibration set, which is not available): accuracy of the i-th best prediction of head k
    = 0.62 * 0.78**k * 0.45**i, i.e. later heads are less accurate and each further rank is about
    half as likely as the one before.  Pure data, no method arithmetic."""
    import numpy as np
    k = np.arange(K, dtype=np.float64)[:, None]
    i = np.arange(S, dtype=np.float64)[None, :]
    return 0.62 * 0.78 ** k * 0.45 ** i
