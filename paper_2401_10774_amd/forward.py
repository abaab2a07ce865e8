"""A stack of simplified decoder blocks (App. G) on the tree tokens, chained: the verification pass of
a whole backbone as far as this library covers it (linear layers, rotary embedding, tree attention; no
embedding, norms, output projection or residual stream).  Layer l reads the hidden states layer l - 1
wrote, attends its own cache, and leaves the K and V of the tree tokens in k_tree[l], v_tree[l] --
the rows kv_commit later copies into the cache -- so that together with step.VerificationStep one
decoding step runs end to end: heads -> top-k/tree -> NL blocks -> LM head -> acceptance -> commit.
Argument marshalling only: every operator runs in the HIP library."""
from __future__ import annotations

from typing import Dict, List

import torch

from . import binding as _b
from .block import SimplifiedBlock


def alloc_qkv(NL: int, B: int, Hq: int, Hkv: int, T: int, D: int, dtype: torch.dtype, device="cuda"):
    """(q, k_tree, v_tree) of a stack: [NL, B, Hq, T, D] and twice [NL, B, Hkv, T, D].  With Hq == Hkv the
    three are slices of one allocation, equally spaced per layer, so that one projection call per layer
    fills q[l], k_tree[l] and v_tree[l]; otherwise k_tree and v_tree are, and share one."""
    if Hq == Hkv:
        qkv = torch.empty((3, NL, B, Hq, T, D), dtype=dtype, device=device)
        return qkv[0], qkv[1], qkv[2]
    kv = torch.empty((2, NL, B, Hkv, T, D), dtype=dtype, device=device)
    return torch.empty((NL, B, Hq, T, D), dtype=dtype, device=device), kv[0], kv[1]


class TreeBackbone:
    """weights: one dict per layer with w_qkv [(Hq + 2 Hkv) D, h] (rows of W_Q, W_K, W_V stacked),
    w_gu [2 inter, Hq D] (binding.interleave_gate_up of W_g and W_u), wd [h, inter], and -- only for
    row counts where gate and up take two calls -- wu, wg [inter, Hq D].
    q, k_tree, v_tree: from alloc_qkv; k_tree, v_tree [NL, B, Hkv, T, D] and k_cache, v_cache
    [NL, B, Hkv, Lcap, D], prefix_len [B], position_ids [B, T] are the step's tensors."""

    def __init__(self, tree: "_b.MedusaTree", B: int, h: int, Hq: int, Hkv: int, D: int, inter: int, Lcap: int,
                 weights: List[Dict[str, torch.Tensor]], q: torch.Tensor, k_tree: torch.Tensor, v_tree: torch.Tensor,
                 k_cache: torch.Tensor, v_cache: torch.Tensor, prefix_len: torch.Tensor, position_ids: torch.Tensor,
                 theta: float = 10000.0):
        self.NL = len(weights)
        self.B, self.T, self.h, self.Hq, self.Hkv, self.D, self.inter = B, tree.T, h, Hq, Hkv, D, inter
        self.weights, self.k_cache, self.v_cache = weights, k_cache, v_cache
        self.q, self.k_tree, self.v_tree = q, k_tree, v_tree
        self.prefix_len, self.position_ids = prefix_len, position_ids
        self.scale = 1.0 / float(D) ** 0.5
        dtype, device = q.dtype, q.device
        self.block = SimplifiedBlock(tree, B, h, Hq, Hkv, D, inter, Lcap, dtype, device, theta)
        self.x_mid = [torch.empty((B * tree.T, h), dtype=dtype, device=device) for _ in range(2)]
        self._views = []
        for w in weights:
            wq = w["w_qkv"][:Hq * D]
            wk = w["w_qkv"][Hq * D:(Hq + Hkv) * D]
            wv = w["w_qkv"][(Hq + Hkv) * D:]
            self._views.append((wq, wk, wv))

    def run_layer(self, l: int, x: torch.Tensor, out: torch.Tensor) -> torch.Tensor:
        """Enqueue block l: x [B*T, h] -> out [B*T, h]; q[l], k_tree[l], v_tree[l] are written on the way."""
        wq, wk, wv = self._views[l]
        w = self.weights[l]
        # (w_u and w_g are only read where gate and up take two calls; the fused weights always serve the
        # tree-token range and large batches)
        return self.block.run(x, wq, wk, wv, w.get("wu"), w.get("wg"), w["wd"], self.k_cache[l], self.v_cache[l],
                              self.prefix_len, self.position_ids, self.scale, w_gu=w["w_gu"],
                              qkv=(self.q[l], self.k_tree[l], self.v_tree[l]), out=out)

    def run(self, x0: torch.Tensor, hidden_tree: torch.Tensor) -> torch.Tensor:
        """Enqueue all layers: x0 [B*T, h] (the tree tokens' input states) -> hidden_tree [B*T, h]."""
        x = x0
        for l in range(self.NL):
            out = hidden_tree if l == self.NL - 1 else self.x_mid[l & 1]
            x = self.run_layer(l, x, out)
        return x
