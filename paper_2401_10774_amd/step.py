"""One whole verification step as a sequence of library calls on preallocated device buffers.

Holds the tensors of one workload and enqueues, in order, the calls of include/medusa.h:
heads -> top-k/tree -> tree attention -> LM-head logits of the tree tokens -> acceptance ->
KV commit.  Nothing is computed here; the class only owns buffers and passes pointers.
"""
from __future__ import annotations

import math
from typing import Dict, Optional

import torch

from . import binding as B_


class VerificationStep:
    """Buffers and launch sequence of one Medusa verification iteration (Sec. 2 of the paper).

    ``dev`` maps tensor names to device tensors: h_last [B,d], hidden_tree [B,T,d], w1 [K,d,d],
    w2 [K,V,d], w_lm [V,d], q [B,Hq,T,D], k_tree/v_tree [NL,B,Hkv,T,D], k_cache/v_cache
    [NL,B,Hkv,Lcap,D], prefix_len [B] int32.
    """

    def __init__(self, dev: Dict[str, torch.Tensor], tree: B_.MedusaTree, mode: str = "greedy",
                 temperature: float = 1.0, eps: float = 0.0, delta: float = 0.0, fused_accept: bool = False):
        self.t = dev
        self.tree = tree
        self.mode, self.temperature, self.eps, self.delta = mode, temperature, eps, delta
        h = dev["h_last"]
        device = h.device
        self.B, self.d = h.shape
        self.K, self.V, _ = dev["w2"].shape
        _, self.Hq, self.T, self.D = dev["q"].shape
        self.NL, _, self.Hkv, self.Lcap, _ = dev["k_cache"].shape
        self.scale = 1.0 / math.sqrt(self.D)
        f32 = dict(dtype=torch.float32, device=device)
        i32 = dict(dtype=torch.int32, device=device)
        B, K, V, T = self.B, self.K, self.V, self.T
        self.resid = torch.empty((B, K, self.d), dtype=h.dtype, device=device)
        self.medusa_logits = torch.empty((B, K, V), **f32)
        self.lm_logits_last = torch.empty((B, 1, V), **f32)
        self.topk_ids = torch.empty((B, tree.K, max(tree.S, 1)), **i32)
        self.tree_tokens = torch.empty((B, T), **i32)
        self.position_ids = torch.empty((B, T), **i32)
        self.attn_out = torch.empty_like(dev["q"])
        self.verify_logits = torch.empty((B * T, 1, V), **f32)
        self.accept_out = (torch.empty(B, **i32), torch.empty(B, **i32), torch.empty((B, tree.K + 1), **i32),
                           torch.empty((B, tree.K + 1), **i32), torch.empty(B, **i32))
        self.ws_topk = B_._scratch(B_.lib().medusa_topk_tree_workspace_bytes(B, tree.K), device)
        self.ws_attn = B_._scratch(B_.tree_attention_workspace_bytes(B, self.Hq, self.Hkv, T, self.D, self.Lcap), device)
        self.ws_accept = B_._scratch(B_.medusa_accept_workspace_bytes(B, T, V), device)
        # fused_accept: where the shape has it (many tree rows), the LM-head kernel also leaves the acceptance
        # step's row reductions behind (medusa_verify_logits / medusa_accept_fused) instead of medusa_heads +
        # medusa_accept.  Off by default: measured on MI355X the reductions cost the GEMM's epilogue more
        # (B = 16: +33 us, B = 4: +18 us) than the lighter acceptance kernel gives back (-16 us, -7 us).
        self.fused = bool(fused_accept) and bool(B_.lib().medusa_verify_fused_available(B * T, self.d, V, B_._dtype_code(h)))
        self.ws_stats = B_._scratch(B_.lib().medusa_verify_stats_bytes(B * T, V) if self.fused else 0, device)
        self.w_lm3 = dev["w_lm"].view(1, V, self.d)
        self.hidden_rows = dev["hidden_tree"].view(B * T, self.d)
        self.prefix_len0 = dev["prefix_len"].clone()
        self.next_prefix_len = None
        self.w1_sets = [dev["w1"]]
        self.w_lm_sets = [self.w_lm3]
        self._plans = {}

    def prepare(self) -> None:
        """The LM head's logits at the last accepted position: in a running decoder they come out of the
        previous step's verification pass; here they are produced once, outside the step."""
        B_.medusa_heads(self.t["h_last"], None, self.w_lm3, None, self.lm_logits_last)

    def reset_prefix(self) -> None:
        self.t["prefix_len"].copy_(self.prefix_len0)

    def commit_out_of_place(self) -> torch.Tensor:
        """Have kv_commit write the advanced lengths to a second array (returned) and leave prefix_len as
        it is, so that the same step can be enqueued again and again on the same inputs."""
        if self.next_prefix_len is None:
            self.next_prefix_len = torch.empty_like(self.t["prefix_len"])
            self._plans = {}
        return self.next_prefix_len

    def add_weight_copies(self, n_w1: int, n_w_lm: int) -> None:
        """Keep n copies of W1 and of the LM head; run(wset=i) reads copy i % n.  A benchmark rotates them so
        that no step finds these weights in the last-level cache (in a decoder the whole backbone streams
        through between two verification steps)."""
        while len(self.w1_sets) < n_w1:
            self.w1_sets.append(self.w1_sets[0].clone())
        while len(self.w_lm_sets) < n_w_lm:
            self.w_lm_sets.append(self.w_lm_sets[0].clone())
        self._plans = {}

    def _calls(self, layer: int, wset: int = 0):
        """The step's library calls with their arguments marshalled once (pointers into layer `layer`,
        weight copies `wset`)."""
        key = (layer, wset % len(self.w1_sets), wset % len(self.w_lm_sets))
        if key in self._plans:
            return self._plans[key]
        w1, w_lm3 = self.w1_sets[key[1]], self.w_lm_sets[key[2]]
        L, t, tree = B_.lib(), self.t, self.tree
        p = lambda x: x.data_ptr()
        code = B_._dtype_code(t["h_last"])
        mode = {"greedy": B_.MEDUSA_GREEDY, "typical": B_.MEDUSA_TYPICAL}[self.mode]
        B, K, V, T, d = self.B, self.K, self.V, self.T, self.d
        nbytes = lambda x: x.numel() * x.element_size()
        kt, vt, kc, vc = (t[n][layer] for n in ("k_tree", "v_tree", "k_cache", "v_cache"))
        a = self.accept_out
        pre = [
            ("medusa_heads", L.medusa_heads, (p(t["h_last"]), p(w1), p(t["w2"]), p(self.resid),
                                              p(self.medusa_logits), B, d, V, K, code)),
            ("medusa_topk_tree", L.medusa_topk_tree, (p(self.medusa_logits), p(self.lm_logits_last), tree.handle,
                                                      p(t["prefix_len"]), B, V, K, p(self.topk_ids),
                                                      p(self.tree_tokens), p(self.position_ids), p(self.ws_topk),
                                                      nbytes(self.ws_topk))),
            ("tree_attention", L.tree_attention, (p(t["q"]), p(kt), p(vt), p(kc), p(vc), p(t["prefix_len"]),
                                                  tree.handle, p(self.attn_out), B, self.Hq, self.Hkv, self.D,
                                                  self.Lcap, self.scale, code, p(self.ws_attn), nbytes(self.ws_attn))),
            ("medusa_verify_logits", L.medusa_verify_logits,
             (p(self.hidden_rows), p(w_lm3), p(self.verify_logits), p(self.ws_stats), nbytes(self.ws_stats), B * T, d, V, code,
              mode, self.temperature)) if self.fused else
            ("medusa_heads", L.medusa_heads, (p(self.hidden_rows), None, p(w_lm3), None, p(self.verify_logits),
                                              B * T, d, V, 1, code)),
        ]
        accept_scan = ("medusa_accept", L.medusa_accept, (p(self.verify_logits), p(self.tree_tokens), tree.handle, B, V, mode,
                                                          self.temperature, self.eps, self.delta, p(a[0]), p(a[1]), p(a[2]),
                                                          p(a[3]), p(a[4]), p(self.ws_accept), nbytes(self.ws_accept)))
        accept_fused = ("medusa_accept_fused", L.medusa_accept_fused,
                        (p(self.verify_logits), p(self.ws_stats), p(self.tree_tokens), tree.handle, B, V, mode, self.temperature,
                         self.eps, self.delta, p(a[0]), p(a[1]), p(a[2]), p(a[3]), p(a[4])))
        self._accept_scan = accept_scan
        post = [
            accept_fused if self.fused else accept_scan,
            ("kv_commit", L.kv_commit, (p(t["k_cache"]), p(t["v_cache"]), p(t["k_tree"]), p(t["v_tree"]), p(a[2]),
                                        int(a[2].shape[1]), p(a[0]), p(t["prefix_len"]),
                                        None if self.next_prefix_len is None else p(self.next_prefix_len),
                                        self.NL, B, self.Hkv, T,
                                        self.D, self.Lcap, code)),
        ]
        self._plans[key] = (pre, post)
        return self._plans[key]

    def run(self, attn_layer: int = 0, plant=None, wset: int = 0, heads_events=None, backbone=None) -> None:
        """Enqueue one step on the current stream.  `plant`, if given, may edit the verification logits
        between the LM-head GEMM and acceptance (parity tests use it to force long accepted paths).
        `heads_events`: three raw hipEvent_t handles recorded before, between and after the two kernels
        of the heads call (medusa_heads_timed) -- a benchmark's way to time them inside a running step.
        `backbone`: a callable that enqueues a stack of decoder blocks on the tree tokens in place of the
        single tree_attention call (forward.TreeBackbone.run): it reads position_ids, prefix_len and the
        caches and fills k_tree, v_tree and hidden_tree, which the rest of the step then uses."""
        stream = torch.cuda.current_stream().cuda_stream
        pre, post = self._calls(attn_layer, wset)
        for i, (name, fn, args) in enumerate(pre):
            if name == "tree_attention" and backbone is not None:
                backbone()
                continue
            if i == 0 and heads_events is not None:
                rc = B_.lib().medusa_heads_timed(*args, stream, *heads_events)
            else:
                rc = fn(*args, stream)
            if rc != 0:
                B_._check(rc, name)
        if plant is not None:
            plant(self.verify_logits.view(self.B, self.T, self.V), self.tree_tokens)
        for i, (name, fn, args) in enumerate(post):
            if i == 0 and plant is not None and self.fused:
                name, fn, args = self._accept_scan     # edited logits: the GEMM's row reductions no longer describe them
            rc = fn(*args, stream)
            if rc != 0:
                B_._check(rc, name)

    def carry_over(self) -> None:
        """Enqueue the hand-over to the next step (Fig. 1): h_last and the LM logits of the last position
        become the rows of the last accepted node.  The caller then supplies the next forward pass's
        hidden_tree, q, k_tree and v_tree (in place) and calls run() again; prefix_len has already grown."""
        stream = torch.cuda.current_stream().cuda_stream
        t = self.t
        rc = B_.lib().medusa_carry_over(t["hidden_tree"].data_ptr(), self.verify_logits.data_ptr(),
                                        self.accept_out[1].data_ptr(), t["h_last"].data_ptr(),
                                        self.lm_logits_last.data_ptr(), self.B, self.T, self.d, self.V,
                                        B_._dtype_code(t["h_last"]), stream)
        if rc != 0:
            B_._check(rc, "medusa_carry_over")

    # ---- byte accounting (algorithmic, per step) --------------------------------------------
    def algorithmic_bytes(self, mean_prefix: float, mean_accept: float) -> Dict[str, float]:
        e = self.t["h_last"].element_size()
        B, K, V, d, T = self.B, self.K, self.V, self.d, self.T
        heads_w1 = K * d * d * e + B * d * e + B * K * d * e
        heads_w2 = K * V * d * e + B * K * d * e + B * K * V * 4
        verify = V * d * e + B * T * d * e + B * T * V * 4
        topk = B * (K + 1) * V * 4
        attn = B * (2 * self.Hkv * mean_prefix * self.D + 2 * self.Hq * T * self.D + 2 * self.Hkv * T * self.D) * e
        accept = B * T * V * 4
        commit = self.NL * B * self.Hkv * mean_accept * self.D * e * 2 * 2
        parts = dict(heads_w1=heads_w1, heads_w2=heads_w2, topk=topk, attention=attn, verify=verify, accept=accept,
                     commit=commit)
        parts["total"] = sum(parts.values())
        return parts
