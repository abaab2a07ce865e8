"""A stack of simplified decoder blocks inside the verification step (App. G operator table chained over
layers; Fig. 1: the tree tokens' K and V of every layer are what kv_commit appends): heads -> top-k/tree
-> NL blocks, each writing k_tree[l], v_tree[l] and feeding the next -> LM head on the last block's output
-> acceptance -> commit of all layers.

Oracle protocol: every block is checked stage by stage from the GPU's own inputs of that stage
(simplified-block operators of the oracle), the step's tail as in the other step tests (floating point
within tolerance, integers exact on the device's logits, caches byte-equal to kv_commit_ref applied to the
device's own k_tree / v_tree).  Then the whole step is enqueued again in one go, without a host
synchronisation inside, and must reproduce every output bit for bit.  Two passes are chained: the second
starts from the first one's carry-over (hidden state and logits of its last accepted node) and attends,
in every layer, the cache the first one's commit grew.
"""
import math

import numpy as np
import pytest
import torch

import paper_2401_10774_amd as M
from paper_2401_10774_amd.forward import TreeBackbone, alloc_qkv
from paper_2401_10774_amd.step import VerificationStep
from oracle import medusa_oracle as O
from workloads import draw_normal, make_step_inputs, scaled_config
from _harness import bits, check_close, to_dev, to_host_bits, to_host_f64

pytestmark = pytest.mark.gpu


def forward_case(cfg, inter, seed, n_pass=2):
    tree_g, tree_o = M.MedusaTree(branching=cfg.branching), O.tree_cartesian(cfg.branching)
    B, T, V, h, NL, Hq, Hkv, D = cfg.B, cfg.T, cfg.V, cfg.d, cfg.NL, cfg.Hq, cfg.Hkv, cfg.D
    dt = torch.bfloat16
    x = make_step_inputs(cfg)
    ws = []
    for l in range(NL):
        w = {n: draw_normal(seed, 10 * (l + 1) + i, shape, 1.0 / math.sqrt(shape[1]), cfg.dtype)
             for i, (n, shape) in enumerate((("wq", (Hq * D, h)), ("wk", (Hkv * D, h)), ("wv", (Hkv * D, h)),
                                             ("wu", (inter, Hq * D)), ("wg", (inter, Hq * D)), ("wd", (h, inter))))}
        ws.append(w)
    q, k_tree, v_tree = alloc_qkv(NL, B, Hq, Hkv, T, D, dt)
    dev = {k: to_dev(v) for k, v in x.items() if k not in ("k_tree", "v_tree", "q")}
    dev["k_tree"], dev["v_tree"], dev["q"] = k_tree, v_tree, q[0]
    step = VerificationStep(dev, tree_g, cfg.accept, cfg.temperature, cfg.eps, cfg.delta)
    step.prepare()
    dws = [{"w_qkv": to_dev(np.concatenate([w["wq"], w["wk"], w["wv"]], axis=0)),
            "w_gu": M.interleave_gate_up(to_dev(w["wg"]), to_dev(w["wu"])), "wd": to_dev(w["wd"]),
            "wu": to_dev(w["wu"]), "wg": to_dev(w["wg"])} for w in ws]
    fused = B * T <= 160            # (above that, and below the large-tile range, gate and up take two calls and `up` is stored)
    bb = TreeBackbone(tree_g, B, h, Hq, Hkv, D, inter, cfg.Lcap, dws, q, k_tree, v_tree, dev["k_cache"], dev["v_cache"],
                      dev["prefix_len"], step.position_ids)
    hidden_rows = dev["hidden_tree"].view(B * T, h)
    scale, theta = 1.0 / math.sqrt(D), 10000.0
    host = {"k_cache": x["k_cache"], "v_cache": x["v_cache"], "prefix_len": x["prefix_len"].copy(), "h_last": x["h_last"]}
    x0_dev = torch.empty((B * T, h), dtype=dt, device="cuda")

    def checked_backbone():
        torch.cuda.synchronize()
        pl0 = host["prefix_len"]
        pos = step.position_ids.cpu().numpy()
        assert np.array_equal(pos, pl0[:, None] + np.asarray(tree_o.depth, np.int32)[None, :])
        xin = x0_dev
        for l in range(NL):
            out = hidden_rows if l == NL - 1 else bb.x_mid[l & 1]
            x_host = to_host_f64(xin)
            bb.run_layer(l, xin, out)
            torch.cuda.synchronize()
            name = f"forward layer {l}"
            g = {n: to_host_f64(t) for n, t in (("q", q[l]), ("k", k_tree[l]), ("v", v_tree[l]), ("attn", bb.block.attn),
                                                ("act", bb.block.act), ("out", out))}
            w = ws[l]
            want_q = O.rope_ref(O.to_heads(O.tree_linear_ref(x_host, w["wq"], cfg.dtype), B, T, Hq), pos, theta, cfg.dtype)
            want_k = O.rope_ref(O.to_heads(O.tree_linear_ref(x_host, w["wk"], cfg.dtype), B, T, Hkv), pos, theta, cfg.dtype)
            want_v = O.to_heads(O.tree_linear_ref(x_host, w["wv"], cfg.dtype), B, T, Hkv)
            # (two roundings deep -- projection, then rotation -- for q and k)
            check_close(name, "q", g["q"], want_q, cfg.dtype, kind="rounded2", bound=2 ** -5)
            check_close(name, "k", g["k"], want_k, cfg.dtype, kind="rounded2", bound=2 ** -5)
            check_close(name, "v", g["v"], want_v, cfg.dtype, kind="rounded2")
            want_attn = O.round_to_storage(O.tree_attention_ref(g["q"], g["k"], g["v"], host["k_cache"][l], host["v_cache"][l], pl0,
                                                                tree_o, scale), cfg.dtype)
            check_close(name, "attn", g["attn"], want_attn, cfg.dtype, kind="rounded2")
            a_tok = O.from_heads(g["attn"])
            if fused:
                check_close(name, "act", g["act"], O.tree_swiglu_ref(a_tok, w["wg"], w["wu"], cfg.dtype), cfg.dtype, kind="rounded2")
            else:
                g_up = to_host_f64(bb.block.up)
                check_close(name, "up", g_up, O.tree_linear_ref(a_tok, w["wu"], cfg.dtype), cfg.dtype, kind="rounded2")
                check_close(name, "act", g["act"], O.tree_linear_ref(a_tok, w["wg"], cfg.dtype, mul=g_up), cfg.dtype, kind="rounded2")
            check_close(name, "out", g["out"], O.tree_linear_ref(g["act"], w["wd"], cfg.dtype), cfg.dtype, kind="rounded2")
            xin = out

    def tail_outputs():
        torch.cuda.synchronize()
        return ([to_host_bits(t) for t in (q, k_tree, v_tree, hidden_rows, dev["k_cache"], dev["v_cache"])] +
                [step.verify_logits.cpu().numpy().copy(), dev["prefix_len"].cpu().numpy().copy()] +
                [t.cpu().numpy().copy() for t in step.accept_out] + [step.tree_tokens.cpu().numpy().copy()])

    seen = []
    for s_ in range(n_pass):
        # the pass's input states (the embedding of the tree tokens is outside this library: drawn)
        x0_dev.copy_(to_dev(draw_normal(seed + s_, 0, (B * T, h), 1.0, cfg.dtype)))
        pl0 = host["prefix_len"].copy()
        state = [t.clone() for t in (dev["k_cache"], dev["v_cache"], dev["prefix_len"], dev["h_last"], step.lm_logits_last)]
        assert np.array_equal(to_host_bits(dev["h_last"]), bits(host["h_last"]))
        step.run(backbone=checked_backbone)
        first = tail_outputs()
        # the tail on the stack's output
        g_hidden = to_host_f64(hidden_rows)
        g_ver = step.verify_logits.view(B, T, V).cpu().numpy()
        r_ver = O.medusa_heads_ref(g_hidden, None, x["w_lm"][None], cfg.dtype)[0][:, 0].reshape(B, T, V)
        check_close(f"forward pass {s_}", "verify_logits", g_ver, r_ver, cfg.dtype)
        g_tokens = step.tree_tokens.cpu().numpy()
        acc = O.medusa_accept_ref(g_ver, g_tokens, tree_o, cfg.accept, cfg.temperature, cfg.eps, cfg.delta)
        g_alen, g_best, g_path, g_toks, g_next = (t.cpu().numpy() for t in step.accept_out)
        for got, want in ((g_alen, acc.accept_len), (g_best, acc.best_node), (g_path, acc.path_nodes),
                          (g_toks, acc.accepted_tokens), (g_next, acc.next_root)):
            assert np.array_equal(got, want)
        # commit of every layer from the device's own K and V of the tree tokens
        kcb, vcb, pl = bits(host["k_cache"]).copy(), bits(host["v_cache"]).copy(), pl0.copy()
        O.kv_commit_ref(kcb, vcb, to_host_bits(k_tree), to_host_bits(v_tree), g_path, g_alen, pl)
        assert np.array_equal(to_host_bits(dev["k_cache"]), kcb) and np.array_equal(to_host_bits(dev["v_cache"]), vcb)
        assert np.array_equal(dev["prefix_len"].cpu().numpy(), pl) and np.array_equal(pl, pl0 + g_alen)
        seen += [int(a) for a in g_alen]

        # once more in one go (no host synchronisation inside) from the same state: bit-identical
        for t, saved in zip((dev["k_cache"], dev["v_cache"], dev["prefix_len"], dev["h_last"], step.lm_logits_last), state):
            t.copy_(saved)
        for t in (q, k_tree, v_tree, hidden_rows):
            t.zero_()
        step.run(backbone=lambda: bb.run(x0_dev, hidden_rows))
        for a_, b_ in zip(first, tail_outputs()):
            assert np.array_equal(a_, b_)
        # hand-over to the next pass (Fig. 1): hidden state and logits of the last accepted node; the caches have grown
        step.carry_over()
        torch.cuda.synchronize()
        host["k_cache"], host["v_cache"], host["prefix_len"] = kcb, vcb, pl
        host["h_last"] = to_host_bits(hidden_rows.view(B, T, h))[np.arange(B), g_best]
        assert np.array_equal(to_host_bits(step.lm_logits_last.view(B, V)), bits(np.stack([g_ver[b_, g_best[b_]] for b_ in range(B)])))
    return seen


def test_forward_three_layers_mha_bf16():
    """Hq == Hkv: one projection call per layer fills q[l], k_tree[l], v_tree[l]."""
    cfg = scaled_config("C2", B=2, d=256, Hq=4, Hkv=4, D=64, V=2048, L_min=30, L_max=90, Lcap=128, NL=3)
    forward_case(cfg, 512, 900)


def test_forward_two_layers_gqa_bf16():
    """Grouped-query attention: Q alone, K and V from one call; 89-token tree, ragged batch of three."""
    cfg = scaled_config("C4", B=3, d=256, Hq=8, Hkv=2, D=64, V=1536, L_min=5, L_max=200, Lcap=256, NL=2)
    forward_case(cfg, 768, 901)
