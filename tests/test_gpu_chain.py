"""Chained decoding steps on the GPU against the oracle run on the same chain (Fig. 1; Sec. 2 opening
paragraph: the accepted prefix is the context of the next step).

Every step uses what the previous one left behind: kv_commit grows prefix_len IN PLACE and appends
the accepted rows to every cache layer; the next step's tree attention and position ids read the
grown cache; medusa_carry_over hands the last accepted node's hidden state and LM logits to the
next step's heads and root.  The forward pass between two steps is absent here, so each step gets
freshly drawn q, k_tree, v_tree and hidden_tree (seeded), on both sides.  After every step: floating
point stages within tolerance, integer stages bit-exact against the oracle fed the device's own
logits, every cache layer and prefix_len byte-equal to the oracle's chain.
"""
import math

import numpy as np
import pytest
import torch

import paper_2401_10774_amd as M
from paper_2401_10774_amd.step import VerificationStep
from oracle import medusa_oracle as O
from workloads import TENSOR_IDS, draw_normal, make_step_inputs, scaled_config
from _harness import BOUND, bits, check_close, poison_tail, to_dev, to_host_bits, to_host_f64

pytestmark = pytest.mark.gpu

FRESH = ("q", "k_tree", "v_tree", "hidden_tree")


def step_picks(tree, B, seed, lengths=None):
    rng = np.random.default_rng(seed)
    picks = []
    for b in range(B):
        path = [int(n) for n in tree.paths[rng.integers(tree.n_leaves)] if n >= 0]
        n = int(rng.integers(1, len(path) + 1)) if lengths is None else min(lengths[b], len(path))
        picks.append(path[:n])
    return picks


def run_chain(label, cfg, n_steps, layers, plant_lengths=None, typical_edges=False):
    tree_g, tree_o = M.MedusaTree(branching=cfg.branching), O.tree_cartesian(cfg.branching)
    B, T, V, d = cfg.B, cfg.T, cfg.V, cfg.d
    scale = 1.0 / math.sqrt(cfg.D)
    x = make_step_inputs(cfg)
    x["k_cache"] = poison_tail(x["k_cache"], x["prefix_len"])
    x["v_cache"] = poison_tail(x["v_cache"], x["prefix_len"])
    step = VerificationStep({k: to_dev(v) for k, v in x.items()}, tree_g, cfg.accept, cfg.temperature, cfg.eps, cfg.delta)
    step.prepare()
    seen_lengths, prev_next_root = set(), None
    for s in range(n_steps):
        print(f"[chain {label}] step {s} layer {layers[s]} prefix {x['prefix_len'].tolist()}", flush=True)
        if s > 0:                                    # the next forward pass's rows, same bytes on both sides
            for name in FRESH:
                x[name] = draw_normal(cfg.seed * 1000 + s, TENSOR_IDS[name], x[name].shape, 1.0, cfg.dtype)
                step.t[name].copy_(to_dev(x[name]))
        picks = plant_dev = plant_host = None
        if cfg.accept == "greedy":
            picks = step_picks(tree_o, B, cfg.seed * 77 + s, None if plant_lengths is None else plant_lengths[s])

            def plant_dev(logits, tokens, picks=picks):
                for b, path in enumerate(picks):
                    for j in range(1, len(path)):
                        logits[b, path[j - 1], tokens[b, path[j]].long()] += 20.0

            def plant_host(logits, tokens, picks=picks):
                logits = logits.copy()
                for b, path in enumerate(picks):
                    for j in range(1, len(path)):
                        logits[b, path[j - 1], tokens[b, path[j]]] += 20.0
                return logits

        pl_before = x["prefix_len"].copy()
        assert np.array_equal(step.t["prefix_len"].cpu().numpy(), pl_before)
        assert np.array_equal(to_host_bits(step.t["h_last"]), bits(x["h_last"]))      # carried over bit for bit
        layer = layers[s]
        step.run(layer, plant=plant_dev)
        torch.cuda.synchronize()

        # heads and the root's logits
        g_heads = step.medusa_logits.cpu().numpy()
        g_lm = step.lm_logits_last.view(B, V).cpu().numpy()
        r_heads, _ = O.medusa_heads_ref(x["h_last"], x["w1"], x["w2"], cfg.dtype)
        r_lm = O.medusa_heads_ref(x["h_last"], None, x["w_lm"][None], cfg.dtype)[0][:, 0]
        check_close(f"chain {label} step {s}", "heads", g_heads, r_heads, cfg.dtype)
        check_close(f"chain {label} step {s}", "lm_logits", g_lm, r_lm, cfg.dtype)
        # tokens and positions: exact on the device's logits, and at the grown lengths
        r_topk, r_tokens, r_pos = O.medusa_topk_tree_ref(g_heads, g_lm, tree_o, pl_before)
        g_tokens = step.tree_tokens.cpu().numpy()
        assert np.array_equal(step.topk_ids.cpu().numpy(), r_topk) and np.array_equal(g_tokens, r_tokens)
        assert np.array_equal(step.position_ids.cpu().numpy(), r_pos)
        if prev_next_root is not None:               # the root is what the last step predicted after its accepted prefix
            assert np.array_equal(g_tokens[:, 0], prev_next_root)
        # attention over the grown cache of this step's layer
        r_attn = O.tree_attention_ref(x["q"], x["k_tree"][layer], x["v_tree"][layer], x["k_cache"][layer],
                                      x["v_cache"][layer], pl_before, tree_o, scale)
        g_attn = to_host_f64(step.attn_out)
        assert np.isfinite(g_attn).all()
        check_close(f"chain {label} step {s}", "attention", g_attn, r_attn, cfg.dtype, rounded_output=True)
        # the oracle's own step on the same state (its caches and prefix_len advance in place)
        res = O.verification_step_ref(x, tree_o, cfg.dtype, scale, cfg.accept, cfg.temperature, cfg.eps, cfg.delta,
                                      attn_layer=layer, plant=plant_host)
        g_ver = step.verify_logits.view(B, T, V).cpu().numpy()
        check_close(f"chain {label} step {s}", "verify_logits", g_ver, res.verify_logits, cfg.dtype)
        # acceptance: exact on the device's logits; the oracle's own chain must agree or name a near-tie
        acc = O.medusa_accept_ref(g_ver, g_tokens, tree_o, cfg.accept, cfg.temperature, cfg.eps, cfg.delta)
        g_alen, g_best, g_path, g_toks, g_next = (t.cpu().numpy() for t in step.accept_out)
        if cfg.accept == "typical" and not np.array_equal(g_path, acc.path_nodes):
            assert acc.margin[:, 1:].min() < 1e-4, "typical acceptance differs with no decision near its threshold"
            pytest.fail("tie-ambiguous typical decision at this seed")
        for got, want in ((g_alen, acc.accept_len), (g_best, acc.best_node), (g_path, acc.path_nodes),
                          (g_toks, acc.accepted_tokens), (g_next, acc.next_root)):
            assert np.array_equal(got, want)
        if not (np.array_equal(res.tree_tokens, g_tokens) and np.array_equal(res.accept.path_nodes, g_path)
                and np.array_equal(res.accept.next_root, g_next)):
            near = min(float(res.accept.margin[:, 1:].min()), float(res.accept.argmax_gap.min()))
            pytest.fail(f"oracle chain and device chain part ways at step {s} (smallest oracle margin {near:.2e})")
        if picks is not None:
            assert g_alen.tolist() == [len(p) for p in picks]
        seen_lengths.update(int(a) for a in g_alen)
        # commit: lengths grown in place, every layer byte-equal to the oracle's cache
        assert np.array_equal(step.t["prefix_len"].cpu().numpy(), pl_before + g_alen)
        assert np.array_equal(x["prefix_len"], pl_before + g_alen)
        for l in range(cfg.NL):
            assert np.array_equal(to_host_bits(step.t["k_cache"][l]), bits(x["k_cache"][l])), f"k layer {l} step {s}"
            assert np.array_equal(to_host_bits(step.t["v_cache"][l]), bits(x["v_cache"][l])), f"v layer {l} step {s}"
        # hand-over
        step.carry_over()
        torch.cuda.synchronize()
        x["h_last"] = np.stack([x["hidden_tree"][b, g_best[b]] for b in range(B)])
        assert np.array_equal(to_host_bits(step.lm_logits_last.view(B, V)),
                              bits(np.stack([g_ver[b, g_best[b]] for b in range(B)])))
        prev_next_root = g_next
    return seen_lengths


def test_chain_greedy_ragged_batch_bf16():
    """B = 4, 89-token tree (mask crosses the 64-bit word), GQA, three cache layers attended in turn,
    planted accept lengths that cover 1..K+1 and differ per sequence and step."""
    cfg = scaled_config("C4", B=4, d=512, Hq=8, Hkv=2, D=128, V=4096, L_min=60, L_max=300, Lcap=384, NL=3)
    lengths = [[1, 6, 3, 2], [4, 1, 6, 5], [6, 6, 1, 3], [2, 5, 4, 1], [3, 2, 5, 6]]
    seen = run_chain("greedy-bf16", cfg, 5, [0, 2, 1, 2, 0], plant_lengths=lengths)
    assert seen == {1, 2, 3, 4, 5, 6}


def test_chain_typical_from_an_empty_prefix_bf16():
    """Typical acceptance, one sequence starting with no prefix at all; lengths are whatever the
    random logits give (ragged), the chain still has to agree step by step."""
    cfg = scaled_config("C5", B=3, d=256, Hq=4, Hkv=4, D=128, V=2048, L_min=0, L_max=40, Lcap=128, NL=2)
    x = make_step_inputs(cfg, names=["prefix_len"])
    assert x["prefix_len"].min() >= 0
    seen = run_chain("typical-bf16", cfg, 4, [1, 0, 1, 0])
    assert min(seen) >= 1


def test_chain_fp32_tiny():
    cfg = scaled_config("C1", B=3, L_min=5, L_max=100, NL=2, Lcap=160)
    lengths = [[3, 1, 2], [1, 3, 3], [2, 2, 1], [3, 3, 3]]
    seen = run_chain("greedy-f32", cfg, 4, [0, 1, 1, 0], plant_lengths=lengths)
    assert seen == {1, 2, 3}


def test_chain_7b_shapes_three_steps():
    """The 7B-shaped workload itself (d = 4096, V = 32000, 32 heads x 128, 64-node tree, prefix 1024) over
    three chained steps on two cache layers: the launch configuration the benchmark times, with the
    in-place commit the benchmark avoids."""
    cfg = scaled_config("C2", NL=2)
    seen = run_chain("7B", cfg, 3, [0, 1, 0], plant_lengths=[[4], [1], [5]])
    assert seen == {1, 4, 5}
