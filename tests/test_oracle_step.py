"""Pins for the oracle's chained step (Sec. 2, opening paragraph: generate, process, accept; Fig. 1:
the accepted prefix is the next step's context).

verification_step_ref only composes the stage functions, so what can go wrong in it is glue: a
wrong cache layer, a wrong reshape of the tree rows, a wrong call order, a commit that is not fed
the acceptance result.  Two kinds of pins catch that: (a) its outputs against the stage functions
composed by hand with glue written a second time here, and (b) outcomes known by construction on a
tiny case, checked with scalar Python loops that use neither the step nor the stage functions.
"""
import math

import numpy as np
import pytest

from oracle import medusa_oracle as O
from workloads import draw_normal, get_config, make_step_inputs, scaled_config
from test_oracle_attention import causal_attention_scalar


def planted(picks):
    """Editor of the verification logits that makes, per sequence, one chosen tree path acceptable:
    +20 on the token of every path node in the row of the node before it."""
    def plant(logits, tokens):
        logits = logits.copy()
        for b, path in enumerate(picks):
            for j in range(1, len(path)):
                logits[b, path[j - 1], tokens[b, path[j]]] += 20.0
        return logits
    return plant


def seeded_picks(tree, B, seed):
    rng = np.random.default_rng(seed)
    picks = []
    for _ in range(B):
        path = [int(n) for n in tree.paths[rng.integers(tree.n_leaves)] if n >= 0]
        picks.append(path[:int(rng.integers(1, len(path) + 1))])
    return picks


def compose_by_hand(x, tree, cfg, attn_layer, plant):
    """The step written out a second time from the stage functions (different glue: explicit loops
    over sequences for the tree rows, caches copied instead of updated in place)."""
    B, T, d, V = cfg.B, tree.T, cfg.d, cfg.V
    scale = 1.0 / math.sqrt(cfg.D)
    heads, _ = O.medusa_heads_ref(x["h_last"], x["w1"], x["w2"], cfg.dtype)
    lm = np.stack([O.medusa_heads_ref(x["h_last"][b:b + 1], None, x["w_lm"][None], cfg.dtype)[0][0, 0] for b in range(B)])
    topk, tokens, pos = O.medusa_topk_tree_ref(heads, lm, tree, x["prefix_len"])
    attn = O.tree_attention_ref(x["q"], x["k_tree"][attn_layer], x["v_tree"][attn_layer], x["k_cache"][attn_layer],
                                x["v_cache"][attn_layer], x["prefix_len"], tree, scale)
    ver = np.empty((B, T, V))
    for b in range(B):
        ver[b] = O.medusa_heads_ref(x["hidden_tree"][b], None, x["w_lm"][None], cfg.dtype)[0][:, 0]
    if plant is not None:
        ver = plant(ver, tokens)
    acc = O.medusa_accept_ref(ver, tokens, tree, cfg.accept, cfg.temperature, cfg.eps, cfg.delta)
    kc, vc, pl = x["k_cache"].copy(), x["v_cache"].copy(), x["prefix_len"].copy()
    O.kv_commit_ref(kc, vc, x["k_tree"], x["v_tree"], acc.path_nodes, acc.accept_len, pl)
    return dict(heads=heads, lm=lm, topk=topk, tokens=tokens, pos=pos, attn=attn, ver=ver, acc=acc, kc=kc, vc=vc, pl=pl)


CASES = [
    ("C1", {}, 0, None),
    ("C1", {}, 0, 7),
    ("C2", dict(B=3, d=128, Hq=4, Hkv=2, D=32, V=257, L_min=20, L_max=70, Lcap=96, NL=3), 2, 11),
    ("C5", dict(B=4, d=64, Hq=4, Hkv=1, D=16, V=101, L_min=3, L_max=40, Lcap=64, NL=2), 1, None),   # typical, ragged
]


@pytest.mark.parametrize("name,over,attn_layer,plant_seed", CASES)
def test_step_equals_the_stage_functions_composed_by_hand(name, over, attn_layer, plant_seed):
    cfg = scaled_config(name, **over) if over else get_config(name)
    tree = O.tree_cartesian(cfg.branching)
    x = make_step_inputs(cfg)
    plant = planted(seeded_picks(tree, cfg.B, plant_seed)) if plant_seed is not None else None
    want = compose_by_hand(x, tree, cfg, attn_layer, plant)
    pl0 = x["prefix_len"].copy()
    res = O.verification_step_ref(x, tree, cfg.dtype, 1.0 / math.sqrt(cfg.D), cfg.accept, cfg.temperature, cfg.eps,
                                  cfg.delta, attn_layer=attn_layer, plant=plant)
    assert np.array_equal(res.medusa_logits, want["heads"])
    assert np.allclose(res.lm_logits_last, want["lm"], rtol=1e-14, atol=0)       # (row-at-a-time product: same sums, other blocking)
    assert np.array_equal(res.topk_ids, want["topk"]) and np.array_equal(res.tree_tokens, want["tokens"])
    assert np.array_equal(res.position_ids, want["pos"])
    assert np.array_equal(res.position_ids, pl0[:, None] + tree.depth[None, :])   # positions use the lengths BEFORE the commit
    assert np.array_equal(res.attn_out, want["attn"])
    assert np.allclose(res.verify_logits, want["ver"], rtol=1e-13, atol=1e-13)
    for f in ("accept_len", "best_node", "path_nodes", "accepted_tokens", "next_root"):
        assert np.array_equal(getattr(res.accept, f), getattr(want["acc"], f)), f
    assert np.array_equal(x["k_cache"], want["kc"]) and np.array_equal(x["v_cache"], want["vc"])
    assert np.array_equal(x["prefix_len"], want["pl"]) and res.prefix_len is x["prefix_len"]
    assert np.array_equal(x["prefix_len"], pl0 + res.accept.accept_len)
    if cfg.NL > 1:                                     # the attended layer matters: another layer gives another result
        other = O.tree_attention_ref(x["q"], x["k_tree"][0], x["v_tree"][0], want["kc"][0], want["vc"][0], pl0, tree,
                                     1.0 / math.sqrt(cfg.D))
        assert not np.allclose(other, res.attn_out)


def test_step_outcomes_known_by_construction_scalar_loops():
    """B = 2, tree (2, 2), NL = 2, attended layer 1, planted paths of lengths 3 and 2.  Everything the
    step returns is re-derived with Python floats: tokens from scalar dot products and a scalar
    top-k, attention from plain causal attention over prefix + path on layer 1's arrays, the
    logits row by row, the accepted path from the plant, the cache from row copies."""
    B, d, V, D, Hq, Hkv, NL, Lcap = 2, 8, 13, 4, 2, 1, 2, 10
    tree = O.tree_cartesian((2, 2))
    T, K = tree.T, tree.K
    seed = 91
    x = {
        "h_last": draw_normal(seed, 0, (B, d), 1.0, "f32"),
        "hidden_tree": draw_normal(seed, 1, (B, T, d), 1.0, "f32"),
        "w1": draw_normal(seed, 2, (K, d, d), 0.3, "f32"),
        "w2": draw_normal(seed, 3, (K, V, d), 0.3, "f32"),
        "w_lm": draw_normal(seed, 4, (V, d), 0.3, "f32"),
        "q": draw_normal(seed, 5, (B, Hq, T, D), 1.0, "f32"),
        "k_tree": draw_normal(seed, 6, (NL, B, Hkv, T, D), 1.0, "f32"),
        "v_tree": draw_normal(seed, 7, (NL, B, Hkv, T, D), 1.0, "f32"),
        "k_cache": draw_normal(seed, 8, (NL, B, Hkv, Lcap, D), 1.0, "f32"),
        "v_cache": draw_normal(seed, 9, (NL, B, Hkv, Lcap, D), 1.0, "f32"),
        "prefix_len": np.array([4, 2], np.int32),
    }
    kc0, vc0 = x["k_cache"].copy(), x["v_cache"].copy()
    picks = [[0, 2, 5], [0, 1]]                     # node 2 = rank tuple (1,), node 5 = (1, 0); node 1 = (0,)
    assert tree.nodes[2] == (1,) and tree.nodes[5] == (1, 0) and tree.nodes[1] == (0,)
    res = O.verification_step_ref(x, tree, "f32", 0.5, "greedy", 1.0, 0.0, 0.0, attn_layer=1, plant=planted(picks))

    dot = lambda a, b: math.fsum(float(p) * float(q) for p, q in zip(a, b))
    def top(row, s):
        return sorted(range(len(row)), key=lambda i: (-row[i], i))[:s]
    for b in range(B):
        h = [float(v) for v in x["h_last"][b]]
        root = top([dot(x["w_lm"][v], h) for v in range(V)], 1)[0]
        lists = []
        for k in range(K):
            u = [dot(x["w1"][k, j], h) for j in range(d)]
            r = [float(np.float32(uj / (1.0 + math.exp(-uj)) + hj)) for uj, hj in zip(u, h)]    # one rounding to storage
            lists.append(top([dot(x["w2"][k, v], r) for v in range(V)], 2))
        want_tokens = [root] + lists[0] + [lists[1][n[1]] for n in tree.nodes[3:]]
        assert res.tree_tokens[b].tolist() == want_tokens
        # verification logits: row t of sequence b is W_lm times hidden_tree[b, t]  (+20 where planted)
        path = picks[b]
        for t in range(T):
            row = [dot(x["w_lm"][v], x["hidden_tree"][b, t]) for v in range(V)]
            if t in path[:-1]:
                row[want_tokens[path[path.index(t) + 1]]] += 20.0
            assert np.allclose(res.verify_logits[b, t], row, rtol=1e-12, atol=1e-12)
        # accepted path = the planted one; the next root is the arg-max of the last accepted node's row
        a = len(path)
        assert res.accept.accept_len[b] == a and res.accept.best_node[b] == path[-1]
        assert res.accept.path_nodes[b].tolist() == path + [-1] * (K + 1 - a)
        assert res.accept.accepted_tokens[b, :a].tolist() == [want_tokens[n] for n in path]
        assert res.accept.next_root[b] == top([dot(x["w_lm"][v], x["hidden_tree"][b, path[-1]]) for v in range(V)], 1)[0]
        # attention on layer 1: each root-to-leaf path as a plain causal sequence behind the prefix
        L = [4, 2][b]
        assert res.position_ids[b].tolist() == [L + len(n) for n in tree.nodes]
        for g in range(Hq):
            for leaf_path in tree.paths:
                nodes = [int(n) for n in leaf_path if n >= 0]
                ks = kc0[1, b, 0, :L].tolist() + [x["k_tree"][1, b, 0, n].tolist() for n in nodes]
                vs = vc0[1, b, 0, :L].tolist() + [x["v_tree"][1, b, 0, n].tolist() for n in nodes]
                want = causal_attention_scalar([x["q"][b, g, n].tolist() for n in nodes], ks, vs, L, 0.5)
                for i, n in enumerate(nodes):
                    assert np.allclose(res.attn_out[b, g, n], want[i], rtol=1e-12, atol=1e-13)
        # commit: every layer gets the path's tree rows behind the prefix, nothing else moves
        assert x["prefix_len"][b] == L + a
        for l in range(NL):
            for j, n in enumerate(path):
                assert np.array_equal(x["k_cache"][l, b, 0, L + j], x["k_tree"][l, b, 0, n])
                assert np.array_equal(x["v_cache"][l, b, 0, L + j], x["v_tree"][l, b, 0, n])
            keep = [r for r in range(Lcap) if not (L <= r < L + a)]
            assert np.array_equal(x["k_cache"][l, b, 0, keep], kc0[l, b, 0, keep])
            assert np.array_equal(x["v_cache"][l, b, 0, keep], vc0[l, b, 0, keep])


def test_two_chained_steps_carry_the_accepted_prefix():
    """Fig. 1: what step 1 accepts is context in step 2.  After a planted 3-token accept, a second
    step (fresh tree rows) must place its tokens at the grown lengths and attend over the rows the
    first step committed: its root row equals plain decode attention over the old prefix, the
    accepted path's tree rows of step 1, and itself."""
    cfg = scaled_config("C2", B=2, d=64, Hq=2, Hkv=2, D=16, V=97, branching=(2, 2), L_min=5, L_max=9, Lcap=24, NL=2)
    tree = O.tree_cartesian(cfg.branching)
    x = make_step_inputs(cfg)
    kt1, vt1, kc0, vc0 = (x[n].copy() for n in ("k_tree", "v_tree", "k_cache", "v_cache"))
    pl0 = x["prefix_len"].copy()
    picks = [[0, 1, 3], [0, 2]]
    r1 = O.verification_step_ref(x, tree, cfg.dtype, 0.25, "greedy", 1.0, 0.0, 0.0, attn_layer=0, plant=planted(picks))
    assert r1.accept.accept_len.tolist() == [3, 2]
    for n in ("q", "k_tree", "v_tree", "hidden_tree"):                       # the next forward pass's rows
        x[n] = draw_normal(1234, {"q": 5, "k_tree": 6, "v_tree": 7, "hidden_tree": 1}[n], x[n].shape, 1.0, cfg.dtype)
    x["h_last"] = np.stack([x["hidden_tree"][b, r1.accept.best_node[b]] for b in range(cfg.B)])
    r2 = O.verification_step_ref(x, tree, cfg.dtype, 0.25, "greedy", 1.0, 0.0, 0.0, attn_layer=1)
    assert np.array_equal(r2.position_ids, (pl0 + np.array([3, 2]))[:, None] + tree.depth[None, :])
    w = O.widen
    for b in range(cfg.B):
        L, path = int(pl0[b]), picks[b]
        for g in range(cfg.Hq):
            ks = w(kc0[1, b, g, :L]).tolist() + [w(kt1[1, b, g, n]).tolist() for n in path] + [w(x["k_tree"][1, b, g, 0]).tolist()]
            vs = w(vc0[1, b, g, :L]).tolist() + [w(vt1[1, b, g, n]).tolist() for n in path] + [w(x["v_tree"][1, b, g, 0]).tolist()]
            want = causal_attention_scalar([w(x["q"][b, g, 0]).tolist()], ks, vs, L + len(path), 0.25)
            assert np.allclose(r2.attn_out[b, g, 0], want[0], rtol=1e-12, atol=1e-13)
