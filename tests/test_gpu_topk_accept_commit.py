"""GPU parity of the integer stages (top-k/tree assembly, acceptance, KV commit): bit-exact
against the CPU oracle on byte-identical inputs."""
import numpy as np
import pytest
import torch

import paper_2401_10774_amd as M
from oracle import medusa_oracle as O
from workloads import draw_normal
from _harness import bits, to_dev, to_host_bits

pytestmark = pytest.mark.gpu


def both_trees(branching=None, nodes=None):
    if branching is not None:
        return M.MedusaTree(branching=branching), O.tree_cartesian(branching)
    return M.MedusaTree(nodes=nodes), O.tree_from_nodes(nodes)


def check_topk(gt, ot, heads, lm, pl):
    topk, tokens, pos = M.medusa_topk_tree(to_dev(heads), to_dev(lm), gt, to_dev(pl))
    torch.cuda.synchronize()
    r_topk, r_tokens, r_pos = O.medusa_topk_tree_ref(heads, lm, ot, pl)
    assert np.array_equal(topk.cpu().numpy()[:, :, :r_topk.shape[2]], r_topk)
    assert np.array_equal(tokens.cpu().numpy(), r_tokens)
    assert np.array_equal(pos.cpu().numpy(), r_pos)


@pytest.mark.parametrize("branching,B,V", [((3, 2), 1, 1000), ((4, 3, 2, 1), 2, 32000), ((4, 3, 2, 1, 1), 4, 32000),
                                           ((2, 2), 3, 5), ((1,), 1, 1), ((16,), 2, 4097)])
def test_topk_random_logits(branching, B, V):
    gt, ot = both_trees(branching)
    heads = draw_normal(90, 1, (B, gt.K + 1, V), 1.3, "f32")         # one unused extra head
    lm = draw_normal(90, 2, (B, V), 1.3, "f32")
    pl = np.arange(B, dtype=np.int32) * 7 + 3
    check_topk(gt, ot, heads, lm, pl)


def test_topk_ties_take_the_lower_id():
    gt, ot = both_trees((4, 3, 2))
    rng = np.random.default_rng(91)
    for V in (9, 64, 1000, 8191):
        heads = rng.integers(-2, 3, (2, 3, V)).astype(np.float32)     # five distinct values: ties everywhere
        lm = rng.integers(-2, 3, (2, V)).astype(np.float32)
        heads[0, 0, :] = 0.0
        heads[0, 0, V // 2] = -0.0                                   # -0.0 must tie with +0.0
        check_topk(gt, ot, heads, lm, np.array([0, 5], np.int32))


def test_topk_sparse_tree_with_wide_ranks():
    nodes = [(0,), (1,), (2,), (9,), (15,), (0, 0), (0, 7), (1, 3), (0, 0, 0), (0, 7, 11)]
    gt, ot = both_trees(nodes=nodes)
    heads = draw_normal(92, 1, (3, 3, 32000), 1.0, "f32")
    lm = draw_normal(92, 2, (3, 32000), 1.0, "f32")
    check_topk(gt, ot, heads, lm, np.array([1, 2, 3], np.int32))


def planted_logits(rng, ot, B, V, scale=1.0):
    logits = (rng.standard_normal((B, ot.T, V)) * scale).astype(np.float32)
    tokens = np.empty((B, ot.T), np.int32)
    for b in range(B):
        tokens[b, 0] = rng.integers(V)
        for p in range(ot.T):
            kids = np.nonzero(ot.parent == p)[0]
            tokens[b, kids] = rng.choice(V, len(kids), replace=False)
        path = [int(n) for n in ot.paths[rng.integers(ot.n_leaves)] if n >= 0]
        for j in range(1, int(rng.integers(1, len(path) + 1))):
            logits[b, path[j - 1], tokens[b, path[j]]] += 20.0
    return logits, tokens


def check_accept(gt, ot, logits, tokens, mode, temperature=1.0, eps=0.0, delta=0.0, tol=1e-4):
    out = M.medusa_accept(to_dev(logits), to_dev(tokens), gt, mode, temperature, eps, delta)
    torch.cuda.synchronize()
    alen, best, path, toks, nxt = (t.cpu().numpy() for t in out)
    ref = O.medusa_accept_ref(logits, tokens, ot, mode, temperature, eps, delta)
    same = (np.array_equal(alen, ref.accept_len) and np.array_equal(best, ref.best_node) and
            np.array_equal(path, ref.path_nodes) and np.array_equal(toks, ref.accepted_tokens))
    if not same and mode == "typical":
        # a threshold decision closer than the fp32 evaluation error may fall either way; anything else is a bug
        assert ref.margin[:, 1:].min() < tol, "typical acceptance differs although no decision was near its threshold"
        pytest.fail(f"tie-ambiguous typical decision (margin {ref.margin[:, 1:].min():.2e}); pick another seed")
    assert same
    assert np.array_equal(nxt, ref.next_root)
    return ref


@pytest.mark.parametrize("branching,B,V", [((3, 2), 1, 1000), ((4, 3, 2, 1), 3, 32000), ((4, 3, 2, 1, 1), 2, 4099),
                                           ((2, 2, 2), 5, 11)])
def test_accept_greedy_planted_paths(branching, B, V):
    gt, ot = both_trees(branching)
    rng = np.random.default_rng(93)
    lens = set()
    for trial in range(3):
        logits, tokens = planted_logits(rng, ot, B, V)
        ref = check_accept(gt, ot, logits, tokens, "greedy")
        lens.update(int(a) for a in ref.accept_len)
    assert len(lens) >= 2


def test_accept_greedy_ties_and_constant_rows():
    gt, ot = both_trees((3, 2))
    V = 257
    logits = np.zeros((2, ot.T, V), np.float32)                     # every row constant: arg-max = token 0
    tokens = np.zeros((2, ot.T), np.int32)
    tokens[0] = np.arange(ot.T)                                      # node 1 holds token 1, ...
    tokens[1, 1] = 0                                                 # node 1 holds token 0 = the tie winner
    tokens[1, 2:] = np.arange(2, ot.T)
    tokens[1, 4] = 0                                                 # (0,0) under node 1 as well
    check_accept(gt, ot, logits, tokens, "greedy")


@pytest.mark.parametrize("branching,B,V,scale", [((3, 2), 2, 1000, 1.3), ((4, 3, 2, 1), 3, 32000, 1.3),
                                                 ((4, 3, 2, 1, 1), 2, 32000, 0.5), ((2, 2), 4, 17, 2.0)])
def test_accept_typical(branching, B, V, scale):
    gt, ot = both_trees(branching)
    rng = np.random.default_rng(94)
    lens = set()
    for trial in range(3):
        logits, tokens = planted_logits(rng, ot, B, V, scale)
        ref = check_accept(gt, ot, logits, tokens, "typical", 0.7, 0.09, 0.3)
        lens.update(int(a) for a in ref.accept_len)
    assert len(lens) >= 2


def test_accept_typical_uniform_rows_accept_everything():
    gt, ot = both_trees((3, 2, 2))
    V = 50
    logits = np.full((1, ot.T, V), 0.25, np.float32)
    tokens = ((np.arange(ot.T, dtype=np.int32)[None, :] * 7) % V).astype(np.int32)
    ref = check_accept(gt, ot, logits, tokens, "typical", 0.7, 0.09, 0.3)
    assert ref.accept_len[0] == ot.K + 1


def test_accept_exhaustive_pass_patterns():
    """All 2^9 pass patterns of the (3,2) tree, and a tree with leaves at unequal depths."""
    import itertools
    for nodes in (None, [(0,), (1,), (2,), (0, 0), (0, 0, 0), (1, 0), (1, 1), (2, 0), (0, 0, 0, 0)]):
        gt, ot = both_trees((3, 2)) if nodes is None else both_trees(nodes=nodes)
        V = 16
        pats = list(itertools.product([False, True], repeat=ot.T - 1))
        B = len(pats)
        tokens = np.tile(np.arange(ot.T, dtype=np.int32) % (V - 1), (B, 1))
        logits = np.full((B, ot.T, V), -30.0, np.float32)
        for b, bits in enumerate(pats):
            ok = (True,) + bits
            for p in range(ot.T):
                good = [tokens[b, c] for c in range(ot.T) if ot.parent[c] == p and ok[c]]
                logits[b, p, good if good else V - 1] = 0.0
        check_accept(gt, ot, logits, tokens, "typical", 1.0, 0.05, 1.0)


# The last two cases have the layer counts of the 13B- and 7B-shaped workloads (40 layers x 4 sequences,
# 32 x 16): the (layer * B + sequence) index of the cache reaches 160 and 512 there.
@pytest.mark.parametrize("dtype,NL,B,Hkv,T,D,Lcap", [("f32", 1, 1, 4, 10, 64, 160), ("bf16", 3, 4, 5, 65, 128, 300),
                                                      ("bf16", 2, 2, 8, 89, 128, 200), ("f32", 2, 3, 2, 7, 8, 40),
                                                      ("bf16", 40, 4, 40, 89, 128, 48), ("bf16", 32, 16, 8, 65, 128, 40)])
def test_kv_commit_bitwise(dtype, NL, B, Hkv, T, D, Lcap):
    rng = np.random.default_rng(95)
    kc = draw_normal(95, 8, (NL, B, Hkv, Lcap, D), 1.0, dtype)
    vc = draw_normal(95, 9, (NL, B, Hkv, Lcap, D), 1.0, dtype)
    kt = draw_normal(95, 6, (NL, B, Hkv, T, D), 1.0, dtype)
    vt = draw_normal(95, 7, (NL, B, Hkv, T, D), 1.0, dtype)
    Kp1 = 6
    alen = rng.integers(1, Kp1 + 1, B).astype(np.int32)
    path = np.full((B, Kp1), -1, np.int32)
    for b in range(B):
        path[b, :alen[b]] = np.sort(rng.choice(T, alen[b], replace=False))
    pl = rng.integers(0, Lcap - Kp1, B).astype(np.int32)
    pl[0] = 0
    d_kc, d_vc, d_pl = to_dev(kc), to_dev(vc), to_dev(pl)
    M.kv_commit(d_kc, d_vc, to_dev(kt), to_dev(vt), to_dev(path), to_dev(alen), d_pl)
    torch.cuda.synchronize()
    O.kv_commit_ref(kc, vc, kt, vt, path, alen, pl)
    assert np.array_equal(to_host_bits(d_kc), bits(kc)) and np.array_equal(to_host_bits(d_vc), bits(vc))
    assert np.array_equal(d_pl.cpu().numpy(), pl)


def test_kv_commit_lengths_to_a_second_array():
    """Out-of-place form: the cache rows are the same, prefix_len is left alone, the new lengths land
    in prefix_len_out; a second call on the same inputs writes the same rows again."""
    NL, B, Hkv, T, D, Lcap, Kp1 = 2, 3, 4, 20, 64, 90, 5
    rng = np.random.default_rng(96)
    kc = draw_normal(96, 8, (NL, B, Hkv, Lcap, D), 1.0, "bf16")
    vc = draw_normal(96, 9, (NL, B, Hkv, Lcap, D), 1.0, "bf16")
    kt = draw_normal(96, 6, (NL, B, Hkv, T, D), 1.0, "bf16")
    vt = draw_normal(96, 7, (NL, B, Hkv, T, D), 1.0, "bf16")
    alen = rng.integers(1, Kp1 + 1, B).astype(np.int32)
    path = np.full((B, Kp1), -1, np.int32)
    for b in range(B):
        path[b, :alen[b]] = np.sort(rng.choice(T, alen[b], replace=False))
    pl = rng.integers(0, Lcap - Kp1, B).astype(np.int32)
    d_kc, d_vc, d_pl = to_dev(kc), to_dev(vc), to_dev(pl)
    d_out = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    for _ in range(2):
        M.kv_commit(d_kc, d_vc, to_dev(kt), to_dev(vt), to_dev(path), to_dev(alen), d_pl, d_out)
    torch.cuda.synchronize()
    pl_ref = pl.copy()
    O.kv_commit_ref(kc, vc, kt, vt, path, alen, pl_ref)
    assert np.array_equal(to_host_bits(d_kc), bits(kc)) and np.array_equal(to_host_bits(d_vc), bits(vc))
    assert np.array_equal(d_pl.cpu().numpy(), pl) and np.array_equal(d_out.cpu().numpy(), pl_ref)


def test_kv_commit_never_writes_past_the_capacity():
    NL, B, Hkv, T, D, Lcap = 1, 2, 2, 5, 8, 6
    n = NL * B * Hkv * Lcap * D
    flat_k = torch.zeros(n + 4096, dtype=torch.float32, device="cuda")     # cache followed by guard words
    flat_v = torch.zeros(n + 4096, dtype=torch.float32, device="cuda")
    d_kc, d_vc = flat_k[:n].view(NL, B, Hkv, Lcap, D), flat_v[:n].view(NL, B, Hkv, Lcap, D)
    kt = to_dev(np.ones((NL, B, Hkv, T, D), np.float32))
    path = to_dev(np.array([[0, 1, 2], [0, 3, 4]], np.int32))
    alen = to_dev(np.array([3, 3], np.int32))
    pl = to_dev(np.array([5, 2], np.int32))                          # sequence 0 has room for one row only
    M.kv_commit(d_kc, d_vc, kt, kt, path, alen, pl)
    torch.cuda.synchronize()
    got = d_kc.cpu().numpy()
    assert got[0, 0, :, 5].min() == 1.0 and got[0, 0, :, :5].max() == 0.0
    assert got[0, 1, :, 2:5].min() == 1.0 and got[0, 1, :, 5].max() == 0.0 and got[0, 1, :, :2].max() == 0.0
    assert float(flat_k[n:].abs().max()) == 0.0 and float(flat_v[n:].abs().max()) == 0.0
    assert pl.cpu().numpy().tolist() == [6, 5]                        # saturates at Lcap


def _random_integer_stage_cases():
    """Seeded cases for the integer stages: random sparse trees of 2-127 nodes, batches of 1-40 sequences, vocabulary
    sizes from a few dozen to 32000, multiples of four or not (the scans read 16 bytes at a time only for the former)."""
    rng = np.random.default_rng(774011)
    cases = []
    while len(cases) < 14:
        nodes = {()}
        want = 2 + int(rng.integers(0, 126))
        while len(nodes) < want:
            p = list(nodes)[int(rng.integers(len(nodes)))]
            if len(p) < 5:
                nodes.add(p + (int(rng.integers(0, 10)),))
        B = int(rng.choice([1, 2, 5, 16, 40]))
        V = int(rng.choice([37, 1000, 4099, 32000, int(rng.integers(16, 33000))]))
        if B * len(nodes) * V > 3e7:
            continue
        cases.append((sorted(n for n in nodes if n), B, V, 500 + len(cases)))
    return cases


@pytest.mark.parametrize("nodes,B,V,seed", _random_integer_stage_cases(), ids=lambda v: None if isinstance(v, list) else str(v))
def test_random_trees_topk_and_greedy_acceptance(nodes, B, V, seed):
    gt, ot = both_trees(nodes=nodes)
    heads = draw_normal(seed, 1, (B, ot.K, V), 1.0, "f32")
    lm = draw_normal(seed, 2, (B, V), 1.0, "f32")
    check_topk(gt, ot, heads, lm, np.arange(B, dtype=np.int32) * 3)
    logits, tokens = planted_logits(np.random.default_rng(seed), ot, B, V)
    check_accept(gt, ot, logits, tokens, "greedy")
