"""Pins for the oracle's acceptance step (Sec. 2.3.1) and the carry-over (Fig. 1)."""
import itertools
import math

import numpy as np
import pytest

from oracle import medusa_oracle as O


def py_argmax(row):
    best = 0
    for i, v in enumerate(row):
        if v > row[best]:
            best = i
    return best


def sequential_greedy_walk(logits_b, tokens_b, tree):
    """What plain greedy decoding would do with the tree as a lookup: start at the root, take the
    original model's arg-max at the current node, move to the child holding that token, else stop."""
    cur, visited = 0, [0]
    while True:
        nxt = py_argmax(logits_b[cur].tolist())
        kids = [c for c in range(tree.T) if tree.parent[c] == cur and tokens_b[c] == nxt]
        if not kids:
            return visited, nxt
        cur = kids[0]
        visited.append(cur)


def random_case(rng, tree, B, V, plant):
    logits = rng.standard_normal((B, tree.T, V)).astype(np.float32)
    tokens = np.empty((B, tree.T), np.int32)
    for b in range(B):
        for p in range(tree.T):                                  # siblings hold distinct tokens
            kids = [c for c in range(tree.T) if tree.parent[c] == p]
            tokens[b, kids] = rng.choice(V, len(kids), replace=False)
        tokens[b, 0] = rng.integers(V)
        if plant:
            path = tree.paths[rng.integers(tree.n_leaves)]
            path = [int(n) for n in path if n >= 0]
            for j in range(1, int(rng.integers(1, len(path) + 1))):
                logits[b, path[j - 1], tokens[b, path[j]]] += 20.0
    return logits, tokens


@pytest.mark.parametrize("branching", [(3, 2), (4, 3, 2, 1), (2, 2, 2)])
def test_greedy_equals_sequential_walk(branching):
    tree = O.tree_cartesian(branching)
    rng = np.random.default_rng(31)
    lens = set()
    for trial in range(30):
        logits, tokens = random_case(rng, tree, 2, 37, plant=True)
        res = O.medusa_accept_ref(logits, tokens, tree, "greedy")
        for b in range(2):
            visited, nxt = sequential_greedy_walk(logits[b], tokens[b], tree)
            a = int(res.accept_len[b])
            assert a == len(visited)
            assert res.path_nodes[b, :a].tolist() == visited and (res.path_nodes[b, a:] == -1).all()
            assert res.best_node[b] == visited[-1]
            assert res.accepted_tokens[b, :a].tolist() == [int(tokens[b, n]) for n in visited]
            assert (res.accepted_tokens[b, a:] == -1).all()
            assert res.next_root[b] == nxt
            lens.add(a)
    assert len(lens) >= 3 and min(lens) >= 1 and max(lens) <= tree.K + 1


def test_greedy_ties_take_the_lower_token_id():
    tree = O.tree_cartesian((2,))
    logits = np.zeros((1, 3, 5), np.float32)
    logits[0, 0, [1, 3]] = 2.0                                    # tie: arg-max is token 1
    tokens = np.array([[0, 3, 1]], np.int32)                      # node 1 holds 3, node 2 holds 1
    res = O.medusa_accept_ref(logits, tokens, tree, "greedy")
    assert res.accept_len[0] == 2 and res.best_node[0] == 2 and res.next_root[0] == 0


def node_definition(ok, tree):
    """acc[t] = ok[t] and acc[parent]; winner = accepted node of greatest depth, lowest index."""
    acc = np.zeros(tree.T, bool)
    acc[0] = True
    for t in range(1, tree.T):
        acc[t] = ok[t] and acc[tree.parent[t]]
    best = max(range(tree.T), key=lambda t: (acc[t] * (tree.depth[t] + 1), -t))
    path = []
    u = best
    while u >= 0:
        path.append(u)
        u = int(tree.parent[u])
    return int(tree.depth[best]) + 1, best, path[::-1]


def logits_for_ok_pattern(ok, tokens, tree, V):
    """Rows on which typical acceptance (eps = 0.05, delta = 1) yields exactly the pattern `ok`."""
    logits = np.full((1, tree.T, V), -30.0, np.float32)
    for p in range(tree.T):
        good = [tokens[0, c] for c in range(tree.T) if tree.parent[c] == p and ok[c]]
        if good:
            logits[0, p, good] = 0.0
        else:
            logits[0, p, V - 1] = 0.0                              # a token no node holds
    return logits


@pytest.mark.parametrize("nodes", [
    None,                                                          # the (3,2) Cartesian tree: 2^9 patterns
    [(0,), (1,), (2,), (0, 0), (0, 0, 0), (1, 0), (1, 1), (2, 0), (0, 0, 0, 0)],   # leaves at unequal depths
])
def test_exhaustive_ok_patterns_candidate_list_equals_node_definition(nodes):
    tree = O.tree_cartesian((3, 2)) if nodes is None else O.tree_from_nodes(nodes)
    V = 16
    tokens = np.arange(tree.T, dtype=np.int32)[None, :] % (V - 1)
    for bits in itertools.product([False, True], repeat=tree.T - 1):
        ok = np.array((True,) + bits)
        logits = logits_for_ok_pattern(ok, tokens, tree, V)
        res = O.medusa_accept_ref(logits, tokens, tree, "typical", 1.0, 0.05, 1.0)
        assert np.array_equal(res.ok[0], ok)
        a, best, path = node_definition(ok, tree)
        assert res.accept_len[0] == a and res.best_node[0] == best
        assert res.path_nodes[0, :a].tolist() == path and (res.path_nodes[0, a:] == -1).all()


def test_typical_threshold_hand_worked_row():
    # p = (1/2, 1/4, 1/8, 1/8): H = 1.75 bits = 1.75 ln 2 nats, exp(-H) = 2^-1.75
    z = np.log(np.array([0.5, 0.25, 0.125, 0.125]))
    p, H, thr = O.typical_threshold_ref(z, 1.0, 0.2, 0.5)
    assert np.allclose(p, [0.5, 0.25, 0.125, 0.125], rtol=1e-15)
    assert abs(H - 1.2130075659799042) < 1e-14
    assert abs(thr - 0.5 * 0.2973017787506803) < 1e-15          # delta * exp(-H) = 0.14865 < eps
    _, _, thr2 = O.typical_threshold_ref(z, 1.0, 0.1, 0.5)
    assert thr2 == 0.1                                            # eps is the smaller one now
    # temperature 1/2 squares the probabilities: (8, 2, 1/2, 1/2) / 11
    p2, H2, _ = O.typical_threshold_ref(z, 0.5, 0.2, 0.5)
    assert np.allclose(p2, np.array([8, 2, 0.5, 0.5]) / 11, rtol=1e-14)
    assert abs(H2 - (math.log(11) - 25 * math.log(2) / 11)) < 1e-14   # closed form of -sum p ln p for (8,2,.5,.5)/11
    # acceptance decisions on that row: tree with three children of the root holding tokens 0, 1, 2
    tree = O.tree_cartesian((3,))
    logits = np.tile(z.astype(np.float32), (1, 4, 1))
    tokens = np.array([[0, 0, 1, 2]], np.int32)
    r = O.medusa_accept_ref(logits, tokens, tree, "typical", 1.0, 0.2, 0.5)
    assert r.ok[0].tolist() == [True, True, True, False]          # 0.125 < 0.14865
    r = O.medusa_accept_ref(logits, tokens, tree, "typical", 1.0, 0.1, 0.5)
    assert r.ok[0].tolist() == [True, True, True, True]           # 0.125 > 0.1
    assert r.accept_len[0] == 2 and r.best_node[0] == 1           # first candidate wins the tie


def test_typical_uniform_rows_accept_everything():
    tree = O.tree_cartesian((3, 2, 2))
    V = 50
    logits = np.full((1, tree.T, V), 0.25, np.float32)
    tokens = (np.arange(tree.T, dtype=np.int32)[None, :] * 7) % V
    p, H, thr = O.typical_threshold_ref(logits[0, 0], 0.7, 0.09, 0.3)
    assert abs(H - math.log(V)) < 1e-13 and abs(thr - 0.3 / V) < 1e-16 and np.allclose(p, 1 / V)
    r = O.medusa_accept_ref(logits, tokens, tree, "typical", 0.7, 0.09, 0.3)
    assert r.ok.all() and r.accept_len[0] == tree.K + 1
    assert r.best_node[0] == int(tree.paths[0, -1]) and r.path_nodes[0].tolist() == tree.paths[0].tolist()
    assert r.next_root[0] == 0                                     # arg-max of a constant row: lowest id


def test_typical_one_hot_rows():
    # a dominant token drives H to 0, so the threshold tends to min(eps, delta)
    z = np.array([40.0, 0.0, 0.0, 0.0])
    p, H, thr = O.typical_threshold_ref(z, 1.0, 0.09, 0.3)
    assert H < 1e-15 and abs(thr - 0.09) < 1e-15 and p[0] > 0.999
    _, _, thr = O.typical_threshold_ref(z, 1.0, 0.5, 0.3)
    assert abs(thr - 0.3) < 1e-12


def test_small_temperature_reverts_to_greedy_and_typical_never_shorter():
    tree = O.tree_cartesian((3, 2, 1))
    rng = np.random.default_rng(33)
    longer = 0
    for trial in range(40):
        logits, tokens = random_case(rng, tree, 2, 29, plant=True)
        g = O.medusa_accept_ref(logits, tokens, tree, "greedy")
        cold = O.medusa_accept_ref(logits, tokens, tree, "typical", 1e-3, 0.09, 0.3)
        assert np.array_equal(cold.accept_len, g.accept_len) and np.array_equal(cold.path_nodes, g.path_nodes)
        assert np.array_equal(cold.next_root, g.next_root)
        warm = O.medusa_accept_ref(logits / 8, tokens, tree, "typical", 0.7, 0.09, 0.3)
        g8 = O.medusa_accept_ref(logits / 8, tokens, tree, "greedy")
        assert (warm.accept_len >= g8.accept_len).all()          # delta < 1: the greedy token always passes
        assert (warm.accept_len >= 1).all()
        longer += int((warm.accept_len > g8.accept_len).sum())
    assert longer > 0


def test_accept_uses_the_parents_row_not_the_nodes_own():
    tree = O.tree_cartesian((1, 1))
    V = 6
    logits = np.zeros((1, 3, V), np.float32)
    logits[0, 0, 4] = 5.0       # root row predicts 4
    logits[0, 1, 2] = 5.0       # node 1 row predicts 2
    logits[0, 2, 3] = 5.0       # node 2 row predicts 3 (only used for next_root)
    tokens = np.array([[9 % V, 4, 2]], np.int32)
    r = O.medusa_accept_ref(logits, tokens, tree, "greedy")
    assert r.accept_len[0] == 3 and r.next_root[0] == 3
    tokens = np.array([[0, 2, 4]], np.int32)                      # rows swapped relative to the tokens
    r = O.medusa_accept_ref(logits, tokens, tree, "greedy")
    assert r.accept_len[0] == 1 and r.next_root[0] == 4


def test_kv_commit_hand_case_and_untouched_rows():
    NL, B, H, T, D, Lcap = 2, 2, 2, 5, 3, 9
    rng = np.random.default_rng(34)
    kc = rng.standard_normal((NL, B, H, Lcap, D)).astype(np.float32)
    vc = rng.standard_normal((NL, B, H, Lcap, D)).astype(np.float32)
    kt = rng.standard_normal((NL, B, H, T, D)).astype(np.float32)
    vt = rng.standard_normal((NL, B, H, T, D)).astype(np.float32)
    kc0, vc0 = kc.copy(), vc.copy()
    pl = np.array([4, 2], np.int32)
    path = np.array([[0, 2, 4], [0, -1, -1]], np.int32)
    alen = np.array([3, 1], np.int32)
    O.kv_commit_ref(kc, vc, kt, vt, path, alen, pl)
    assert pl.tolist() == [7, 3]
    for l in range(NL):
        for h in range(H):
            assert np.array_equal(kc[l, 0, h, 4], kt[l, 0, h, 0])
            assert np.array_equal(kc[l, 0, h, 5], kt[l, 0, h, 2])
            assert np.array_equal(vc[l, 0, h, 6], vt[l, 0, h, 4])
            assert np.array_equal(kc[l, 1, h, 2], kt[l, 1, h, 0])
    mask = np.ones((B, Lcap), bool)
    mask[0, 4:7] = False
    mask[1, 2:3] = False
    for b in range(B):
        assert np.array_equal(kc[:, b][:, :, mask[b]], kc0[:, b][:, :, mask[b]])
        assert np.array_equal(vc[:, b][:, :, mask[b]], vc0[:, b][:, :, mask[b]])


def test_commit_then_attend_equals_attending_the_path_in_the_tree():
    """Carry-over consistency: after the accepted path is appended to the cache, a next-step root
    attending over the grown prefix sees exactly the keys the last accepted node saw in the tree."""
    tree = O.tree_cartesian((2, 2))
    B, H, D, Lcap, L = 1, 2, 4, 12, 5
    rng = np.random.default_rng(35)
    kc = rng.standard_normal((1, B, H, Lcap, D)).astype(np.float32)
    vc = rng.standard_normal((1, B, H, Lcap, D)).astype(np.float32)
    kt = rng.standard_normal((1, B, H, tree.T, D)).astype(np.float32)
    vt = rng.standard_normal((1, B, H, tree.T, D)).astype(np.float32)
    q = rng.standard_normal((B, H, tree.T, D)).astype(np.float32)
    pl = np.array([L], np.int32)
    before = O.tree_attention_ref(q, kt[0], vt[0], kc[0], vc[0], pl, tree, 0.5)
    path = tree.paths[2:3].copy()                                  # root -> (1,) -> (1,0)
    best = int(path[0, 2])
    O.kv_commit_ref(kc, vc, kt, vt, path, np.array([3], np.int32), pl)
    assert pl[0] == L + 3
    # a single query equal to q[best], whose own key/value row is already the last cache row
    one = O.tree_from_nodes([])
    pl2 = np.array([L + 2], np.int32)
    after = O.tree_attention_ref(q[:, :, best:best + 1], kt[0][:, :, best:best + 1], vt[0][:, :, best:best + 1],
                                 kc[0], vc[0], pl2, one, 0.5)
    assert np.allclose(after[:, :, 0], before[:, :, best], rtol=1e-13)
