"""Pins for the oracle's rejection-sampling acceptance (Sec. 2 opening paragraph and Sec. 2.3.1 name
the speculative-decoding scheme; the rule itself is this build's reading, stated in the oracle).

The paper prints no formula for it, so the pin is the property the scheme exists for: whatever the
candidates are, the tokens a step emits are distributed exactly as the original model would emit
them one by one.  On a tiny case whose probabilities are multiples of 1/8 every decision boundary
of the walk is a multiple of 1/8, so the unit cube of the uniforms splits into 8^5 equal cells
inside each of which the outcome is constant; enumerating all cells gives the exact distribution.
"""
import itertools
import math
from collections import defaultdict
from fractions import Fraction

import numpy as np

from oracle import medusa_oracle as O


def logits_of(p):
    return np.log(np.asarray(p, np.float64))


def test_emitted_tokens_follow_the_original_model_exactly():
    tree = O.tree_cartesian((2, 1))                  # root; children 1, 2; grandchild 3 under 1, 4 under 2
    assert tree.parent.tolist() == [-1, 0, 0, 1, 2]
    V = 4
    rows = {0: [1 / 2, 1 / 4, 1 / 8, 1 / 8], 1: [1 / 4, 1 / 2, 1 / 8, 1 / 8], 2: [1 / 8, 1 / 8, 1 / 4, 1 / 2],
            3: [1 / 4, 1 / 4, 1 / 4, 1 / 4], 4: [1 / 2, 1 / 8, 1 / 8, 1 / 4]}
    logits = np.stack([logits_of(rows[t]) for t in range(5)])[None]              # [1, T, V]
    tokens = np.array([[9, 0, 1, 1, 3]], np.int32)   # root token is irrelevant; children of the root hold 0 and 1
    G = 8
    mids = [(g + 0.5) / G for g in range(G)]
    first = defaultdict(Fraction)                    # P(first emitted token)
    second = defaultdict(Fraction)                   # P(first, second) for steps that emit two or more
    third = defaultdict(Fraction)
    cell = Fraction(1, G ** 5)
    for u in itertools.product(mids, repeat=5):      # u[0] is the sampling uniform, u[t] the test of node t
        r = O.medusa_accept_sampled_ref(logits, tokens, tree, np.array([u]), 1.0)
        assert r.margin[0] >= 1 / (2 * G) - 1e-12    # no cell touches a decision boundary
        emitted = [int(t) for t in r.accepted_tokens[0, 1:r.accept_len[0]]] + [int(r.next_token[0])]
        assert r.path_nodes[0, 0] == 0 and r.accept_len[0] == len(emitted)
        first[emitted[0]] += cell
        if len(emitted) >= 2:
            second[(emitted[0], emitted[1])] += cell
        if len(emitted) >= 3:
            third[tuple(emitted[:3])] += cell
    F = lambda x: Fraction(x).limit_denominator(64)
    # the first token after the root is a draw from the root's row, accepted candidate or not
    for y in range(V):
        assert first[y] == F(rows[0][y]), (y, first[y])
    # after an accepted candidate (token 0 -> node 1, token 1 -> node 2) the second token is a draw from that node's row
    for y, node in ((0, 1), (1, 2)):
        for z in range(V):
            assert second[(y, z)] == F(rows[0][y]) * F(rows[node][z]), (y, z)
    # a first token outside the candidates ends the step
    assert all(k[0] in (0, 1) for k in second)
    # and after two accepted candidates the third token is a draw from the grandchild's row
    for (y, z, node) in ((0, 1, 3), (1, 3, 4)):
        for w in range(V):
            assert third[(y, z, w)] == F(rows[0][y]) * F(rows[{0: 1, 1: 2}[y]][z]) * F(rows[node][w])
    assert sum(first.values()) == 1


def test_hand_worked_walk():
    """Root row p = (0.5, 0.3, 0.2) with candidates 1 then 0: the first is accepted iff u < 0.3; else the second iff
    u' < 0.5 / 0.7; else token 2 for certain.  Temperature 2 flattens the row first."""
    tree = O.tree_cartesian((2,))
    logits = np.stack([logits_of([0.5, 0.3, 0.2])] * 3)[None]
    tokens = np.array([[7, 1, 0]], np.int32)
    run = lambda u0, u1, u2, temp=1.0: O.medusa_accept_sampled_ref(logits, tokens, tree, np.array([[u0, u1, u2]]), temp)
    r = run(0.9, 0.29, 0.0)
    assert r.accept_len[0] == 2 and r.best_node[0] == 1 and r.accepted_tokens[0].tolist() == [7, 1]
    assert r.next_token[0] == 2                      # leaf: inversion on p itself, 0.9 lies in token 2's interval (0.8, 1)
    r = run(0.55, 0.31, 0.71)                        # 0.31 >= 0.3 rejected; 0.71 < 0.5 / 0.7 = 0.714 accepted
    assert r.path_nodes[0].tolist() == [0, 2] and r.next_token[0] == 1     # leaf again: 0.55 in (0.5, 0.8)
    r = run(0.0, 0.31, 0.72)                         # both rejected: the residual is token 2 alone
    assert r.accept_len[0] == 1 and r.best_node[0] == 0 and r.next_token[0] == 2
    assert abs(r.margin[0] - min(0.01, 0.72 - 0.5 / 0.7)) < 1e-12
    q = np.array([0.5, 0.3, 0.2]) ** 0.5
    q /= q.sum()                                     # softmax(logits / 2)
    r = run(0.0, float(q[1]) - 1e-9, 0.0, temp=2.0)
    assert r.accept_len[0] == 2
    r = run(0.0, float(q[1]) + 1e-9, 0.999, temp=2.0)
    assert r.accept_len[0] == 1


def test_extremes_and_invariants():
    rng = np.random.default_rng(5)
    tree = O.tree_cartesian((3, 2, 1))
    B, V = 4, 17
    logits = rng.standard_normal((B, tree.T, V))
    tokens = np.empty((B, tree.T), np.int32)
    for b in range(B):
        for pnode in range(tree.T):
            kids = [c for c in range(tree.T) if tree.parent[c] == pnode]
            tokens[b, kids] = rng.choice(V, len(kids), replace=False)
        tokens[b, 0] = 0
    zero = O.medusa_accept_sampled_ref(logits, tokens, tree, np.zeros((B, tree.T)), 0.7)
    assert (zero.accept_len == tree.K + 1).all()                     # u = 0 accepts every first child
    assert (zero.path_nodes == tree.paths[0]).all()
    one = O.medusa_accept_sampled_ref(logits, tokens, tree, np.full((B, tree.T), 1.0 - 1e-12), 0.7)
    assert (one.accept_len == 1).all()                               # u -> 1 rejects everything (no ratio reaches 1 here)
    for b in range(B):                                               # ... and never draws a rejected candidate
        assert one.next_token[b] not in tokens[b, 1:4]
    u = rng.random((B, tree.T))
    r = O.medusa_accept_sampled_ref(logits, tokens, tree, u, 0.7)
    for b in range(B):
        n = int(r.accept_len[b])
        path = r.path_nodes[b, :n]
        assert path[0] == 0 and all(tree.parent[path[j]] == path[j - 1] for j in range(1, n))
        assert (r.path_nodes[b, n:] == -1).all() and r.best_node[b] == path[-1]
        assert r.accepted_tokens[b, :n].tolist() == tokens[b, path].tolist()
        kids = [c for c in range(tree.T) if tree.parent[c] == path[-1]]
        assert r.next_token[b] not in tokens[b, kids]
    # a one-hot row accepts its candidate whatever the uniform, and samples the hot token at a leaf
    hot = np.full((1, 3, 5), -1e4)
    hot[0, :, 2] = 0.0
    r = O.medusa_accept_sampled_ref(hot, np.array([[0, 2, 4]], np.int32), O.tree_cartesian((2,)), np.array([[0.99, 0.999, 0.5]]))
    assert r.accept_len[0] == 2 and r.best_node[0] == 1 and r.next_token[0] == 2
