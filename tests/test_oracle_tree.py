"""Pins for the oracle's candidate-tree tables (Sec. 2.1.2, Fig. 2)."""
import itertools
import os

import numpy as np
import pytest

from oracle import medusa_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tree_counts.txt")


def golden_rows():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        br, n, leaves = [f.strip() for f in line.split("|")]
        rows.append((tuple(int(x) for x in br.split(",")), int(n), int(leaves)))
    return rows


@pytest.mark.parametrize("branching,n_nodes,n_leaves", golden_rows())
def test_counts_from_the_paper(branching, n_nodes, n_leaves):
    t = O.tree_cartesian(branching)
    assert t.T == n_nodes + 1 and t.n_leaves == n_leaves and t.K == len(branching)
    # the formula itself, evaluated independently
    assert n_nodes == sum(int(np.prod(branching[:k])) for k in range(1, len(branching) + 1))
    assert list(t.topk_per_head) == list(branching)


def second_construction(branching):
    """Independent build: breadth-first queue of (rank tuple, parent index)."""
    nodes, parent = [()], [-1]
    frontier = [0]
    for s in branching:
        nxt = []
        for p in frontier:                       # frontier is already in lexicographic order
            for r in range(s):
                nodes.append(nodes[p] + (r,))
                parent.append(p)
                nxt.append(len(nodes) - 1)
        frontier = nxt
    return nodes, parent


@pytest.mark.parametrize("branching", [(2, 3), (3, 2), (4, 3, 2, 1), (4, 3, 2, 1, 1), (1,), (2, 2, 2, 2, 2)])
def test_tables_against_second_construction_and_invariants(branching):
    t = O.tree_cartesian(branching)
    nodes, parent = second_construction(branching)
    assert t.nodes == nodes
    assert list(t.parent) == parent
    base = [1] + list(1 + np.cumsum(branching)[:-1])
    for i in range(1, t.T):
        p = t.parent[i]
        assert t.depth[p] == t.depth[i] - 1
        assert t.rank[i] == nodes[i][-1]
        assert t.token_src[i] == base[len(nodes[i]) - 1] + nodes[i][-1]
        m = int(t.anc_mask[i, 0]) | (int(t.anc_mask[i, 1]) << 64)
        mp = int(t.anc_mask[p, 0]) | (int(t.anc_mask[p, 1]) << 64)
        assert m == mp | (1 << i)
        assert bin(m).count("1") == t.depth[i] + 1
    assert int(t.anc_mask[0, 0]) == 1 and t.token_src[0] == 0 and t.depth[0] == 0
    # children of one parent are consecutive and rank-ordered
    for p in range(t.T):
        kids = [i for i in range(t.T) if t.parent[i] == p]
        assert kids == list(range(kids[0], kids[0] + len(kids))) if kids else True
        assert [t.rank[i] for i in kids] == sorted(t.rank[i] for i in kids)
    # candidates = Cartesian product of the per-head ranks, in lexicographic order
    want = list(itertools.product(*[range(s) for s in branching]))
    got = [tuple(t.rank[n] for n in path[1:]) for path in t.paths]
    assert got == want
    for path in t.paths:
        assert path[0] == 0 and all(t.parent[path[j]] == path[j - 1] for j in range(1, len(path)))


def test_sparse_tree_from_nodes():
    cand = [(0,), (1,), (3,), (0, 0), (0, 2), (1, 0), (0, 0, 0)]
    t = O.tree_from_nodes(cand)
    assert t.T == 8 and t.K == 3
    assert t.nodes == [(), (0,), (1,), (3,), (0, 0), (0, 2), (1, 0), (0, 0, 0)]
    assert list(t.topk_per_head) == [4, 3, 1]
    assert list(t.token_src) == [0, 1, 2, 4, 5, 7, 5, 8]
    # leaves in lexicographic order of their rank tuples: (0,0,0) (0,2) (1,0) (3,)
    assert t.paths.tolist() == [[0, 1, 4, 7], [0, 1, 5, -1], [0, 2, 6, -1], [0, 3, -1, -1]]
    with pytest.raises(ValueError):
        O.tree_from_nodes([(0,), (1, 0)])         # (1,) missing: not prefix closed
    # a Cartesian tree given as an explicit node list is the same tree
    a, b = O.tree_cartesian((3, 2)), O.tree_from_nodes(O.tree_cartesian((3, 2)).nodes[1:])
    assert a.nodes == b.nodes and np.array_equal(a.paths, b.paths) and np.array_equal(a.anc_mask, b.anc_mask)


def test_mask_crosses_64_bit_boundary():
    t = O.tree_cartesian((4, 3, 2, 1, 1))
    assert t.T == 89
    for i in (64, 70, 88):
        m = int(t.anc_mask[i, 0]) | (int(t.anc_mask[i, 1]) << 64)
        u, want = i, 0
        while u >= 0:
            want |= 1 << u
            u = int(t.parent[u])
        assert m == want and (m >> 64) != 0
