"""Pins for the oracle's tree attention (Sec. 2.1.2).

The central pin is the paper's own statement of what the mask is for: a tree
token only sees its predecessors on its own continuation, so processing the
tree at once must give, at every node, what ordinary causal attention gives
when that node's root-to-leaf path is appended to the prefix as a plain
sequence.  The causal reference below is written with scalar loops and
math.exp and shares nothing with the oracle.
"""
import math

import numpy as np
import pytest

from oracle import medusa_oracle as O
from workloads import draw_normal


def causal_attention_scalar(q_rows, k_rows, v_rows, n_ctx, scale):
    """q_rows [n, D] are the last n tokens of a sequence whose keys/values are
    k_rows, v_rows [n_ctx + n, D]; token i sees keys 0 .. n_ctx + i."""
    n, D = len(q_rows), len(q_rows[0])
    out = []
    for i in range(n):
        visible = n_ctx + i + 1
        s = [scale * math.fsum(q_rows[i][c] * k_rows[j][c] for c in range(D)) for j in range(visible)]
        m = max(s)
        e = [math.exp(x - m) for x in s]
        z = math.fsum(e)
        out.append([math.fsum(e[j] * v_rows[j][c] for j in range(visible)) / z for c in range(D)])
    return out


def make_inputs(dtype, B, Hq, Hkv, T, D, Lcap, seed):
    q = draw_normal(seed, 5, (B, Hq, T, D), 1.0, dtype)
    kt = draw_normal(seed, 6, (B, Hkv, T, D), 1.0, dtype)
    vt = draw_normal(seed, 7, (B, Hkv, T, D), 1.0, dtype)
    kc = draw_normal(seed, 8, (B, Hkv, Lcap, D), 1.0, dtype)
    vc = draw_normal(seed, 9, (B, Hkv, Lcap, D), 1.0, dtype)
    return q, kt, vt, kc, vc


@pytest.mark.parametrize("dtype,branching,Hq,Hkv,prefix", [
    ("f32", (3, 2), 2, 2, [5]),
    ("bf16", (2, 2, 1), 4, 2, [7, 0]),          # GQA, one sequence with an empty prefix
    ("f32", (2, 3), 2, 1, [3, 9]),              # MQA, ragged prefixes
])
def test_path_equivalence(dtype, branching, Hq, Hkv, prefix):
    tree = O.tree_cartesian(branching)
    B, D, Lcap = len(prefix), 8, 12
    q, kt, vt, kc, vc = make_inputs(dtype, B, Hq, Hkv, tree.T, D, Lcap, 21)
    pl = np.array(prefix, np.int32)
    scale = 1.0 / math.sqrt(D)
    out = O.tree_attention_ref(q, kt, vt, kc, vc, pl, tree, scale)
    qf, ktf, vtf, kcf, vcf = (O.widen(x) for x in (q, kt, vt, kc, vc))
    seen = set()
    for b in range(B):
        L = int(pl[b])
        for g in range(Hq):
            h = g // (Hq // Hkv)
            for path in tree.paths:
                nodes = [int(n) for n in path if n >= 0]
                ks = kcf[b, h, :L].tolist() + [ktf[b, h, n].tolist() for n in nodes]
                vs = vcf[b, h, :L].tolist() + [vtf[b, h, n].tolist() for n in nodes]
                qs = [qf[b, g, n].tolist() for n in nodes]
                want = causal_attention_scalar(qs, ks, vs, L, scale)
                for i, n in enumerate(nodes):
                    assert np.allclose(out[b, g, n], want[i], rtol=1e-12, atol=1e-13)
                    seen.add(n)
    assert seen == set(range(tree.T))


def test_chain_tree_is_plain_causal_attention():
    tree = O.tree_cartesian((1, 1, 1))
    D, L = 4, 6
    q, kt, vt, kc, vc = make_inputs("f32", 1, 1, 1, tree.T, D, L, 22)
    out = O.tree_attention_ref(q, kt, vt, kc, vc, np.array([L], np.int32), tree, 0.5)
    ks = np.concatenate([kc[0, 0], kt[0, 0]]).astype(np.float64)
    vs = np.concatenate([vc[0, 0], vt[0, 0]]).astype(np.float64)
    want = causal_attention_scalar(q[0, 0].astype(np.float64).tolist(), ks.tolist(), vs.tolist(), L, 0.5)
    assert np.allclose(out[0, 0], want, rtol=1e-12, atol=1e-13)


def test_single_token_is_decode_attention_and_empty_prefix_is_identity():
    tree = O.tree_from_nodes([])
    assert tree.T == 1 and tree.K == 0
    D, L = 4, 5
    q, kt, vt, kc, vc = make_inputs("f32", 1, 1, 1, 1, D, L, 23)
    out = O.tree_attention_ref(q, kt, vt, kc, vc, np.array([L], np.int32), tree, 1.0)
    keys = np.concatenate([kc[0, 0], kt[0, 0]]).astype(np.float64)
    vals = np.concatenate([vc[0, 0], vt[0, 0]]).astype(np.float64)
    s = keys @ q[0, 0, 0].astype(np.float64)
    p = np.exp(s - s.max())
    p /= p.sum()
    assert np.allclose(out[0, 0, 0], p @ vals, rtol=1e-13)
    # L = 0: the root sees only itself, so its output is its own value row
    out0 = O.tree_attention_ref(q, kt, vt, kc, vc, np.array([0], np.int32), tree, 1.0)
    assert np.allclose(out0[0, 0, 0], vt[0, 0, 0].astype(np.float64), rtol=1e-15)


def test_constant_values_and_scale_sensitivity():
    tree = O.tree_cartesian((2, 2))
    D, L = 4, 6
    q, kt, vt, kc, vc = make_inputs("f32", 1, 2, 2, tree.T, D, L, 24)
    vt[:] = 3.0
    vc[:] = 3.0
    out = O.tree_attention_ref(q, kt, vt, kc, vc, np.array([L], np.int32), tree, 0.5)
    assert np.allclose(out, 3.0, rtol=1e-14)
    # scale 0 makes every visible key equally weighted: output = mean over the visible set
    q2, kt2, vt2, kc2, vc2 = make_inputs("f32", 1, 1, 1, tree.T, D, L, 25)
    out = O.tree_attention_ref(q2, kt2, vt2, kc2, vc2, np.array([L], np.int32), tree, 0.0)
    for t in range(tree.T):
        anc = [u for u in range(tree.T) if (int(tree.anc_mask[t, 0]) >> u) & 1]
        rows = np.concatenate([vc2[0, 0, :L], vt2[0, 0, anc]]).astype(np.float64)
        assert len(anc) == tree.depth[t] + 1
        assert np.allclose(out[0, 0, t], rows.mean(axis=0), rtol=1e-13)


def test_rows_beyond_prefix_and_sibling_rows_are_ignored():
    tree = O.tree_cartesian((2, 2))
    D, Lcap, L = 4, 10, 6
    q, kt, vt, kc, vc = make_inputs("f32", 1, 2, 2, tree.T, D, Lcap, 26)
    pl = np.array([L], np.int32)
    a = O.tree_attention_ref(q, kt, vt, kc, vc, pl, tree, 0.5)
    kc2, vc2 = kc.copy(), vc.copy()
    kc2[:, :, L:] = 1e6
    vc2[:, :, L:] = -1e6
    assert np.array_equal(a, O.tree_attention_ref(q, kt, vt, kc2, vc2, pl, tree, 0.5))
    # node 1 = (0,) must not depend on its sibling node 2 = (1,) nor on any descendant
    kt2, vt2 = kt.copy(), vt.copy()
    kt2[:, :, 2:] += 5.0
    vt2[:, :, 2:] -= 5.0
    b = O.tree_attention_ref(q, kt2, vt2, kc, vc, pl, tree, 0.5)
    assert np.array_equal(a[:, :, :2], b[:, :, :2]) and not np.allclose(a[:, :, 2:], b[:, :, 2:])
