"""Pins for the oracle's Medusa heads (Sec. 2.1.1) and top-k / tree-token assembly (Sec. 2.1.2)."""
import math

import numpy as np
import pytest

from oracle import medusa_oracle as O
from workloads import bf16_bits_from_f32, draw_normal


def test_silu_closed_form_values():
    # SiLU(x) = x * sigmoid(x); literals evaluated by hand from sigmoid(1) = 0.7310585786300049
    x = np.array([0.0, 1.0, -1.0, 20.0, -20.0])
    want = np.array([0.0, 0.7310585786300049, -0.2689414213699951, 20.0 * (1 - 2.061153618190011e-09),
                     -20.0 * 2.0611536181902037e-09])
    assert np.allclose(O.silu(x), want, rtol=1e-13, atol=0)


def test_head_hand_case_d2():
    # d = 2, V = 3, K = 1, one row, float32 storage (all numbers exactly representable)
    h = np.array([[1.0, -2.0]], np.float32)
    w1 = np.array([[[0.5, 0.25], [-1.0, 0.0]]], np.float32)          # out x in
    w2 = np.array([[[1.0, 0.0], [0.0, 1.0], [2.0, -1.0]]], np.float32)
    u = [0.5 * 1 + 0.25 * -2, -1.0 * 1 + 0.0 * -2]                   # W1 . h = [0, -1]
    r = [u[0] / (1 + math.exp(-u[0])) + 1.0, u[1] / (1 + math.exp(-u[1])) - 2.0]
    r = [float(np.float32(v)) for v in r]                             # rounded to storage
    want = [r[0], r[1], 2 * r[0] - r[1]]
    logits, resid = O.medusa_heads_ref(h, w1, w2, "f32")
    assert logits.shape == (1, 1, 3)
    assert np.allclose(logits[0, 0], want, rtol=1e-15, atol=0)
    assert np.allclose(resid[0, 0], r, rtol=0, atol=0)
    # transposing W1 must change the answer (orientation is out x in)
    logits_t, _ = O.medusa_heads_ref(h, w1.transpose(0, 2, 1).copy(), w2, "f32")
    assert not np.allclose(logits_t, logits)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_zero_w1_head_equals_lm_head(dtype):
    """Sec. 2.1.1: W1 = 0 and W2 = LM head make a Medusa head reproduce the LM head."""
    M, d, V, K = 3, 64, 50, 2
    h = draw_normal(11, 0, (M, d), 1.0, dtype)
    w_lm = draw_normal(11, 4, (V, d), 0.02, dtype)
    w1 = np.zeros((K, d, d), h.dtype)
    w2 = np.stack([w_lm] * K)
    logits, resid = O.medusa_heads_ref(h, w1, w2, dtype)
    lm, _ = O.medusa_heads_ref(h, None, w_lm[None], dtype)
    plain = O.widen(h) @ O.widen(w_lm).T                              # the library routine it reduces to
    for k in range(K):
        assert np.array_equal(logits[:, k], lm[:, 0])
        assert np.array_equal(resid[:, k], O.widen(h))
    assert np.allclose(lm[:, 0], plain, rtol=1e-14, atol=1e-16)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_heads_against_scalar_loops(dtype):
    """Every element recomputed with Python floats and math.exp, one dot product at a time."""
    M, d, V, K = 2, 8, 5, 2
    h = draw_normal(12, 0, (M, d), 1.0, dtype)
    w1 = draw_normal(12, 2, (K, d, d), 0.5, dtype)
    w2 = draw_normal(12, 3, (K, V, d), 0.5, dtype)
    hf, w1f, w2f = O.widen(h), O.widen(w1), O.widen(w2)
    logits, resid = O.medusa_heads_ref(h, w1, w2, dtype)
    for m in range(M):
        for k in range(K):
            r = []
            for n in range(d):
                u = math.fsum(float(w1f[k, n, j]) * float(hf[m, j]) for j in range(d))
                val = u / (1.0 + math.exp(-u)) + float(hf[m, n])
                r.append(float(O.round_to_storage(np.array([val]), dtype)[0]))
            assert np.allclose(resid[m, k], r, rtol=0, atol=1e-7 if dtype == "f32" else 1e-2)
            # the stored residual is what the projection must consume
            rr = [float(x) for x in resid[m, k]]
            for v in range(V):
                want = math.fsum(float(w2f[k, v, j]) * rr[j] for j in range(d))
                assert abs(logits[m, k, v] - want) <= 1e-13 * max(1.0, abs(want))
    if dtype == "bf16":
        bits = bf16_bits_from_f32(resid.astype(np.float32))
        assert np.array_equal(O.widen(bits), resid)                   # residual is exactly bf16-representable


def py_topk(row, s):
    return [i for _, i in sorted((-float(v), i) for i, v in enumerate(row))][:s]


def test_topk_bruteforce_with_ties():
    rng = np.random.default_rng(2)
    for trial in range(200):
        V = int(rng.integers(1, 17))
        row = rng.integers(-2, 3, V).astype(np.float32)               # many ties
        s = int(rng.integers(1, V + 1))
        assert list(O.topk_ids_ref(row, s)) == py_topk(row, s)
    assert list(O.topk_ids_ref(np.array([0.0, -0.0, 0.0], np.float32), 3)) == [0, 1, 2]   # -0.0 == +0.0
    assert list(O.topk_ids_ref(np.array([1.0, 3.0, 3.0, 2.0], np.float32), 3)) == [1, 2, 3]


def test_topk_tree_assembly_hand_case():
    tree = O.tree_cartesian((2, 3))
    V = 6
    lm = np.array([[0.0, 5.0, 1.0, 5.0, 0.0, 0.0]], np.float32)                  # tie 1 vs 3 -> 1
    heads = np.array([[[9.0, 0.0, 8.0, 0.0, 0.0, 0.0],                           # head 1: 0, 2
                       [0.0, 1.0, 2.0, 3.0, 4.0, 5.0]]], np.float32)             # head 2: 5, 4, 3
    topk, tokens, pos = O.medusa_topk_tree_ref(heads, lm, tree, np.array([7], np.int32))
    assert topk.tolist() == [[[0, 2, -1], [5, 4, 3]]]
    # nodes: root, (0),(1), (0,0),(0,1),(0,2),(1,0),(1,1),(1,2)
    assert tokens.tolist() == [[1, 0, 2, 5, 4, 3, 5, 4, 3]]
    assert pos.tolist() == [[7, 8, 8, 9, 9, 9, 9, 9, 9]]
    # every candidate is one element of the Cartesian product of the per-head top lists
    cands = {tuple(tokens[0, n] for n in p[1:]) for p in tree.paths}
    assert cands == {(a, b) for a in (0, 2) for b in (5, 4, 3)}


def test_topk_tree_random_against_python_sort():
    tree = O.tree_cartesian((3, 2))
    B, V = 3, 40
    rng = np.random.default_rng(8)
    heads = rng.integers(-5, 6, (B, 2, V)).astype(np.float32)
    lm = rng.integers(-5, 6, (B, V)).astype(np.float32)
    pl = np.array([3, 0, 11], np.int32)
    topk, tokens, pos = O.medusa_topk_tree_ref(heads, lm, tree, pl)
    for b in range(B):
        flat = py_topk(lm[b], 1) + py_topk(heads[b, 0], 3) + py_topk(heads[b, 1], 2)
        assert tokens[b].tolist() == [flat[s] for s in tree.token_src]
        assert pos[b].tolist() == [int(pl[b]) + int(dd) for dd in tree.depth]
