"""Pins of the oracle's backbone-operator functions (App. G operator table and simplified block;
Sec. 2.1.2 positional indices).  Everything here is recomputed by independent code: explicit
loops, complex-number rotations, and a plain causal block run on each root-to-leaf path."""
import math

import numpy as np
import pytest

from oracle import medusa_oracle as O


def test_linear_is_row_times_matrix_brute_force():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 7)).astype(np.float32)
    w = rng.standard_normal((3, 7)).astype(np.float32)
    got = O.tree_linear_ref(x, w, "f32")
    for m in range(5):
        for n in range(3):
            s = 0.0
            for j in range(7):
                s += float(x[m, j]) * float(w[n, j])
            assert got[m, n] == np.float64(np.float32(s)) or abs(got[m, n] - s) <= 1e-6 * max(1.0, abs(s))
    # a transposed weight must fail this pin: check that the shapes really are out x in
    assert got.shape == (5, 3)


def test_gated_linear_closed_forms():
    # SiLU(0) = 0; SiLU(x) + SiLU(-x) = x tanh(x/2); SiLU(x) -> x for large x
    x = np.array([[1.0, 0.0], [0.0, 1.0]], np.float32)
    w = np.array([[0.0, 0.0], [3.0, 0.0], [-3.0, 0.0], [40.0, 0.0]], np.float32)     # rows: 0, 3, -3, 40 for token 0
    mul = np.full((2, 4), 2.0, np.float32)
    got = O.tree_linear_ref(x, w, "f32", mul=mul)
    assert got[0, 0] == 0.0
    assert abs((got[0, 1] + got[0, 2]) / 2.0 - 3.0 * math.tanh(1.5)) < 1e-6
    assert abs(got[0, 3] / 2.0 - 40.0) < 1e-5
    assert np.all(got[1] == 0.0)                                                   # token 1 sees only zeros


def test_swiglu_brute_force_and_special_cases():
    # independent loops with math.exp; a swapped gate and up, a missing SiLU or a transposed weight fail
    rng = np.random.default_rng(1)
    x = rng.standard_normal((4, 6)).astype(np.float32)
    wg = rng.standard_normal((5, 6)).astype(np.float32)
    wu = rng.standard_normal((5, 6)).astype(np.float32)
    got = O.tree_swiglu_ref(x, wg, wu, "f32")
    assert got.shape == (4, 5)
    for m in range(4):
        for n in range(5):
            g = sum(float(x[m, j]) * float(wg[n, j]) for j in range(6))
            u = sum(float(x[m, j]) * float(wu[n, j]) for j in range(6))
            want = g / (1.0 + math.exp(-g)) * u
            assert abs(got[m, n] - want) <= 1e-6 * max(1.0, abs(want))
    # zero gate rows give zero whatever the up rows are; a large gate passes the up projection times the gate
    e = np.eye(2, dtype=np.float32)
    assert np.all(O.tree_swiglu_ref(e, np.zeros((3, 2), np.float32), np.ones((3, 2), np.float32), "f32") == 0.0)
    big = O.tree_swiglu_ref(e, np.full((1, 2), 50.0, np.float32), np.full((1, 2), 3.0, np.float32), "f32")
    assert np.allclose(big, 150.0, rtol=1e-6)
    # it is the two-operator form without the intermediate rounding: equal to it in fp32 up to that rounding
    two_step = O.tree_linear_ref(x, wg, "f32", mul=O.tree_linear_ref(x, wu, "f32"))
    assert np.allclose(got, two_step, rtol=1e-5, atol=1e-6)


def _rope_complex(x, pos, theta):
    """Independent statement: the pair (x[j], x[j + D/2]) is the complex number x[j] + i x[j + D/2],
    multiplied by exp(i * pos * theta**(-2j/D))."""
    D = x.shape[-1]
    half = D // 2
    z = x[..., :half] + 1j * x[..., half:]
    freq = np.array([theta ** (-2.0 * j / D) for j in range(half)])
    z = z * np.exp(1j * pos * freq)
    return np.concatenate([z.real, z.imag], axis=-1)


def test_rope_closed_form_and_invariants():
    rng = np.random.default_rng(1)
    B, H, T, D = 2, 3, 5, 8
    x = rng.standard_normal((B, H, T, D))
    pos = np.array([[0, 1, 1, 2, 7], [10, 11, 12, 12, 13]])
    got = O.rope_ref(x, pos, 10000.0, "f32")
    for b in range(B):
        for h in range(H):
            for t in range(T):
                want = _rope_complex(x[b, h, t], pos[b, t], 10000.0)
                assert np.allclose(got[b, h, t], want, rtol=1e-6, atol=1e-6)
    # position 0 is the identity; equal positions (tree nodes of equal depth) get equal rotations
    assert np.allclose(got[0, :, 0], x[0, :, 0].astype(np.float32))
    same = O.rope_ref(np.broadcast_to(x[:, :, :1], x.shape).copy(), pos, 10000.0, "f32")
    assert np.array_equal(same[0, :, 1], same[0, :, 2]) and np.array_equal(same[1, :, 2], same[1, :, 3])
    # rotations preserve the norm of every pair
    half = D // 2
    assert np.allclose(got[..., :half] ** 2 + got[..., half:] ** 2, x[..., :half] ** 2 + x[..., half:] ** 2, rtol=1e-5)
    # D = 2: a plain rotation by the angle `position`
    v = np.array([[[[1.0, 0.0]]]])
    r = O.rope_ref(v, np.array([[3]]), 10000.0, "f32")
    assert np.allclose(r[0, 0, 0], [math.cos(3.0), math.sin(3.0)], atol=1e-6)


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(2)
    D = 16
    q = rng.standard_normal((1, 1, 1, D))
    k = rng.standard_normal((1, 1, 1, D))
    def score(m, n):
        a = O.rope_ref(q, np.array([[m]]), 500.0, "f32")
        b = O.rope_ref(k, np.array([[n]]), 500.0, "f32")
        return float((a * b).sum())
    assert abs(score(9, 4) - score(5, 0)) < 1e-4
    assert abs(score(100, 97) - score(3, 0)) < 1e-4
    assert abs(score(9, 4) - score(4, 9)) > 1e-3           # the sign of the offset matters


def _plain_causal_block(xs, wq, wk, wv, wu, wg, wd, Hq, Hkv, scale, theta):
    """A plain causal decoder block (same simplified data flow) on one sequence xs [n, h], positions
    0..n-1, written with explicit loops over tokens and heads."""
    n, h = xs.shape
    D = wq.shape[0] // Hq
    q = (xs @ wq.T).reshape(n, Hq, D)
    k = (xs @ wk.T).reshape(n, Hkv, D)
    v = (xs @ wv.T).reshape(n, Hkv, D)
    for t in range(n):
        for g in range(Hq):
            q[t, g] = _rope_complex(q[t, g], t, theta)
        for g in range(Hkv):
            k[t, g] = _rope_complex(k[t, g], t, theta)
    a = np.zeros((n, Hq, D))
    for t in range(n):
        for g in range(Hq):
            kv = g // (Hq // Hkv)
            s = np.array([scale * float(q[t, g] @ k[u, kv]) for u in range(t + 1)])
            p = np.exp(s - s.max())
            p /= p.sum()
            for u in range(t + 1):
                a[t, g] += p[u] * v[u, kv]
    a = a.reshape(n, Hq * D)
    gate = a @ wg.T
    act = gate / (1.0 + np.exp(-gate)) * (a @ wu.T)
    return act @ wd.T, k, v


@pytest.mark.parametrize("branching", [(2, 2), (3, 1, 2)])
def test_block_on_tree_equals_plain_causal_block_on_every_path(branching):
    """Sec. 2.1.2: a tree token sees exactly its own continuation, at positions that follow the tree.
    So the block's output at the nodes of a root-to-leaf path equals a plain causal block run on
    prefix + that path as an ordinary sequence."""
    rng = np.random.default_rng(3)
    tree = O.tree_cartesian(branching)
    T = tree.T
    B, L, Hq, Hkv, D, inter = 1, 6, 4, 2, 8, 24
    h = Hq * D
    theta, scale = 100.0, 1.0 / math.sqrt(D)
    wq, wk, wv = (rng.standard_normal((n, h)) * 0.3 for n in (Hq * D, Hkv * D, Hkv * D))
    wu, wg, wd = rng.standard_normal((inter, h)) * 0.3, rng.standard_normal((inter, h)) * 0.3, rng.standard_normal((h, inter)) * 0.3
    x_prefix = rng.standard_normal((L, h))
    x_tree = rng.standard_normal((T, h))
    # the cache holds the prefix keys (rotated at their positions) and values, as a decoder would have left them
    _, k_pre, v_pre = _plain_causal_block(x_prefix, wq, wk, wv, wu, wg, wd, Hq, Hkv, scale, theta)
    k_cache = np.zeros((B, Hkv, L + 4, D))
    v_cache = np.zeros((B, Hkv, L + 4, D))
    k_cache[0, :, :L] = k_pre.transpose(1, 0, 2)
    v_cache[0, :, :L] = v_pre.transpose(1, 0, 2)
    pos = (L + np.asarray(tree.depth))[None, :]
    res = O.simplified_block_ref(x_tree, wq, wk, wv, wu, wg, wd, k_cache, v_cache, np.array([L]), pos, tree,
                                 Hq, Hkv, scale, theta, "f32")
    for path in tree.paths:
        nodes = [int(n) for n in path if n >= 0]
        seq = np.concatenate([x_prefix, x_tree[nodes]], axis=0)
        want, _, _ = _plain_causal_block(seq, wq, wk, wv, wu, wg, wd, Hq, Hkv, scale, theta)
        got = res["out"][nodes]
        assert np.allclose(got, want[L:], rtol=2e-4, atol=2e-4), np.abs(got - want[L:]).max()


def test_head_layout_helpers_are_pure_reindexing():
    y = np.arange(2 * 3 * 4 * 5, dtype=np.float64).reshape(2 * 3, 4 * 5)      # B=2, T=3, H=4, Dh=5
    hm = O.to_heads(y, 2, 3, 4)
    assert hm.shape == (2, 4, 3, 5)
    assert hm[1, 2, 0, 3] == y[1 * 3 + 0, 2 * 5 + 3]
    assert np.array_equal(O.from_heads(hm), y)
