"""CPU oracle for one Medusa verification step (arXiv 2401.10774).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain statement of what the
hot path computes; it exists so the HIP kernels can be checked against it.
Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
import it.  It shares no code with the HIP library and imports nothing from it.

Everything floating point is evaluated in float64 from the stored input bits
(float32 arrays, or bfloat16 bit patterns in ``uint16`` arrays, widened
exactly).  Each function states the passage of the paper it follows.  Where a
step has a textbook definition the function is that definition written out;
numpy's ``@`` and sort routines are used as library primitives.

Readings of points the paper leaves open (all mirrored by the HIP path):
  * weights are stored out x in, no biases (Sec. 2.1.1 writes W.h);
  * the residual-block output is rounded once to the storage dtype before the
    vocabulary projection; logits are never rounded;
  * ties in arg-max / top-k: larger value first, then lower token id;
  * the tree has N candidate nodes plus a root (node 0); nodes are numbered
    depth-major and lexicographically by rank tuple inside a depth;
  * candidates (root-to-leaf paths) are enumerated in lexicographic order of
    their rank tuples; among candidates with equally long accepted prefixes
    the first one wins;
  * p_original = softmax(logits / temperature); entropy in nats; strict ">";
  * accept length counts the root (1..K+1); the next root is the arg-max of the
    original model's logits at the last accepted node;
  * rejection-sampling acceptance: the paper names the scheme and defines
    nothing, so medusa_accept_sampled_ref is a reading (stated in its
    docstring): "parity unpinned" by the paper, pinned by the exact
    reproduction of the original model's distribution on a tiny case.

Pins: every function below is pinned by tests/test_oracle_*.py (closed forms,
brute force on tiny inputs, invariants from the paper).  The paper prints no
numeric worked example of the step, so no pin is a paper-printed value except
the node counts of Sec. 2.1.2 / Fig. 2.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------
# storage formats
# --------------------------------------------------------------------------

def widen(x: np.ndarray) -> np.ndarray:
    """Stored bits -> float64, exactly.  uint16 arrays hold bfloat16 patterns."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if x.dtype in (np.float32, np.float64):
        return x.astype(np.float64)
    raise TypeError(f"unsupported storage dtype {x.dtype}")


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float64 -> nearest bfloat16 value (ties to even), returned as float64.

    bfloat16: 1 sign, 8 exponent, 7 fraction bits.  Rounded directly from
    float64 (no intermediate float32 rounding).
    """
    x = np.asarray(x, dtype=np.float64)
    out = np.empty_like(x)
    finite = np.isfinite(x)
    out[~finite] = x[~finite]
    a = np.abs(x)
    tiny = finite & (a < 2.0 ** -126)           # bfloat16 subnormal range: spacing 2^-133
    normal = finite & ~tiny
    out[tiny] = np.rint(x[tiny] * 2.0 ** 133) * 2.0 ** -133
    bits = np.ascontiguousarray(x[normal]).view(np.uint64)
    drop = np.uint64(52 - 7)
    one = np.uint64(1)
    bias = ((bits >> drop) & one) + ((one << (drop - one)) - one)
    bits = (bits + bias) & ~((one << drop) - one)
    r = bits.view(np.float64)
    r = np.where(np.abs(r) >= 2.0 ** 128, np.copysign(np.inf, r), r)
    out[normal] = r
    return out


def round_to_f32(x: np.ndarray) -> np.ndarray:
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "f32":
        return round_to_f32(x)
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# candidate tree (Sec. 2.1.2, Fig. 2; sparse trees: Sec. 2.3.3)
# --------------------------------------------------------------------------

@dataclass
class Tree:
    K: int                       # levels below the root = Medusa heads used
    T: int                       # tokens: root + candidates
    nodes: List[Tuple[int, ...]]  # rank tuple of every node; nodes[0] == ()
    parent: np.ndarray           # [T] int32, parent[0] = -1
    depth: np.ndarray            # [T] int32, depth[0] = 0
    rank: np.ndarray             # [T] int32, rank[0] = -1
    topk_per_head: np.ndarray    # [K] int32: S_k = 1 + largest rank used at level k
    token_src: np.ndarray        # [T] int32 index into [root, top-S_1 of head 1, top-S_2 of head 2, ...]
    anc_mask: np.ndarray         # [T, 2] uint64: bit u set iff u is an ancestor of t or u == t
    paths: np.ndarray            # [n_leaves, K+1] int32 root-to-leaf node lists, -1 padded
    n_leaves: int


def tree_from_nodes(rank_tuples: Sequence[Sequence[int]]) -> Tree:
    """Tree tables from the set of candidate nodes, each given as its rank tuple
    (i_1, ..., i_k): the i_j-th top prediction of head j, for j = 1..k."""
    cand = sorted({tuple(int(r) for r in t) for t in rank_tuples}, key=lambda t: (len(t), t))
    if any(len(t) == 0 for t in cand):
        raise ValueError("the root is implicit; give candidate nodes only")
    nodes: List[Tuple[int, ...]] = [()] + cand
    index = {t: i for i, t in enumerate(nodes)}
    T = len(nodes)
    K = max((len(t) for t in nodes), default=0)
    parent = np.full(T, -1, np.int32)
    depth = np.zeros(T, np.int32)
    rank = np.full(T, -1, np.int32)
    for i, t in enumerate(nodes[1:], start=1):
        if min(t) < 0:
            raise ValueError("negative rank")
        if t[:-1] not in index:
            raise ValueError(f"node {t} has no parent in the set")
        parent[i], depth[i], rank[i] = index[t[:-1]], len(t), t[-1]
    S = np.zeros(K, np.int32)
    for t in nodes[1:]:
        S[len(t) - 1] = max(S[len(t) - 1], t[-1] + 1)
    head_base = np.concatenate([[1], 1 + np.cumsum(S)[:-1]]).astype(np.int32) if K else np.zeros(0, np.int32)
    token_src = np.zeros(T, np.int32)
    for i in range(1, T):
        token_src[i] = head_base[depth[i] - 1] + rank[i]
    anc = np.zeros((T, 2), np.uint64)
    for i in range(T):
        u = i
        while u >= 0:
            anc[i, u // 64] |= np.uint64(1) << np.uint64(u % 64)
            u = parent[u]
    has_child = np.zeros(T, bool)
    has_child[parent[1:]] = True
    leaves = sorted((nodes[i] for i in range(T) if not has_child[i]))     # lexicographic = DFS order
    paths = np.full((len(leaves), K + 1), -1, np.int32)
    for p, t in enumerate(leaves):
        for j in range(len(t) + 1):
            paths[p, j] = index[t[:j]]
    return Tree(K, T, nodes, parent, depth, rank, S, token_src, anc, paths, len(leaves))


def tree_cartesian(branching: Sequence[int]) -> Tree:
    """Sec. 2.1.2: level k holds every combination of the top-s_j predictions of
    heads j <= k, so s_k branches leave every level-(k-1) node."""
    level: List[Tuple[int, ...]] = [()]
    cand: List[Tuple[int, ...]] = []
    for s in branching:
        level = [t + (r,) for t in level for r in range(int(s))]
        cand.extend(level)
    return tree_from_nodes(cand)


def tree_optimized(accuracy: np.ndarray, n_nodes: int):
    """Sec. 2.3.3: accuracy[k-1][i] is the accuracy of the i-th best prediction of head k; a node
    (i_1..i_k) is estimated correct with probability prod_j accuracy[j-1][i_j] and contributes that
    much to the expected acceptance length.  Nodes are added one by one: always the node connected
    to the current tree (its parent is in it) with the highest estimate; ties go to the shallower
    node, then to the lexicographically smaller rank tuple.  Returns (Tree, expected accept length
    with the root counted)."""
    accuracy = np.asarray(accuracy, dtype=np.float64)
    K, S = accuracy.shape

    def estimate(t):
        p = 1.0
        for j, r in enumerate(t):
            p *= accuracy[j, r]
        return p

    tree_nodes = [()]
    chosen: List[Tuple[int, ...]] = []
    expect = 1.0
    for _ in range(n_nodes):
        cands = [t + (r,) for t in tree_nodes if len(t) < K for r in range(S) if t + (r,) not in tree_nodes]
        if not cands:
            raise ValueError("fewer nodes exist than requested")
        best = min(cands, key=lambda t: (-estimate(t), len(t), t))
        tree_nodes.append(best)
        chosen.append(best)
        expect += estimate(best)
    return tree_from_nodes(chosen), expect


# --------------------------------------------------------------------------
# (1) candidate generation: Medusa heads (Sec. 2.1.1) and top-k / tree tokens (Sec. 2.1.2)
# --------------------------------------------------------------------------

def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def medusa_heads_ref(hidden, w1, w2, dtype: str):
    """Sec. 2.1.1: logits_k = W2_k . (SiLU(W1_k . h) + h) for every row h of
    ``hidden`` [M, d]; w1 [K, d, d] (or None: no residual block, the plain LM
    head), w2 [K, V, d].  Returns (logits [M, K, V] float64, resid [M, K, d]
    float64 already rounded to the storage dtype)."""
    h = widen(hidden)
    M, d = h.shape
    K, V = w2.shape[0], w2.shape[1]
    logits = np.empty((M, K, V), np.float64)
    resid = np.empty((M, K, d), np.float64)
    for k in range(K):
        if w1 is None:
            r = h.copy()
        else:
            u = h @ widen(w1[k]).T
            r = round_to_storage(silu(u) + h, dtype)
        resid[:, k, :] = r
        logits[:, k, :] = r @ widen(w2[k]).T
    return logits, resid


def topk_ids_ref(row: np.ndarray, s: int) -> np.ndarray:
    """Indices of the s largest entries of a 1-D row, best first; equal values
    are ordered by lower index first."""
    row = np.asarray(row, dtype=np.float64)
    order = np.lexsort((np.arange(row.size), -row))
    return order[:s].astype(np.int32)


def medusa_topk_tree_ref(medusa_logits, lm_logits, tree: Tree, prefix_len):
    """Sec. 2.1.2: head k contributes its top-s_k tokens; the root is the LM
    head's greedy token (Sec. 2.3.1, first token); node t carries the token its
    (head, rank) selects and position prefix_len + depth (Fig. 2 caption).
    medusa_logits [B, K', V] with K' >= tree.K, lm_logits [B, V].
    Returns (topk_ids [B, K, S] -1 padded, tree_tokens [B, T], position_ids [B, T])."""
    B = lm_logits.shape[0]
    S = int(tree.topk_per_head.max()) if tree.K else 0
    topk = np.full((B, tree.K, S), -1, np.int32)
    tokens = np.empty((B, tree.T), np.int32)
    pos = np.empty((B, tree.T), np.int32)
    for b in range(B):
        flat = [int(topk_ids_ref(lm_logits[b], 1)[0])]
        for k in range(tree.K):
            s = int(tree.topk_per_head[k])
            ids = topk_ids_ref(medusa_logits[b, k], s)
            topk[b, k, :s] = ids
            flat.extend(int(i) for i in ids)
        for t in range(tree.T):
            tokens[b, t] = flat[tree.token_src[t]]
            pos[b, t] = int(prefix_len[b]) + int(tree.depth[t])
    return topk, tokens, pos


# --------------------------------------------------------------------------
# (2) candidate processing: tree attention (Sec. 2.1.2)
# --------------------------------------------------------------------------

def tree_attention_ref(q, k_tree, v_tree, k_cache, v_cache, prefix_len, tree: Tree, scale: float):
    """Sec. 2.1.2: softmax attention in which tree token t sees the whole
    prefix and, among tree tokens, only its predecessors on its own
    continuation (and itself).  q [B, Hq, T, D]; k_tree, v_tree [B, Hkv, T, D];
    k_cache, v_cache [B, Hkv, Lcap, D] of which rows < prefix_len[b] are the
    prefix.  Query head g reads KV head g // (Hq // Hkv).  Returns float64
    [B, Hq, T, D]."""
    B, Hq, T, D = q.shape
    Hkv = k_tree.shape[1]
    group = Hq // Hkv
    visible_tree = np.zeros((T, T), bool)
    for t in range(T):
        for u in range(T):
            visible_tree[t, u] = bool((int(tree.anc_mask[t, u // 64]) >> (u % 64)) & 1)
    out = np.empty((B, Hq, T, D), np.float64)
    for b in range(B):
        L = int(prefix_len[b])
        visible = np.concatenate([np.ones((T, L), bool), visible_tree], axis=1)
        for g in range(Hq):
            h = g // group
            keys = np.concatenate([widen(k_cache[b, h, :L]), widen(k_tree[b, h])], axis=0)
            vals = np.concatenate([widen(v_cache[b, h, :L]), widen(v_tree[b, h])], axis=0)
            s = (widen(q[b, g]) @ keys.T) * scale
            s = np.where(visible, s, -np.inf)
            p = np.exp(s - s.max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            out[b, g] = p @ vals
    return out


# --------------------------------------------------------------------------
# (3) accepting candidates (Sec. 2.3.1) and carrying the result over (Fig. 1)
# --------------------------------------------------------------------------

@dataclass
class AcceptResult:
    accept_len: np.ndarray        # [B] int32, root included: 1..K+1
    best_node: np.ndarray         # [B] int32 last accepted node
    path_nodes: np.ndarray        # [B, K+1] int32, -1 padded
    accepted_tokens: np.ndarray   # [B, K+1] int32, -1 padded
    next_root: np.ndarray         # [B] int32 greedy token of the original model at best_node
    ok: np.ndarray                # [B, T] bool per-node test (ok[:, 0] = True)
    margin: np.ndarray            # [B, T] float64 distance of each per-node decision from flipping
    argmax_gap: np.ndarray        # [B, T] float64 top-1 minus top-2 logit of every row


def typical_threshold_ref(z_row: np.ndarray, temperature: float, eps: float, delta: float):
    """Sec. 2.3.1: for one row of original-model logits, p = softmax(z / temperature),
    H = -sum p ln p, threshold = min(eps, delta * exp(-H)).  Returns (p, H, threshold)."""
    z = np.asarray(z_row, dtype=np.float64) / temperature
    e = np.exp(z - z.max())
    p = e / e.sum()
    nz = p > 0
    H = -np.sum(p[nz] * np.log(p[nz]))
    return p, H, min(eps, delta * np.exp(-H))


def medusa_accept_ref(logits, tree_tokens, tree: Tree, mode: str,
                      temperature: float = 1.0, eps: float = 0.0, delta: float = 0.0) -> AcceptResult:
    """Sec. 2.3.1.  Every candidate (root-to-leaf path) is examined; its token at
    depth j >= 1 passes if the original model, reading the row of the node
    before it, (greedy) has it as arg-max, or (typical) gives it probability
    above min(eps, delta exp(-H)).  The root is accepted unconditionally.  A
    candidate's accepted prefix ends before its first failing token; the
    longest accepted prefix over all candidates wins (first candidate on ties).
    logits [B, T, V] rows of the original model at every tree token."""
    logits = np.asarray(logits, dtype=np.float64)
    B, T, V = logits.shape
    K = tree.K
    ok = np.zeros((B, T), bool)
    margin = np.full((B, T), np.inf)
    gap = np.empty((B, T))
    res = AcceptResult(np.zeros(B, np.int32), np.zeros(B, np.int32), np.full((B, K + 1), -1, np.int32),
                       np.full((B, K + 1), -1, np.int32), np.zeros(B, np.int32), ok, margin, gap)
    for b in range(B):
        top1 = np.empty(T, np.int64)
        for t in range(T):
            two = np.lexsort((np.arange(V), -logits[b, t]))[:2]
            top1[t] = two[0]
            gap[b, t] = logits[b, t, two[0]] - logits[b, t, two[1]] if V > 1 else np.inf
        ok[b, 0] = True
        for t in range(1, T):
            par, tok = int(tree.parent[t]), int(tree_tokens[b, t])
            if mode == "greedy":
                ok[b, t] = tok == top1[par]
                margin[b, t] = abs(logits[b, par, top1[par]] - logits[b, par, tok]) if not ok[b, t] else gap[b, par]
            elif mode == "typical":
                p, H, thr = typical_threshold_ref(logits[b, par], temperature, eps, delta)
                ok[b, t] = p[tok] > thr
                margin[b, t] = abs(np.log(max(p[tok], 1e-300)) - np.log(max(thr, 1e-300)))
            else:
                raise ValueError(mode)
        best_len, best_path = 0, None
        for path in tree.paths:
            n = 1
            while n <= K and path[n] >= 0 and ok[b, path[n]]:
                n += 1
            if n > best_len:
                best_len, best_path = n, path
        res.accept_len[b] = best_len
        res.best_node[b] = best_path[best_len - 1]
        res.path_nodes[b, :best_len] = best_path[:best_len]
        res.accepted_tokens[b, :best_len] = tree_tokens[b, best_path[:best_len]]
        res.next_root[b] = top1[res.best_node[b]]
    return res


@dataclass
class SampledAcceptResult:
    accept_len: np.ndarray        # [B] int32, root included
    best_node: np.ndarray         # [B] int32 last accepted node
    path_nodes: np.ndarray        # [B, K+1] int32, -1 padded
    accepted_tokens: np.ndarray   # [B, K+1] int32, -1 padded
    next_token: np.ndarray        # [B] int32 token sampled after the last accepted node
    margin: np.ndarray            # [B] float64 smallest distance of a uniform from the boundary it was compared with


def medusa_accept_sampled_ref(logits, tree_tokens, tree: Tree, uniforms, temperature: float = 1.0) -> SampledAcceptResult:
    """Sec. 2 (opening paragraph) and Sec. 2.3.1 (first paragraph) name "the rejection sampling
    scheme as used in speculative decoding" as the acceptance rule that keeps the original model's
    distribution, without defining it.  READING (parity unpinned by the paper; pinned by the
    distribution it must reproduce): Medusa's candidates under a node are a deterministic list, so
    each child, in rank order, is a draft whose proposal distribution is a point mass on its token x.
    Speculative rejection sampling against the current target distribution r then accepts x with
    probability min(1, r(x) / 1) = r(x), and after a rejection continues with the normalised
    residual max(r - point mass, 0), i.e. r with x removed and renormalised.  With
    p = softmax(logits[node] / temperature) as the first target, child i of a node is therefore
    accepted iff all earlier children were rejected and
        u_i < p(x_i) / (1 - sum_{j<i} p(x_j)),
    u_i = uniforms[b, child i].  The walk starts at the root (always accepted) and moves to the
    accepted child while there is one.  At the node where it stops the next token is drawn from
    the final residual (p without the tokens of that node's children, renormalised; p itself at a
    leaf) by inversion in token-id order with the uniform uniforms[b, 0] (the root's slot, which no
    test uses): the smallest token y whose cumulative residual mass exceeds u * total.
    logits [B, T, V]; tree_tokens [B, T]; uniforms [B, T] in [0, 1)."""
    logits = np.asarray(logits, dtype=np.float64)
    uniforms = np.asarray(uniforms, dtype=np.float64)
    B, T, V = logits.shape
    K = tree.K
    res = SampledAcceptResult(np.zeros(B, np.int32), np.zeros(B, np.int32), np.full((B, K + 1), -1, np.int32),
                              np.full((B, K + 1), -1, np.int32), np.zeros(B, np.int32), np.full(B, np.inf))
    children = [[c for c in range(T) if tree.parent[c] == t] for t in range(T)]      # in node order = rank order
    for b in range(B):
        node, path = 0, [0]
        while True:
            z = logits[b, node] / temperature
            e = np.exp(z - z.max())
            p = e / e.sum()
            removed = 0.0                      # probability mass of the children rejected so far
            moved = False
            for c in children[node]:
                x = int(tree_tokens[b, c])
                ratio = p[x] / (1.0 - removed) if removed < 1.0 else 0.0
                res.margin[b] = min(res.margin[b], abs(uniforms[b, c] - ratio))
                if uniforms[b, c] < ratio:
                    node, moved = c, True
                    path.append(c)
                    break
                removed += p[x]
            if moved:
                continue
            resid = p.copy()
            for c in children[node]:
                resid[int(tree_tokens[b, c])] = 0.0
            cdf = np.cumsum(resid)
            target = uniforms[b, 0] * cdf[-1]
            y = int(np.searchsorted(cdf, target, side="right"))
            y = min(y, V - 1)
            while resid[y] == 0.0 and y > 0:   # (rounding at the upper end only; a removed token is never drawn)
                y -= 1
            lo, hi = cdf[y] - resid[y], cdf[y]       # the drawn token's interval; its ends at 0 and at the total decide nothing
            if lo > 0.0:
                res.margin[b] = min(res.margin[b], (target - lo) / cdf[-1])
            if hi < cdf[-1]:
                res.margin[b] = min(res.margin[b], (hi - target) / cdf[-1])
            res.next_token[b] = y
            break
        n = len(path)
        res.accept_len[b] = n
        res.best_node[b] = path[-1]
        res.path_nodes[b, :n] = path
        res.accepted_tokens[b, :n] = [int(tree_tokens[b, t]) for t in path]
    return res


def kv_commit_ref(k_cache, v_cache, k_tree, v_tree, path_nodes, accept_len, prefix_len):
    """Fig. 1 / Sec. 2: the accepted prefix becomes context for the next step.
    For every layer and KV head the tree rows of the accepted path are appended,
    in path order, behind the prefix; the prefix grows by the accept length.
    Caches [NL, B, Hkv, Lcap, D] and prefix_len [B] are updated in place."""
    B = prefix_len.shape[0]
    for b in range(B):
        L, a = int(prefix_len[b]), int(accept_len[b])
        for j in range(a):
            node = int(path_nodes[b, j])
            k_cache[:, b, :, L + j, :] = k_tree[:, b, :, node, :]
            v_cache[:, b, :, L + j, :] = v_tree[:, b, :, node, :]
        prefix_len[b] = L + a


# --------------------------------------------------------------------------
# backbone operators on the tree tokens (App. G: table of operator shapes, "Parallel decoding"
# rows, and the simplified block of the latency model)
# --------------------------------------------------------------------------

def tree_linear_ref(x, w, dtype: str, mul=None):
    """App. G, operator table, parallel-decoding rows X W_Q / X W_K / X W_V / X W_u / X W_g /
    X W_d: every tree token's feature row times a weight matrix.  x [M, d_in], w [d_out, d_in]
    (stored out x in, as for the heads), result [M, d_out] rounded once to the storage dtype.
    With ``mul`` [M, d_out] given, the result is SiLU(x w^T) * mul before rounding (the gated
    feed-forward of the Llama family the appendix models: gate and up projections combined)."""
    y = widen(x) @ widen(w).T
    if mul is not None:
        y = silu(y) * widen(mul)
    return round_to_storage(y, dtype)


def tree_swiglu_ref(x, w_gate, w_up, dtype: str):
    """The gated feed-forward's inner product of App. G's operator table (X W_g and X W_u), combined
    as the Llama family does: SiLU(x w_gate^T) * (x w_up^T), with no rounding of either projection
    on the way; result [M, d_out] rounded once to the storage dtype."""
    xv = widen(x)
    return round_to_storage(silu(xv @ widen(w_gate).T) * (xv @ widen(w_up).T), dtype)


def rope_ref(x, position_ids, theta: float, dtype: str):
    """Rotary position embedding at the tree's positional indices (Sec. 2.1.2: the indices follow
    the tree structure, i.e. position = prefix length + depth of the node; they are an input
    here).  x [B, H, T, D]; position_ids [B, T].  Half-split pairing of the Llama family: element
    j < D/2 is paired with element j + D/2 and the pair is rotated by the angle
    position * theta**(-2j/D).  Result rounded once to the storage dtype."""
    xv = widen(x)
    B, H, T, D = xv.shape
    half = D // 2
    inv_freq = theta ** (-(2.0 * np.arange(half, dtype=np.float64)) / D)
    ang = np.asarray(position_ids, np.float64)[:, None, :, None] * inv_freq[None, None, None, :]   # [B,1,T,half]
    c, sn = np.cos(ang), np.sin(ang)
    lo, hi = xv[..., :half], xv[..., half:]
    out = np.concatenate([lo * c - hi * sn, hi * c + lo * sn], axis=-1)
    return round_to_storage(out, dtype)


def to_heads(y, B: int, T: int, H: int):
    """[B*T, H*Dh] token-major -> [B, H, T, Dh] head-major (pure re-indexing)."""
    return np.ascontiguousarray(np.asarray(y).reshape(B, T, H, -1).transpose(0, 2, 1, 3))


def from_heads(y):
    """[B, H, T, Dh] head-major -> [B*T, H*Dh] token-major (pure re-indexing)."""
    B, H, T, Dh = np.asarray(y).shape
    return np.ascontiguousarray(np.asarray(y).transpose(0, 2, 1, 3).reshape(B * T, H * Dh))


def simplified_block_ref(x, wq, wk, wv, wu, wg, wd, k_cache, v_cache, prefix_len, position_ids, tree: Tree,
                         Hq: int, Hkv: int, scale: float, theta: float, dtype: str):
    """The simplified decoder block whose latency App. G models, run on the tree tokens: the
    operators X W_Q, X W_K, X W_V, Q K^T, P V, X W_u, X W_g, X W_d in sequence.  The appendix
    lists the operators only; the data flow taken here is the Llama one without norms, output
    projection and residuals: q, k, v = x W^T, rotary embedding of q and k at the tree positions,
    tree attention against the cache, then down(SiLU(gate(a)) * up(a)) on the attention output a.
    x [B*T, h] token-major.  Every operator's result is rounded to the storage dtype.  Returns a
    dict of all intermediates (float64 values on the storage grid)."""
    B = len(prefix_len)
    T = tree.T
    q = rope_ref(to_heads(tree_linear_ref(x, wq, dtype), B, T, Hq), position_ids, theta, dtype)
    k = rope_ref(to_heads(tree_linear_ref(x, wk, dtype), B, T, Hkv), position_ids, theta, dtype)
    v = to_heads(tree_linear_ref(x, wv, dtype), B, T, Hkv)
    attn = round_to_storage(tree_attention_ref(q, k, v, k_cache, v_cache, prefix_len, tree, scale), dtype)
    a = from_heads(attn)
    up = tree_linear_ref(a, wu, dtype)
    act = tree_linear_ref(a, wg, dtype, mul=up)
    out = tree_linear_ref(act, wd, dtype)
    return {"q": q, "k": k, "v": v, "attn": attn, "up": up, "act": act, "out": out}


# --------------------------------------------------------------------------
# the whole step, chained (Sec. 2, opening paragraph: the three substeps of a decoding step)
# --------------------------------------------------------------------------

@dataclass
class StepResult:
    medusa_logits: np.ndarray     # [B, K, V]
    lm_logits_last: np.ndarray    # [B, V]
    topk_ids: np.ndarray
    tree_tokens: np.ndarray
    position_ids: np.ndarray
    attn_out: np.ndarray          # [B, Hq, T, D]
    verify_logits: np.ndarray     # [B, T, V]
    accept: AcceptResult
    prefix_len: np.ndarray        # after the commit


def verification_step_ref(x: dict, tree: Tree, dtype: str, scale: float, mode: str, temperature: float,
                          eps: float, delta: float, attn_layer: int = 0, plant=None) -> StepResult:
    """One verification iteration on the arrays of ``x`` (names as in workloads.TENSOR_IDS):
    heads on h_last, top-k and tree assembly, tree attention on one cache layer, the original
    model's logits at every tree token (LM head on hidden_tree), acceptance, commit.
    Caches and prefix_len in ``x`` are updated in place.  ``plant`` may adjust the verification
    logits before acceptance (test harness only)."""
    B, T = x["hidden_tree"].shape[0], x["hidden_tree"].shape[1]
    d = x["h_last"].shape[1]
    medusa_logits, _ = medusa_heads_ref(x["h_last"], x["w1"], x["w2"], dtype)
    lm_last, _ = medusa_heads_ref(x["h_last"], None, x["w_lm"][None], dtype)
    lm_last = lm_last[:, 0]
    topk, tokens, pos = medusa_topk_tree_ref(medusa_logits, lm_last, tree, x["prefix_len"])
    attn = tree_attention_ref(x["q"], x["k_tree"][attn_layer], x["v_tree"][attn_layer], x["k_cache"][attn_layer],
                              x["v_cache"][attn_layer], x["prefix_len"], tree, scale)
    ver, _ = medusa_heads_ref(x["hidden_tree"].reshape(B * T, d), None, x["w_lm"][None], dtype)
    ver = ver[:, 0].reshape(B, T, -1)
    if plant is not None:
        ver = plant(ver, tokens)
    acc = medusa_accept_ref(ver, tokens, tree, mode, temperature, eps, delta)
    kv_commit_ref(x["k_cache"], x["v_cache"], x["k_tree"], x["v_tree"], acc.path_nodes, acc.accept_len, x["prefix_len"])
    return StepResult(medusa_logits, lm_last, topk, tokens, pos, attn, ver, acc, x["prefix_len"])
