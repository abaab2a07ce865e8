"""medusa_verify_logits + medusa_accept_fused (the acceptance step's row reductions taken in the epilogue
of the LM-head GEMM, Sec. 2.3.1) against medusa_heads + the oracle: the logits must be the same bits,
greedy acceptance exact on them, typical acceptance exact unless the oracle reports a probability
within 1e-4 of its threshold."""
import math

import numpy as np
import pytest
import torch

import paper_2401_10774_amd as M
from oracle import medusa_oracle as O
from workloads import draw_normal
from _harness import check_close, to_dev, to_host_bits, bits

pytestmark = pytest.mark.gpu


def case(branching, B, d, V, mode, temperature, eps, delta, seed, plant=True):
    gt, ot = M.MedusaTree(branching=branching), O.tree_cartesian(branching)
    T = ot.T
    rows = B * T
    assert M.medusa_verify_fused_available(rows, d, V, torch.bfloat16), "the case is here for the fused epilogue"
    rng = np.random.default_rng(seed)
    w = draw_normal(seed, 4, (V, d), 0.02, "bf16")
    hidden = draw_normal(seed, 1, (B, T, d), 1.0, "bf16")
    tokens = np.empty((B, T), np.int32)
    for b in range(B):
        for p in range(T):
            kids = [c for c in range(T) if ot.parent[c] == p]
            tokens[b, kids] = rng.choice(V, len(kids), replace=False)
        tokens[b, 0] = rng.integers(V)
    if plant:                                   # make one path per sequence acceptable: its parents' hidden rows point at the child token
        wf = O.widen(w)
        for b in range(B):
            path = [int(n) for n in ot.paths[rng.integers(ot.n_leaves)] if n >= 0]
            for j in range(1, int(rng.integers(1, len(path) + 1))):
                row = 40.0 * wf[tokens[b, path[j]]]
                hidden[b, path[j - 1]] = (torch.from_numpy(row).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    dh, dw = to_dev(hidden.reshape(rows, d)), to_dev(w)
    logits, stats = M.medusa_verify_logits(dh, dw, mode, temperature)
    plain, _ = M.medusa_heads(dh, None, dw.view(1, V, d))
    torch.cuda.synchronize()
    assert torch.equal(logits.view(torch.int32), plain.view(rows, V).view(torch.int32))          # the same kernel, the same bits
    ref_logits, _ = O.medusa_heads_ref(hidden.reshape(rows, d), None, w[None], "bf16")
    check_close(f"verify_logits fused M={rows} d={d} V={V}", "logits", logits.cpu().numpy(), ref_logits[:, 0], "bf16")
    g_logits = logits.view(B, T, V)
    got = [t.cpu().numpy() for t in M.medusa_accept_fused(g_logits, stats, to_dev(tokens), gt, mode, temperature, eps, delta)]
    scan = [t.cpu().numpy() for t in M.medusa_accept(g_logits, to_dev(tokens), gt, mode, temperature, eps, delta)]
    ref = O.medusa_accept_ref(g_logits.cpu().numpy(), tokens, ot, mode, temperature, eps, delta)
    want = [ref.accept_len, ref.best_node, ref.path_nodes, ref.accepted_tokens, ref.next_root]
    if mode == "typical" and not all(np.array_equal(x, y) for x, y in zip(got, want)):
        assert ref.margin[:, 1:].min() < 1e-4, "typical acceptance differs with no decision near its threshold"
        pytest.fail("tie-ambiguous typical decision at this seed")
    for x, y, z in zip(got, want, scan):
        assert np.array_equal(x, y) and np.array_equal(z, y)
    return ref.accept_len


def test_greedy_batch4_tree89():
    a = case((4, 3, 2, 1, 1), 4, 512, 32000, "greedy", 1.0, 0.0, 0.0, 301)
    assert len(set(a.tolist())) >= 2


def test_typical_batch16_tree65():
    a = case((4, 3, 2, 1), 16, 512, 32000, "typical", 0.7, 0.09, 0.3, 302, plant=False)
    assert a.min() >= 1
    a = case((4, 3, 2, 1), 16, 512, 32000, "typical", 0.7, 0.09, 0.3, 303, plant=True)
    assert len(set(a.tolist())) >= 2


def test_ragged_vocabulary_and_rows():
    # V is no multiple of 8 (scalar epilogue, ragged last column tile), rows no multiple of the tile height
    case((4, 3, 2, 1), 7, 256, 32003, "greedy", 1.0, 0.0, 0.0, 304)
    case((4, 3, 2, 1), 7, 256, 32003, "typical", 1.3, 0.09, 0.3, 305)


def test_mismatched_statistics_are_reported():
    gt = M.MedusaTree(branching=(4, 3, 2, 1))
    B, d, V = 8, 256, 32000
    dh = to_dev(draw_normal(306, 1, (B * gt.T, d), 1.0, "bf16"))
    dw = to_dev(draw_normal(306, 4, (V, d), 0.02, "bf16"))
    tok = torch.zeros((B, gt.T), dtype=torch.int32, device="cuda")
    logits, stats = M.medusa_verify_logits(dh, dw, "greedy", 1.0)
    out = M.medusa_accept_fused(logits.view(B, gt.T, V), stats, tok, gt, "typical", 0.7, 0.09, 0.3)
    torch.cuda.synchronize()
    assert (out[0].cpu().numpy() == -1).all()                  # statistics were produced without a temperature
    logits, stats = M.medusa_verify_logits(dh, dw, "typical", 0.7)
    out = M.medusa_accept_fused(logits.view(B, gt.T, V), stats, tok, gt, "typical", 0.9, 0.09, 0.3)
    torch.cuda.synchronize()
    assert (out[0].cpu().numpy() == -1).all()                  # ... or for another one
    out = M.medusa_accept_fused(logits.view(B, gt.T, V), stats, tok, gt, "greedy")
    torch.cuda.synchronize()
    assert (out[0].cpu().numpy() >= 1).all()                   # keys are always there
    assert M.lib().medusa_verify_logits(dh.data_ptr(), dw.data_ptr(), logits.data_ptr(), stats.data_ptr(), 1024, B * gt.T, d, V,
                                        1, 0, 1.0, None) == -3
    assert not M.medusa_verify_fused_available(65, 4096, 32000, torch.bfloat16)
    assert M.lib().medusa_verify_logits(dh.data_ptr(), dw.data_ptr(), logits.data_ptr(), stats.data_ptr(), 1 << 30, 65, d, V,
                                        1, 0, 1.0, None) == -2
