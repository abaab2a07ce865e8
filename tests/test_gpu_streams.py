"""Calls of the same entry point on different streams may overlap: every stream gets its own set of the
ticket counters that elect a launch's last workgroup.  Two streams run acceptance and top-k/tree
assembly on different inputs at the same time, many times over; every result must equal what the
same call gives alone."""
import numpy as np
import pytest
import torch

import paper_2401_10774_amd as M
from _harness import to_dev

pytestmark = pytest.mark.gpu


def test_accept_and_topk_on_two_streams_at_once():
    tree = M.MedusaTree(branching=(4, 3, 2, 1))
    B, V, K = 6, 32000, 4
    rng = np.random.default_rng(900)
    data = []
    for s in range(2):
        logits = to_dev(rng.standard_normal((B, tree.T, V)).astype(np.float32))
        tokens = to_dev(rng.integers(0, V, (B, tree.T)).astype(np.int32))
        heads = to_dev(rng.standard_normal((B, K, V)).astype(np.float32))
        lm = to_dev(rng.standard_normal((B, V)).astype(np.float32))
        pl = to_dev(rng.integers(0, 1000, B).astype(np.int32))
        alone_a = [t.clone() for t in M.medusa_accept(logits, tokens, tree, "typical", 0.7, 0.09, 0.3)]
        alone_t = [t.clone() for t in M.medusa_topk_tree(heads, lm, tree, pl)]
        data.append((logits, tokens, heads, lm, pl, alone_a, alone_t))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    results = [[], []]
    for it in range(25):
        for s in range(2):
            logits, tokens, heads, lm, pl, _, _ = data[s]
            with torch.cuda.stream(streams[s]):
                a = M.medusa_accept(logits, tokens, tree, "typical", 0.7, 0.09, 0.3)
                t = M.medusa_topk_tree(heads, lm, tree, pl)
            results[s].append((a, t))
    torch.cuda.synchronize()
    for s in range(2):
        _, _, _, _, _, alone_a, alone_t = data[s]
        for a, t in results[s]:
            assert all(torch.equal(x, y) for x, y in zip(a, alone_a))
            assert all(torch.equal(x, y) for x, y in zip(t, alone_t))
