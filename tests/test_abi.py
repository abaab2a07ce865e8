"""CPU-side checks of the boundary: the library loads, exports what include/medusa.h declares,
builds the same tree tables as the oracle, and rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2401_10774_amd as M
from paper_2401_10774_amd import binding
from oracle import medusa_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "medusa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+char\s*\*|int|size_t)\s+(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    L = M.lib()
    names = declared_functions()
    assert len(names) >= 14
    for n in names:
        assert hasattr(L, n), f"{n} declared in medusa.h but not exported"
    assert sorted(binding.EXPORTED_SYMBOLS) == names


def test_status_strings():
    L = M.lib()
    assert L.medusa_status_string(0) == b"ok"
    assert len({L.medusa_status_string(c) for c in (0, -1, -2, -3, -4, -99)}) == 6


TABLES = "parent depth rank token_src anc_mask paths topk_per_head".split()


@pytest.mark.parametrize("branching", [(2, 3), (3, 2), (4, 3, 2, 1), (4, 3, 2, 1, 1), (1,), (16,), (2, 2, 2, 2, 2, 2)])
def test_cartesian_tables_equal_the_oracles(branching):
    g, o = M.MedusaTree(branching=branching), O.tree_cartesian(branching)
    assert (g.T, g.K, g.n_leaves, g.S) == (o.T, o.K, o.n_leaves, int(o.topk_per_head.max()))
    for name in TABLES:
        assert np.array_equal(getattr(g, name), getattr(o, name)), name


def test_sparse_tables_equal_the_oracles():
    rng = np.random.default_rng(41)
    for trial in range(20):
        nodes = {()}
        while len(nodes) < 1 + int(rng.integers(1, 100)):
            p = list(nodes)[int(rng.integers(len(nodes)))]
            if len(p) < 6:
                nodes.add(p + (int(rng.integers(0, 12)),))
        cand = [n for n in nodes if n]
        rng.shuffle(cand)
        g, o = M.MedusaTree(nodes=cand), O.tree_from_nodes(cand)
        assert (g.T, g.K, g.n_leaves) == (o.T, o.K, o.n_leaves)
        for name in TABLES:
            assert np.array_equal(getattr(g, name), getattr(o, name)), name


def test_tree_limits_and_errors():
    with pytest.raises(M.MedusaError, match="invalid"):
        M.MedusaTree(nodes=[(0,), (1, 0)])                  # parent (1,) missing
    with pytest.raises(M.MedusaError, match="invalid"):
        M.MedusaTree(nodes=[(0,), (0,)])                    # duplicate
    with pytest.raises(M.MedusaError, match="range"):
        M.MedusaTree(branching=(4, 4, 4, 4))                # 340 nodes > 127
    with pytest.raises(M.MedusaError, match="range"):
        M.MedusaTree(branching=(17,))                       # rank >= 16
    with pytest.raises(M.MedusaError, match="invalid"):
        M.MedusaTree(branching=(2, 0))
    t = M.MedusaTree(branching=(126,)) if False else M.MedusaTree(nodes=[(i,) for i in range(16)])
    assert t.T == 17 and t.S == 16
    one = M.MedusaTree(nodes=[])
    assert (one.T, one.K, one.n_leaves) == (1, 0, 1) and one.paths.tolist() == [[0]]


def test_argument_checks_happen_on_the_host():
    """Null pointers and unsupported sizes are refused with a status code; nothing is launched."""
    L = M.lib()
    t = M.MedusaTree(branching=(2, 2))
    p = ctypes.c_void_p(4096)                              # never dereferenced: checks fail first
    assert L.medusa_heads(None, None, p, None, p, 1, 64, 10, 1, 1, None) == -1
    assert L.medusa_heads(p, p, p, None, p, 1, 64, 10, 1, 1, None) == -1          # w1 without resid
    assert L.medusa_heads(p, None, p, None, p, 0, 64, 10, 1, 1, None) == -1
    assert L.medusa_heads(p, None, p, None, p, 1, 72, 10, 1, 1, None) == -2       # bf16 needs d % 64 == 0
    assert L.medusa_heads(p, None, p, None, p, 1, 64, 10, 9, 1, None) == -2       # K > 8
    assert L.medusa_heads(p, None, p, None, p, 1, 64, 10, 1, 7, None) == -1       # unknown dtype
    assert L.medusa_heads(p, None, p, None, p, 16385, 64, 10, 1, 1, None) == -2   # more rows than a call takes
    assert L.tree_linear(p, p, None, p, 129, 128, 64, 64, 0, 0, 1, None, 0, None) == -2        # 16512 rows
    assert L.tree_attention(p, p, p, p, p, p, t.handle, p, 1, 4, 3, 128, 64, 1.0, 1, p, 1 << 30, None) == -1
    assert L.tree_attention(p, p, p, p, p, p, t.handle, p, 1, 4, 4, 96, 64, 1.0, 1, p, 1 << 30, None) == -2
    assert L.tree_attention(None, p, p, p, p, p, t.handle, p, 1, 4, 4, 128, 64, 1.0, 1, p, 1 << 30, None) == -1
    assert L.medusa_accept(p, p, t.handle, 1, 100, 5, 1.0, 0.1, 0.1, p, p, p, p, p, p, 1 << 20, None) == -1
    assert L.medusa_accept(p, p, t.handle, 1, 100, 1, 0.0, 0.1, 0.1, p, p, p, p, p, p, 1 << 20, None) == -1
    big = M.MedusaTree(branching=(4, 3, 2, 1))                                    # T = 65
    assert L.medusa_accept(p, p, big.handle, 1024, 100, 0, 1.0, 0.1, 0.1, p, p, p, p, p, p, 1 << 40, None) == -2   # B*T rows exceed a grid dimension
    # one activation row beyond the 64 KB the wave-per-row kernels stage in LDS: refused, not a division by zero
    assert L.tree_linear(p, p, None, p, 1, 1, 40960, 64, 0, 0, 1, None, 0, None) == -2
    assert L.tree_linear(p, p, None, p, 1, 4, 65536, 64, 0, 0, 1, None, 0, None) == -2
    assert L.tree_linear(p, p, None, p, 1, 2, 32768, 64, 0, 0, 0, None, 0, None) == -2         # fp32: 128 KB per row
    assert L.kv_commit(p, p, p, p, p, 3, p, p, None, 1, 1, 1, 7, 4, 16, 1, None) == -2  # 8-byte rows
    assert L.kv_commit(p, p, p, None, p, 3, p, p, None, 1, 1, 1, 7, 64, 16, 1, None) == -1
    assert L.medusa_topk_tree(p, None, t.handle, p, 1, 100, 2, p, p, p, p, 1 << 20, None) == -1
    assert L.medusa_topk_tree(p, p, t.handle, p, 1, 100, 1, p, p, p, p, 1 << 20, None) == -1   # fewer heads than levels
    assert L.tree_interleave_gate_up(p, None, p, 32, 64, 1, None) == -1
    assert L.tree_interleave_gate_up(p, p, p, 24, 64, 1, None) == -2                            # rows in blocks of 16
    assert L.tree_interleave_gate_up(p, p, p, 32, 12, 1, None) == -2                            # 24-byte rows
    assert L.tree_interleave_gate_up(p, p, ctypes.c_void_p(4100), 32, 64, 1, None) == -2        # misaligned
    assert L.tree_attention_workspace_bytes(1, 32, 32, 65, 128, 1152) % 256 == 0
    assert L.tree_attention_workspace_bytes(1, 32, 5, 65, 128, 1152) == 0
    assert L.medusa_accept_workspace_bytes(2, 65, 32000) > 0
    assert L.medusa_topk_tree_workspace_bytes(2, 4) > 0


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(M.MedusaError, match="device memory"):
        M.medusa_heads(torch.zeros(1, 64), None, torch.zeros(1, 10, 64))


def test_gemm_plans_are_launchable():
    """Host logic of the GEMM planning: over a grid of shapes every plan names an arrangement the
    launch code has a kernel for, its row blocks cover all rows, and a split reduction appears
    only with a workspace and is matched by a workspace size."""
    import paper_2401_10774_amd as M
    L = M.lib()
    shapes = [(4096, 4096), (11008, 4096), (4096, 11008), (12288, 4096), (22016, 4096), (32000, 4096),
              (1024, 4096), (5120, 5120), (13824, 5120), (5120, 13824), (32000, 5120), (192, 64), (64, 128)]
    for N, d in shapes:
        for K in (1, 5):
            for rows in (1, 2, 3, 4, 5, 16, 17, 64, 65, 80, 81, 96, 128, 129, 192, 256, 356, 512, 640, 768, 1040, 2080, 3584):
                for ws in (False, True):
                    p = M.medusa_gemm_plan(rows, N, d, K, ws)
                    what = f"M={rows} N={N} d={d} K={K} ws={ws}: {p}"
                    if p["kind"] == "gemv":     # one or two rows; three or four only on small matrices
                        assert rows <= 2 or (rows <= 4 and K * N * d <= 8 << 20), what
                        continue
                    assert rows > 1, what
                    assert p["kind"] in ("skinny", "square", "big"), what
                    if p["kind"] == "big":
                        assert rows > 96, what
                        continue
                    if p["kind"] == "square":       # 128 x 128 tiles
                        assert rows > 96 and p["ksplit"] == 1 and p["m_blocks"] * 128 >= rows, what
                        continue
                    assert 1 <= p["mt"] <= 8 and p["m_blocks"] >= 1, what
                    assert p["m_blocks"] * p["mt"] * 16 >= rows, what
                    assert p["ksplit"] in (1, 2, 4, 8), what
                    assert ws or p["ksplit"] == 1, what
                    assert not p["wide"] or p["mt"] <= 6, what
                    assert p["tile"] in (48, 64, 96, 128), what
                    assert not p["ring"] or p["mt"] <= 6, what
                    assert not (p["ring"] and p["ksplit"] > 1) or (d + 511) // 512 // p["ksplit"] >= 3, what
                    assert p["ring"] or p["tile"] in (64, 128), what
                    if p["ksplit"] > 1:
                        assert (d // 64) // p["ksplit"] >= 1, what
                        if K == 1:
                            assert L.tree_linear_workspace_bytes(1, rows, d, N, 1) > 0, what
    with pytest.raises(M.MedusaError):
        M.medusa_gemm_plan(0, 64, 64)
