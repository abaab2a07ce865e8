"""tree_attention_static, the entry point for callers that cannot allocate: its split partials live in
an array built into the library instead of a caller workspace.  Called through the C ABI, two calls
in a row (the second on a smaller input, so stale partials of the first are still in the array), it
must reproduce tree_attention bit for bit and match the oracle; shapes beyond the array are refused
on the host."""
import ctypes
import math

import numpy as np
import pytest
import torch

import paper_2401_10774_amd as M
from oracle import medusa_oracle as O
from workloads import draw_normal
from _harness import check_close, poison_tail, to_dev, to_host_f64

pytestmark = pytest.mark.gpu


def one_call(tree_g, tree_o, B, Hq, Hkv, D, Lcap, prefix, seed):
    T = tree_o.T
    q = draw_normal(seed, 5, (B, Hq, T, D), 1.0, "bf16")
    kt = draw_normal(seed, 6, (B, Hkv, T, D), 1.0, "bf16")
    vt = draw_normal(seed, 7, (B, Hkv, T, D), 1.0, "bf16")
    kc = draw_normal(seed, 8, (B, Hkv, Lcap, D), 1.0, "bf16")
    vc = draw_normal(seed, 9, (B, Hkv, Lcap, D), 1.0, "bf16")
    pl = np.asarray(prefix, np.int32)
    scale = 1.0 / math.sqrt(D)
    dq, dkt, dvt, dpl = to_dev(q), to_dev(kt), to_dev(vt), to_dev(pl)
    dkc, dvc = to_dev(poison_tail(kc, pl)), to_dev(poison_tail(vc, pl))
    out = torch.full_like(dq, float("nan"))
    L = M.lib()
    stream = torch.cuda.current_stream().cuda_stream
    before = torch.cuda.memory_allocated()
    rc = L.tree_attention_static(dq.data_ptr(), dkt.data_ptr(), dvt.data_ptr(), dkc.data_ptr(), dvc.data_ptr(),
                                 dpl.data_ptr(), tree_g.handle, out.data_ptr(), B, Hq, Hkv, D, Lcap,
                                 ctypes.c_float(scale), 1, stream)
    assert rc == 0, L.medusa_status_string(rc)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    want = M.tree_attention(dq, dkt, dvt, dkc, dvc, dpl, tree_g, scale)       # caller workspace, same kernels
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), want.view(torch.int16))
    ref = O.tree_attention_ref(q, kt, vt, kc, vc, pl, tree_o, scale)
    got = to_host_f64(out)
    assert np.isfinite(got).all()
    check_close(f"tree_attention_static B={B} heads={Hq}/{Hkv} prefix={list(prefix)}", "out", got, ref, "bf16", kind="rounded")


def test_two_calls_in_a_row_second_smaller():
    branching = (4, 3, 2, 1)
    tree_g, tree_o = M.MedusaTree(branching=branching), O.tree_cartesian(branching)
    one_call(tree_g, tree_o, 2, 8, 4, 128, 1400, [1300, 700], 120)     # several splits per head
    one_call(tree_g, tree_o, 1, 4, 2, 128, 700, [333], 121)            # smaller: fewer heads, splits and keys
    one_call(tree_g, tree_o, 1, 2, 2, 128, 64, [0], 122)               # a single split: the array is not used at all


def test_shapes_beyond_the_array_are_refused_on_the_host():
    L = M.lib()
    tree = M.MedusaTree(branching=(4, 3, 2, 1))
    assert L.tree_attention_static_scratch_bytes() == 8 << 20
    p = ctypes.c_void_p(4096)                                           # never dereferenced: the size check comes first
    assert L.tree_attention_workspace_bytes(16, 32, 8, 65, 128, 4224) > 8 << 20
    rc = L.tree_attention_static(p, p, p, p, p, p, tree.handle, p, 16, 32, 8, 128, 4224, ctypes.c_float(0.1), 1, None)
    assert rc == -5 and b"scratch" in L.medusa_status_string(rc)
    assert L.tree_attention_static(p, p, p, p, p, p, None, p, 1, 4, 4, 128, 64, ctypes.c_float(0.1), 1, None) == -1
