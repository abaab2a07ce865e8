"""GPU parity of the backbone operators on the tree tokens (App. G operator table and simplified
block; Sec. 2.1.2 positional indices) against the CPU oracle, through the C ABI."""
import math

import numpy as np
import pytest
import torch

import paper_2401_10774_amd as M
from paper_2401_10774_amd.block import SimplifiedBlock
from oracle import medusa_oracle as O
from workloads import draw_normal
from _harness import BOUND, TOL, check_close, record, row_rel_err, to_dev, to_host_f64

pytestmark = pytest.mark.gpu


def _bits_to_f64(x):
    return O.widen(x)


def linear_case(dtype, B, T, d_in, d_out, x_heads, y_heads, gated, seed):
    Mrows = B * T
    x = draw_normal(seed, 0, (Mrows, d_in), 1.0, dtype)
    w = draw_normal(seed, 1, (d_out, d_in), 0.02, dtype)
    mul = draw_normal(seed, 2, (Mrows, d_out), 1.0, dtype) if gated else None
    xd = to_dev(x)
    if x_heads:
        xd = xd.view(B, T, x_heads, d_in // x_heads).permute(0, 2, 1, 3).contiguous()     # head-major copy of the same values
    y = M.tree_linear(xd, to_dev(w), B, T, mul=None if mul is None else to_dev(mul), y_heads=y_heads)
    torch.cuda.synchronize()
    ref = O.tree_linear_ref(x, w, dtype, mul=mul)
    got = to_host_f64(y)
    if y_heads:
        got = O.from_heads(got)
    check_close(f"tree_linear {dtype} M={Mrows} {d_in}->{d_out}" + (" gated" if gated else ""), "y", got, ref, dtype, kind="rounded2")


@pytest.mark.parametrize("rows", [(1, 1), (1, 3), (1, 10), (1, 65), (2, 50), (4, 89)])
@pytest.mark.parametrize("variant", ["plain", "gated", "heads_in", "heads_out"])
def test_linear_bf16(rows, variant):
    B, T = rows
    linear_case("bf16", B, T, 512, 384, 4 if variant == "heads_in" else 0, 3 if variant == "heads_out" else 0,
                variant == "gated", 300 + B * T)


def test_linear_bf16_large_m_and_ragged_n():
    linear_case("bf16", 16, 65, 256, 1000, 0, 0, False, 401)          # 1040 rows: the large-M kernel, N not a tile multiple
    linear_case("bf16", 16, 65, 256, 1024, 2, 8, True, 402)           # all options at once
    linear_case("bf16", 3, 70, 1024, 200, 8, 0, False, 403)


def test_linear_bf16_large_tile_kernel():
    # enough output tiles (M/192 x N/256 >= 200) for the large-tile kernel: its vector epilogues,
    # both layouts on both sides, and the element-wise fallback for a ragged N
    linear_case("bf16", 16, 65, 128, 8704, 0, 0, False, 420)
    linear_case("bf16", 16, 65, 128, 8704, 2, 68, True, 421)
    linear_case("bf16", 16, 65, 128, 8700, 0, 0, True, 422)
    linear_case("bf16", 4, 89, 192, 25600, 0, 0, False, 423)          # 356 rows: two 192-row tiles


@pytest.mark.parametrize("rows,N,d,want", [
    (128, 4096, 128, dict(kind="skinny", m_blocks=4, mt=2, ksplit=1)),    # short reduction, narrow output: more row blocks, unsplit
    (96, 4096, 192, dict(kind="skinny", m_blocks=3, mt=2, ksplit=1)),
    (256, 5120, 128, dict(kind="skinny", m_blocks=3, mt=6, ksplit=1)),    # one more row block instead of eight row groups per workgroup
    (640, 4096, 128, dict(kind="square")),                                # a skinny launch would exceed one workgroup per CU
    (384, 11008, 128, dict(kind="big", wide=False)),                      # 129 tiles of 128 x 256: one round
    (768, 11008, 128, dict(kind="big", wide=True)),                       # 172 tiles of 192 x 256 beat 516 of 128 x 128
    (1040, 4096, 128, dict(kind="big", wide=False)),
    (2080, 4096, 128, dict(kind="big", wide=True)),
    (640, 4096, 8192, dict(kind="big", wide=False, ksplit=2)),            # long reduction into few large tiles: split over workgroups
    (640, 4096, 11008, dict(kind="big", wide=True, ksplit=4)),
    (420, 5000, 8192, dict(kind="big", wide=False, ksplit=2)),            # 20 column tiles, ragged: rotated over the dies per split
    (356, 5110, 13824, dict(kind="big", wide=False, ksplit=4)),
    (1040, 4096, 11008, dict(kind="big", wide=True, ksplit=2)),
    (4, 4096, 256, dict(kind="gemv")),                                    # eight-wavefront GEMV, 16 rows per workgroup
    (3, 16390, 256, dict(kind="gemv")),                                   # 32 rows per workgroup, ragged last workgroup
])
def test_linear_bf16_planner_branches(rows, N, d, want):
    """One shape per branch of the GEMM planning above 80 rows (and the wide GEMV); the plan is
    asserted first, so the case keeps testing the branch it was written for."""
    plan = M.medusa_gemm_plan(rows, N, d, 1, True)
    for key, value in want.items():
        assert plan[key] == value, f"plan {plan}, wanted {want}"
    linear_case("bf16", 1, rows, d, N, 0, 0, False, 440 + rows)
    linear_case("bf16", 1, rows, d, N, 0, 0, True, 441 + rows)


@pytest.mark.parametrize("dtype,B,T,d_in,heads,dh,segments,x_heads", [
    ("bf16", 4, 89, 320, 5, 64, 3, 0),        # 356 rows, Q, K, V of equal size
    ("bf16", 16, 65, 256, 2, 128, 2, 0),      # 1040 rows (large tiles), K and V of a grouped-query block
    ("bf16", 2, 10, 512, 4, 32, 3, 8),        # few rows, head-major activations
    ("bf16", 1, 3, 192, 3, 16, 2, 0),         # wave-per-row kernel
    ("f32", 2, 7, 64, 2, 8, 3, 0),
])
def test_linear_segments(dtype, B, T, d_in, heads, dh, segments, x_heads):
    """One call over the stacked weight rows fills `segments` head-major tensors; every segment must be
    what tree_linear gives for its own rows of the weight (oracle: the plain definition per segment)."""
    rows, d_out = B * T, segments * heads * dh
    x = draw_normal(460, 0, (rows, d_in), 1.0, dtype)
    w = draw_normal(460, 1, (d_out, d_in), 0.05, dtype)
    xd = to_dev(x)
    if x_heads:
        xd = xd.view(B, T, x_heads, d_in // x_heads).permute(0, 2, 1, 3).contiguous()
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    y = torch.full((segments, B, heads, T, dh), float("nan"), dtype=tdt, device="cuda")
    M.tree_linear_segments(xd, to_dev(w), B, T, y, heads)
    torch.cuda.synchronize()
    w64 = np.asarray(w)
    for s_ in range(segments):
        ref = O.tree_linear_ref(x, w64[s_ * heads * dh:(s_ + 1) * heads * dh], dtype)
        got = O.from_heads(to_host_f64(y[s_]))
        check_close(f"tree_linear_segments {dtype} M={rows} {d_in}->{d_out}", f"segment {s_}", got, ref, dtype, kind="rounded2")
    lib = M.lib()
    args = lambda seg, stride: (xd.data_ptr(), to_dev(w).data_ptr(), None, y.data_ptr(), B, T, d_in, d_out, x_heads, heads, seg,
                                stride, 1 if dtype == "bf16" else 0, None, 0, None)
    assert lib.tree_linear_segments(*args(segments, y[0].numel() - 1)) != 0      # segments would overlap
    assert lib.tree_linear_segments(*args(0, y[0].numel())) != 0
    if d_out % 7 != 0:
        assert lib.tree_linear_segments(*args(7, y[0].numel())) != 0             # no whole heads per segment


def test_linear_bf16_ring_kernel():
    # up to 96 rows per block: the kernel that fetches 1 KB runs into an LDS ring, with the gated epilogue,
    # head-major activations on both sides and tiles of 128, 96, 64 and 48 columns
    linear_case("bf16", 1, 65, 192, 25600, 0, 0, True, 430)
    linear_case("bf16", 2, 33, 256, 25600, 2, 200, False, 431)
    linear_case("bf16", 1, 10, 1024, 25610, 8, 0, True, 432)
    linear_case("bf16", 1, 65, 576, 19200, 0, 150, True, 433)        # 96 columns per workgroup
    linear_case("bf16", 1, 70, 1024, 12800, 8, 100, False, 434)      # 64
    linear_case("bf16", 1, 33, 320, 9600, 0, 0, True, 435)           # 48
    assert M.medusa_gemm_plan(130, 6400, 1024, 1, True)["m_blocks"] == 2
    linear_case("bf16", 2, 65, 1024, 6400, 8, 50, False, 445)        # two row blocks (interleaved with the column tiles), head-major both sides
    linear_case("bf16", 1, 150, 3072, 4224, 0, 0, True, 446)         # two row blocks, ragged second one, 88 column tiles (no multiple of 8)
    # two rows of a long reduction and three rows of a matrix of some size leave the wave-per-row kernel for this one
    assert M.medusa_gemm_plan(2, 4096, 11008, 1, True)["ring"] and M.medusa_gemm_plan(2, 4096, 8192, 1, True)["kind"] == "gemv"
    linear_case("bf16", 1, 2, 11008, 4096, 0, 0, True, 449)
    assert M.medusa_gemm_plan(3, 12288, 4096, 1, True)["ring"] and M.medusa_gemm_plan(4, 2048, 2048, 1, True)["kind"] == "gemv"
    linear_case("bf16", 1, 3, 4096, 12288, 32, 96, False, 450)
    assert M.medusa_gemm_plan(89, 19200, 576, 1, True)["mt"] == 6
    linear_case("bf16", 1, 89, 576, 19200, 0, 150, True, 447)        # six row groups (the 89 tokens of the 13B tree), 96 columns, gated, head-major output
    assert (M.medusa_gemm_plan(192, 5120, 5120, 1, True)["mt"], M.medusa_gemm_plan(192, 5120, 5120, 1, True)["m_blocks"]) == (6, 2)
    linear_case("bf16", 2, 96, 5120, 5120, 40, 0, False, 448)        # two blocks of six row groups, 48 columns
    # narrow outputs over a long reduction: the same kernel with its reduction split over workgroups;
    # a short reduction stays with the register-staged split kernel
    for rows, d_in, d_out, want in ((16, 3072, 4224, (True, 64, 2)), (65, 6144, 2176, (True, 64, 4)), (40, 12288, 256, (True, 64, 8)),
                                    (65, 6144, 4224, (True, 96, 4)), (16, 11776, 6272, (True, 128, 4)),
                                    (97, 11008, 4096, (True, 64, 2)), (97, 6144, 2048, (True, 64, 2)),      # ... with two and four row blocks
                                    (96, 11008, 4096, (True, 64, 4)), (178, 11008, 4096, (True, 64, 2)),     # ... with six row groups, one and two blocks
                                    (65, 2752, 4096, (False, 64, 2)), (16, 4096, 1024, (False, 64, 4))):
        plan = M.medusa_gemm_plan(rows, d_out, d_in, 1, True)
        assert (plan["ring"], plan["tile"], plan["ksplit"]) == want, plan
        linear_case("bf16", 1, rows, d_in, d_out, 0, 0, d_in == 4096, 436 + rows)


def interleave16(wg, wu):
    """Blocks of 16 gate rows followed by the same 16 up rows (numpy, independent of the library's helper)."""
    n, d = wg.shape
    out = np.empty((2 * n, d), wg.dtype)
    for b in range(n // 16):
        out[32 * b:32 * b + 16] = wg[16 * b:16 * b + 16]
        out[32 * b + 16:32 * b + 32] = wu[16 * b:16 * b + 16]
    return out


@pytest.mark.parametrize("B,T,d_in,d_out,x_heads,y_heads", [
    (1, 65, 512, 384, 0, 0), (1, 65, 512, 384, 4, 0), (2, 50, 256, 1008, 0, 3),
    (1, 5, 192, 64, 0, 0), (1, 1, 128, 48, 0, 0), (4, 89, 320, 400, 0, 0), (1, 33, 1024, 2064, 8, 0),
    (1, 89, 512, 2576, 0, 0), (1, 96, 1024, 2064, 8, 0), (2, 89, 320, 400, 0, 4),      # six row groups, one and two blocks
    # many rows: the large-tile kernel's epilogue (192- and 128-row tiles, ragged last column tile, both layouts)
    (16, 65, 128, 2688, 0, 0), (4, 89, 192, 6928, 3, 0), (16, 65, 128, 2560, 2, 20),
    (4, 89, 64, 13840, 0, 0)])
def test_linear_swiglu_bf16(B, T, d_in, d_out, x_heads, y_heads):
    swiglu_case(B, T, d_in, d_out, x_heads, y_heads)


def swiglu_case(B, T, d_in, d_out, x_heads, y_heads):
    seed = 700 + B * T
    M_rows = B * T
    x = draw_normal(seed, 0, (M_rows, d_in), 1.0, "bf16")
    wg = draw_normal(seed, 1, (d_out, d_in), 1.0 / math.sqrt(d_in), "bf16")
    wu = draw_normal(seed, 2, (d_out, d_in), 1.0 / math.sqrt(d_in), "bf16")
    xd = to_dev(x)
    if x_heads:
        xd = to_dev(np.ascontiguousarray(x.reshape(B, T, x_heads, d_in // x_heads).transpose(0, 2, 1, 3)))
    w_gu = to_dev(interleave16(wg, wu))
    assert torch.equal(w_gu, M.interleave_gate_up(to_dev(wg), to_dev(wu)))
    if M_rows > 100 and d_out >= 2560:
        assert M.medusa_gemm_plan(M_rows, 2 * d_out, d_in, 1, False)["kind"] == "big"      # (the case is here for that kernel)
    y = M.tree_linear_swiglu(xd, w_gu, B, T, y_heads=y_heads)
    torch.cuda.synchronize()
    got = to_host_f64(y)
    if y_heads:
        got = got.transpose(0, 2, 1, 3).reshape(M_rows, d_out)
    ref = O.tree_swiglu_ref(x, wg, wu, "bf16")
    check_close(f"tree_linear_swiglu M={M_rows} {d_in}->{d_out}", "y", got, ref, "bf16", kind="rounded2")


def test_linear_swiglu_rejects_what_it_does_not_cover():
    x = torch.zeros((4, 128), dtype=torch.float32, device="cuda")
    w = torch.zeros((64, 128), dtype=torch.float32, device="cuda")
    with pytest.raises(M.MedusaError):
        M.tree_linear_swiglu(x, w, 1, 4)                                # fp32
    xb, wb = x.bfloat16(), torch.zeros((40, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(M.MedusaError):
        M.tree_linear_swiglu(xb, wb, 1, 4)                              # 20 output columns: not a multiple of 16


def test_linear_f32():
    linear_case("f32", 1, 10, 256, 96, 0, 0, False, 410)
    linear_case("f32", 2, 10, 256, 128, 4, 2, True, 411)


def test_linear_rejects_bad_shapes():
    x = torch.zeros((4, 96), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((64, 96), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(M.MedusaError):
        M.tree_linear(x, w, 1, 4)                                      # d_in not a multiple of 64


@pytest.mark.parametrize("dtype,D,maxpos", [("bf16", 128, 8300), ("bf16", 64, 300), ("f32", 64, 200), ("f32", 128, 9000)])
def test_rope(dtype, D, maxpos):
    B, Hq, Hkv, T = 2, 4, 2, 9
    q = draw_normal(500, 0, (B, Hq, T, D), 1.0, dtype)
    k = draw_normal(500, 1, (B, Hkv, T, D), 1.0, dtype)
    rng = np.random.default_rng(7)
    pos = rng.integers(0, maxpos, size=(B, T)).astype(np.int32)
    pos[0, 0] = 0
    pos[1, -1] = maxpos
    qd, kd = to_dev(q), to_dev(k)
    M.tree_rope(qd, kd, to_dev(pos), 10000.0)
    torch.cuda.synchronize()
    for got, src in ((qd, q), (kd, k)):
        ref = O.rope_ref(src, pos, 10000.0, dtype)
        check_close(f"tree_rope {dtype} max position {maxpos}", "q/k", to_host_f64(got), ref, dtype, kind="rounded2")


def block_case(dtype, branching, B, h, Hq, Hkv, D, inter, Lcap, prefix, seed, adjacent_qkv=False, fused_gate_up=False):
    tree_o = O.tree_cartesian(branching)
    tree_g = M.MedusaTree(branching=branching)
    T = tree_o.T
    x = draw_normal(seed, 0, (B * T, h), 1.0, dtype)
    ws = {n: draw_normal(seed, 10 + i, shape, 1.0 / math.sqrt(shape[1]), dtype)
          for i, (n, shape) in enumerate((("wq", (Hq * D, h)), ("wk", (Hkv * D, h)), ("wv", (Hkv * D, h)),
                                          ("wu", (inter, Hq * D)), ("wg", (inter, Hq * D)), ("wd", (h, inter))))}
    kc = draw_normal(seed, 20, (B, Hkv, Lcap, D), 1.0, dtype)
    vc = draw_normal(seed, 21, (B, Hkv, Lcap, D), 1.0, dtype)
    pl = np.asarray(prefix, np.int32)
    pos = (pl[:, None] + np.asarray(tree_o.depth, np.int32)[None, :]).astype(np.int32)
    scale, theta = 1.0 / math.sqrt(D), 10000.0
    blk = SimplifiedBlock(tree_g, B, h, Hq, Hkv, D, inter, Lcap, torch.bfloat16 if dtype == "bf16" else torch.float32)
    dw = {n: to_dev(ws[n]) for n in ("wq", "wk", "wv", "wu", "wg", "wd")}
    if adjacent_qkv:      # W_Q, W_K, W_V as consecutive row blocks of one allocation: one projection call at B = 1
        wqkv = torch.cat([dw["wq"], dw["wk"], dw["wv"]], dim=0)
        dw["wq"], dw["wk"], dw["wv"] = wqkv[:Hq * D], wqkv[Hq * D:(Hq + Hkv) * D], wqkv[(Hq + Hkv) * D:]
    w_gu = M.interleave_gate_up(dw["wg"], dw["wu"]) if fused_gate_up else None
    out = blk.run(to_dev(x), *(dw[n] for n in ("wq", "wk", "wv", "wu", "wg", "wd")), to_dev(kc), to_dev(vc),
                  to_dev(pl), to_dev(pos), scale, w_gu)
    if adjacent_qkv and B == 1:
        assert len(blk._plans) == 1 and len(next(iter(blk._plans.values()))) == (5 if fused_gate_up else 6)   # the fused form did run
    if adjacent_qkv and B > 1:
        names = [c[0] for c in next(iter(blk._plans.values()))]
        assert names.count("tree_linear_segments") == 1 and names.index("tree_rope") == (1 if Hq == Hkv else 2)
    torch.cuda.synchronize()
    ref = O.simplified_block_ref(x, ws["wq"], ws["wk"], ws["wv"], ws["wu"], ws["wg"], ws["wd"], kc, vc, pl, pos, tree_o,
                                 Hq, Hkv, scale, theta, dtype)
    got = {"q": blk.q, "k": blk.k, "v": blk.v, "attn": blk.attn, "up": blk.up, "act": blk.act, "out": out}
    # end to end every intermediate inherits the rounding differences of its predecessors: a few
    # storage roundings deep, so the bound is the per-operator tolerance times the chain length
    depth = {"q": 2, "k": 2, "v": 1, "attn": 3, "up": 4, "act": 5, "out": 6}
    names = [n for n in ("q", "k", "v", "attn", "up", "act", "out") if not (fused_gate_up and n == "up")]   # no `up` in memory when fused
    for name in names:
        err = row_rel_err(to_host_f64(got[name]), ref[name])
        record(f"block {dtype} B={B} h={h} T={T} end to end", name, err)
        assert err <= BOUND[dtype]["rounded2"] * depth[name], f"{name}: rel err {err}"
    # stage-wise, from the GPU's own inputs: each operator alone meets the per-operator tolerance
    g64 = {n: to_host_f64(t) for n, t in got.items()}
    a_tok = O.from_heads(g64["attn"])
    checks = {
        "attn": (O.round_to_storage(O.tree_attention_ref(g64["q"], g64["k"], g64["v"], kc, vc, pl, tree_o, scale), dtype), g64["attn"]),
        "out": (O.tree_linear_ref(g64["act"], ws["wd"], dtype), g64["out"]),
    }
    if fused_gate_up:
        checks["act"] = (O.tree_swiglu_ref(a_tok, ws["wg"], ws["wu"], dtype), g64["act"])
    else:
        checks["up"] = (O.tree_linear_ref(a_tok, ws["wu"], dtype), g64["up"])
        checks["act"] = (O.tree_linear_ref(a_tok, ws["wg"], dtype, mul=g64["up"]), g64["act"])
    for name, (want, have) in checks.items():
        check_close(f"block {dtype} B={B} h={h} T={T} stage-wise", name, have, want, dtype, kind="rounded2")


def test_block_f32_small():
    block_case("f32", (3, 2), 1, 256, 4, 4, 64, 512, 160, [128], 600)


def test_block_bf16_gqa_ragged():
    block_case("bf16", (4, 3, 2, 1), 2, 512, 8, 2, 64, 1024, 700, [600, 37], 601)


def test_block_bf16_head_dim_128():
    block_case("bf16", (2, 2, 1), 1, 512, 4, 4, 128, 768, 400, [300], 602)


def test_block_bf16_fused_gate_and_up():
    block_case("bf16", (3, 2, 1), 2, 512, 8, 2, 64, 1024, 700, [600, 37], 605, fused_gate_up=True)       # 2 x 16 rows
    block_case("bf16", (2, 2, 1), 1, 512, 4, 4, 128, 768, 400, [300], 606, adjacent_qkv=True, fused_gate_up=True)
    block_case("bf16", (4, 3, 2, 1), 2, 512, 8, 2, 64, 1024, 700, [600, 37], 607, fused_gate_up=True)    # 130 rows: two row blocks
    block_case("bf16", (4, 3, 2, 1, 1), 1, 512, 8, 2, 64, 1024, 700, [600], 608, fused_gate_up=True)     # 89 rows: one block of six row groups
    block_case("bf16", (4, 3, 2, 1, 1), 2, 512, 8, 2, 64, 1024, 700, [37, 600], 609, fused_gate_up=True) # 178 rows: two such blocks


def test_block_bf16_batch_with_stacked_projection_weights():
    # a batch with W_Q, W_K, W_V in one allocation: one call for three tensors (equal head counts) or
    # one for Q and one for K and V (grouped-query attention)
    block_case("bf16", (4, 3, 2, 1), 3, 512, 4, 4, 128, 768, 400, [300, 17, 380], 605, adjacent_qkv=True)
    block_case("bf16", (3, 2, 1), 4, 512, 8, 2, 64, 1024, 300, [200, 0, 290, 100], 606, adjacent_qkv=True)


def test_block_bf16_fused_qkv_projection():
    block_case("bf16", (4, 3, 2, 1), 1, 512, 8, 2, 64, 1024, 300, [200], 603, adjacent_qkv=True)
    block_case("bf16", (2, 2, 1), 1, 512, 4, 4, 128, 768, 400, [300], 604, adjacent_qkv=True)


def test_block_replays_under_a_hip_graph():
    """The block's calls (split reductions with their tickets and workspace included) captured into
    one HIP graph reproduce the eager result bit for bit on every replay."""
    branching, B, h, Hq, Hkv, D, inter, Lcap = (4, 3, 2, 1), 1, 512, 8, 2, 64, 1024, 300
    tree = M.MedusaTree(branching=branching)
    T = tree.T
    x = to_dev(draw_normal(701, 0, (B * T, h), 1.0, "bf16"))
    shapes = (("wq", (Hq * D, h)), ("wk", (Hkv * D, h)), ("wv", (Hkv * D, h)), ("wu", (inter, Hq * D)),
              ("wg", (inter, Hq * D)), ("wd", (h, inter)))
    dw = {n: to_dev(draw_normal(701, 10 + i, s, 1.0 / math.sqrt(s[1]), "bf16")) for i, (n, s) in enumerate(shapes)}
    kc, vc = (to_dev(draw_normal(701, 20 + i, (B, Hkv, Lcap, D), 1.0, "bf16")) for i in range(2))
    pl = np.asarray([200], np.int32)
    pos = to_dev((pl[:, None] + np.asarray(tree.depth, np.int32)[None, :]).astype(np.int32))
    blk = SimplifiedBlock(tree, B, h, Hq, Hkv, D, inter, Lcap, torch.bfloat16)
    args = (x, *(dw[n] for n in ("wq", "wk", "wv", "wu", "wg", "wd")), kc, vc, to_dev(pl), pos, 1.0 / math.sqrt(D))
    for _ in range(2):
        out = blk.run(*args)
    torch.cuda.synchronize()
    eager = [t.clone() for t in (blk.q, blk.k, blk.v, blk.attn, blk.up, blk.act, out)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        blk.run(*args)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            blk.run(*args)
    torch.cuda.synchronize()
    for replay in range(4):
        for t in (blk.q, blk.k, blk.v, blk.attn, blk.up, blk.act, out):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager, (blk.q, blk.k, blk.v, blk.attn, blk.up, blk.act, out)):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"replay {replay}"
        blk.run(*args)                         # eager work between the replays
        torch.cuda.synchronize()


def _random_linear_shapes():
    """Seeded shapes across the planning's whole range: 1-400 rows, ragged column counts (multiples of 8), reductions
    that are any multiple of 64 -- partial last super-stages, ragged last tiles, every kernel family."""
    rng = np.random.default_rng(20240119)
    shapes = []
    while len(shapes) < 40:
        rows = int(rng.choice([1, 2, 3, 4, 5, 16, 33, 65, 80, 81, 89, 96, 97, 128, 130, 161, 192, 200, 260, 356, 400]))
        d_in = 64 * int(rng.integers(1, 180))
        d_out = 8 * int(rng.integers(8, 2600))
        if rows * d_in * d_out > 6e9:                      # keeps the float64 oracle product to about a second
            continue
        shapes.append((rows, d_in, d_out, bool(rng.integers(0, 2)), 700 + len(shapes)))
    return shapes


@pytest.mark.parametrize("rows,d_in,d_out,gated,seed", _random_linear_shapes())
def test_linear_bf16_random_shapes(rows, d_in, d_out, gated, seed):
    linear_case("bf16", 1, rows, d_in, d_out, 0, 0, gated, seed)


def _random_swiglu_shapes():
    """Seeded shapes for the fused gate/up projection: one to several row blocks of the ring kernel (1-6 row groups
    each), the large-tile kernel's epilogue, outputs that are any multiple of 16, reductions any multiple of 64."""
    rng = np.random.default_rng(20240774)
    shapes = []
    while len(shapes) < 14:
        rows = int(rng.choice([1, 3, 5, 16, 40, 65, 81, 89, 96, 97, 130, 178, 200, 260, 400]))
        d_in = 64 * int(rng.integers(1, 100))
        d_out = 16 * int(rng.integers(1, 900))
        if rows * d_in * d_out > 2.5e9:                    # keeps the float64 oracle products to about a second
            continue
        shapes.append((1, rows, d_in, d_out, 0, 0))
    return shapes


@pytest.mark.parametrize("B,T,d_in,d_out,x_heads,y_heads", _random_swiglu_shapes())
def test_linear_swiglu_bf16_random_shapes(B, T, d_in, d_out, x_heads, y_heads):
    swiglu_case(B, T, d_in, d_out, x_heads, y_heads)


def test_linear_bf16_more_than_4096_rows():
    """64 trees of 65 tokens (4160 rows) and beyond: plain, gated with head-major output, and the fused gate/up projection."""
    linear_case("bf16", 64, 65, 512, 768, 0, 0, False, 460)
    linear_case("bf16", 64, 65, 256, 1024, 2, 8, True, 461)
    linear_case("bf16", 128, 65, 128, 256, 0, 0, False, 462)         # 8320 rows
    swiglu_case(64, 65, 256, 512, 0, 0)
