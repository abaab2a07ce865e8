"""GPU parity: medusa_heads (HIP, through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

import paper_2401_10774_amd as M
from oracle import medusa_oracle as O
from workloads import draw_normal, get_config, make_step_inputs
from _harness import TOL, bits, check_close, resid_bound, row_rel_err, to_dev, to_host_bits, to_host_f64

pytestmark = pytest.mark.gpu


def run_case(dtype, M_rows, d, V, K, with_w1, seed):
    h = draw_normal(seed, 0, (M_rows, d), 1.0, dtype)
    w1 = draw_normal(seed, 2, (K, d, d), 0.02, dtype) if with_w1 else None
    w2 = draw_normal(seed, 3, (K, V, d), 0.02, dtype)
    logits, resid = M.medusa_heads(to_dev(h), None if w1 is None else to_dev(w1), to_dev(w2))
    torch.cuda.synchronize()
    ref_logits, ref_resid = O.medusa_heads_ref(h, w1, w2, dtype)
    case = f"heads {dtype} M={M_rows} d={d} V={V} K={K}"
    err = check_close(case, "logits behind the residual block" if with_w1 else "logits", to_host_f64(logits), ref_logits, dtype,
                      kind="resid" if with_w1 else "logits", bound=resid_bound(dtype, d) if with_w1 else None)
    if with_w1:
        check_close(case, "residual", to_host_f64(resid), ref_resid, dtype, kind="rounded2")
    return err


# M spans the wave-per-row path (<= 4) and the MFMA path (> 4) with ragged row tiles; V = 1000 / 333
# leaves ragged 64-row workgroup tails; d spans several reduction steps.
@pytest.mark.parametrize("M_rows", [1, 2, 3, 4, 5, 16, 17, 65, 81, 100])
@pytest.mark.parametrize("with_w1", [True, False])
def test_bf16_shapes(M_rows, with_w1):
    run_case("bf16", M_rows, 512, 1000, 2, with_w1, 50 + M_rows)


@pytest.mark.parametrize("d,V,K", [(64, 7, 1), (192, 333, 3), (4096, 130, 1), (5120, 70, 2)])
def test_bf16_odd_sizes(d, V, K):
    for M_rows in (1, 4, 10):
        run_case("bf16", M_rows, d, V, K, True, 60)


# The skinny MFMA kernel walks the reduction in stages of 128 elements: an odd number of 64-element
# steps leaves half of the last stage empty.  Narrow (64-column) and wide (128-column, from 200
# tiles) workgroup tiles, few and many row groups, with and without a ragged last tile.
@pytest.mark.parametrize("M_rows,d,V,K", [(65, 320, 1000, 2), (70, 192, 12800, 2), (128, 64, 300, 1),
                                          (120, 448, 12900, 2), (33, 704, 25700, 1)])
def test_bf16_odd_step_counts(M_rows, d, V, K):
    run_case("bf16", M_rows, d, V, K, False, 80 + M_rows)


# Up to 96 rows per block with 160 tiles or more: the kernel that fetches 1 KB runs per weight row
# straight into an LDS ring (super-stages of 512 elements, tiles of 48 to 128 columns).  Row groups
# 1..6, ragged last tile, one to several super-stages, partial last one, every tile width
# (250 / 200 / 200 / 201 workgroups), reductions shorter than the ring (three sub-stages in all), and
# two row blocks with a ragged second one.
@pytest.mark.parametrize("M_rows,d,V,K", [(70, 192, 12800, 2), (33, 704, 25700, 1),
                                          (5, 512, 25600, 1), (17, 1024, 6400, 4), (48, 1600, 12803, 2),
                                          (64, 64, 25600, 1), (80, 2560, 25601, 1),
                                          (65, 1088, 19190, 1), (40, 576, 12790, 1), (75, 512, 9640, 1),
                                          (10, 64, 7700, 1), (10, 192, 7700, 1), (16, 512, 7700, 1),
                                          (130, 1024, 6400, 1), (155, 1024, 6400, 1),
                                          (89, 1024, 6400, 4), (96, 1600, 25600, 1), (81, 192, 12800, 2)])   # six row groups: the partial tiles pass through LDS in two halves
def test_bf16_ring_kernel(M_rows, d, V, K):
    assert M.medusa_gemm_plan(M_rows, V, d, K, False)["ring"]
    run_case("bf16", M_rows, d, V, K, False, 90 + M_rows)


@pytest.mark.parametrize("M_rows", [1, 3, 4, 10])
def test_f32_shapes(M_rows):
    err = run_case("f32", M_rows, 256, 1000, 2, True, 70 + M_rows)
    assert err < 1e-5
    run_case("f32", M_rows, 8, 5, 1, False, 71)


def test_config1_exact_shapes():
    cfg = get_config("C1")
    x = make_step_inputs(cfg, ["h_last", "hidden_tree", "w1", "w2", "w_lm"])
    logits, _ = M.medusa_heads(to_dev(x["h_last"]), to_dev(x["w1"]), to_dev(x["w2"]))
    ref, _ = O.medusa_heads_ref(x["h_last"], x["w1"], x["w2"], "f32")
    assert row_rel_err(to_host_f64(logits), ref) <= 1e-5
    hid = x["hidden_tree"].reshape(cfg.B * cfg.T, cfg.d)
    ver, _ = M.medusa_heads(to_dev(hid), None, to_dev(x["w_lm"][None]))
    ref, _ = O.medusa_heads_ref(hid, None, x["w_lm"][None], "f32")
    assert row_rel_err(to_host_f64(ver), ref) <= 1e-5


def test_zero_w1_head_reproduces_the_lm_head_bitwise():
    """Sec. 2.1.1 initialisation: W1 = 0, W2 = LM head.  SiLU(0) + h = h exactly, so both paths
    must feed identical operands to the same projection kernel."""
    d, V, K = 256, 500, 2
    for dtype in ("bf16", "f32"):
        h = to_dev(draw_normal(80, 0, (3, d), 1.0, dtype))
        w_lm = to_dev(draw_normal(80, 4, (V, d), 0.02, dtype))
        w1 = torch.zeros((K, d, d), dtype=h.dtype, device="cuda")
        w2 = torch.stack([w_lm] * K).contiguous()
        heads, resid = M.medusa_heads(h, w1, w2)
        lm, _ = M.medusa_heads(h, None, w_lm[None].contiguous())
        assert np.array_equal(to_host_bits(resid[:, 0]), to_host_bits(h))
        for k in range(K):
            assert torch.equal(heads[:, k], lm[:, 0])


def test_run_twice_is_bit_identical():
    h = to_dev(draw_normal(81, 0, (65, 512), 1.0, "bf16"))
    w2 = to_dev(draw_normal(81, 3, (1, 2000, 512), 0.02, "bf16"))
    a, _ = M.medusa_heads(h, None, w2)
    b, _ = M.medusa_heads(h, None, w2)
    assert torch.equal(a, b)


def _random_head_shapes():
    """Seeded shapes over the whole range of medusa_heads: 1-400 rows, 1-5 heads, any vocabulary size (odd ones take
    the element-wise epilogue), hidden sizes that are any multiple of 64."""
    rng = np.random.default_rng(240110774)
    shapes = []
    while len(shapes) < 24:
        rows = int(rng.choice([1, 2, 3, 4, 5, 16, 48, 65, 81, 89, 96, 97, 130, 178, 260, 400]))
        d = 64 * int(rng.integers(1, 90))
        V = int(rng.integers(1, 33000))
        K = int(rng.integers(1, 6))
        with_w1 = bool(rng.integers(0, 2))
        if rows * K * d * (V + (d if with_w1 else 0)) > 5e9:      # keeps the float64 oracle to about a second
            continue
        shapes.append((rows, d, V, K, with_w1, 300 + len(shapes)))
    return shapes


@pytest.mark.parametrize("M_rows,d,V,K,with_w1,seed", _random_head_shapes())
def test_bf16_random_shapes(M_rows, d, V, K, with_w1, seed):
    run_case("bf16", M_rows, d, V, K, with_w1, seed)


@pytest.mark.parametrize("M_rows,d,V,K,with_w1", [(4160, 256, 1000, 1, False), (5000, 128, 300, 2, True), (8200, 64, 520, 1, False)])
def test_bf16_more_than_4096_rows(M_rows, d, V, K, with_w1):
    """A batch of 64 trees of 65 tokens is 4160 rows: the row limit of a call is 16384."""
    run_case("bf16", M_rows, d, V, K, with_w1, 400 + M_rows % 100)
