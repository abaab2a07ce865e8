"""The GEMM planning must not have cliffs: on a fixed weight matrix, a projection of fewer tree rows
never takes much longer than one of more rows (Sec. 2.1.1 / App. G operator table: the same matrices serve
every batch size and tree size).  A wrong arrangement for some row count -- a kernel past its best range, a
split that does not pay, a tile that leaves the chip idle -- shows up as exactly that.  (A timing test: the file
name makes pytest collect it after the parity tests.)"""
import pytest
import torch

import paper_2401_10774_amd as M

pytestmark = pytest.mark.gpu

ROWS = [1, 2, 3, 4, 5, 16, 65, 80, 81, 128, 129, 160, 161, 192, 193, 256, 260, 356, 385, 512, 1040]
# 7B: LM head, Q/K/V, gate and up, down, output projection; 13B: down
# measured worst ratio on MI355X: 1.04; the limit leaves room for run-to-run placement effects (about 5 %)
LIMIT = 1.3
SHAPES = [(32000, 4096), (12288, 4096), (22016, 4096), (4096, 11008), (4096, 4096), (5120, 13824)]


def time_us(x, ws, rows, y):
    best = float("inf")
    for rep in range(3):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n = 16
        a.record()
        for i in range(n):
            M.tree_linear(x, ws[i % len(ws)], 1, rows, y=y)
        b.record()
        torch.cuda.synchronize()
        best = min(best, a.elapsed_time(b) / n * 1e3)
    return best


@pytest.mark.parametrize("N,d", SHAPES)
def test_no_cliffs_over_row_counts(N, d):
    g = torch.Generator(device="cuda").manual_seed(N + d)
    copies = max(2, min(8, int(6e8 // (N * d * 2))))            # weights come from HBM, as between two decoding steps
    ws = [(torch.randn(N, d, device="cuda", generator=g) * 0.02).bfloat16() for _ in range(copies)]
    times, inputs = [], []
    for rows in ROWS:
        x = torch.randn(rows, d, device="cuda", generator=g).bfloat16()
        y = M.tree_linear(x, ws[0], 1, rows)
        for i in range(3):
            M.tree_linear(x, ws[i % copies], 1, rows, y=y)
        torch.cuda.synchronize()
        inputs.append((x, y))
        times.append(time_us(x, ws, rows, y))

    def worst_pair():
        return max((times[i] / (times[j] + 2.0), i, j) for i in range(len(ROWS)) for j in range(i + 1, len(ROWS)))

    ratio, i, j = worst_pair()
    for attempt in range(2):                    # a pair over the line is timed again before it counts (a hiccup of the box is not a cliff)
        if ratio <= LIMIT:
            break
        for k in (i, j):
            times[k] = min(times[k], time_us(inputs[k][0], ws, ROWS[k], inputs[k][1]))
        ratio, i, j = worst_pair()
    print(f"N={N} d={d}: " + " ".join(f"{r}:{t:.0f}" for r, t in zip(ROWS, times)) + f"  worst ratio {ratio:.2f} ({ROWS[i]} vs {ROWS[j]} rows)")
    assert ratio <= LIMIT, f"{ROWS[i]} rows take {ratio:.2f}x as long as {ROWS[j]} rows: " + str(dict(zip(ROWS, [round(t, 1) for t in times])))
