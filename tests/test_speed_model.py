"""The analytical model of the appendix on hardware constraints against what the paper prints:
every operational-intensity cell of its three operator tables, the fitted acceleration rate, and the
qualitative claims of its simulation (closed-form latencies stand in for a machine)."""
import math
import os
import re

import pytest

from paper_2401_10774_amd import speed_model as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "operational_intensity.txt")


def golden_rows():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        kind, params, value = (x.strip() for x in line.split("|"))
        rows.append((kind, {k: int(v) for k, v in re.findall(r"(\w+)=(\d+)", params)}, float(value)))
    return rows


def test_every_printed_operational_intensity_cell():
    rows = golden_rows()
    assert len(rows) == 3 * 7 * 8
    for kind, p, printed in rows:
        got = S.attention_intensity(p["q"], p["s"], p["d"]) if kind == "attention" else S.linear_intensity(p["m"], p["h"], p["i"])
        # cells are printed with two decimals (a few with one or none)
        assert abs(got - printed) <= 0.0051 + 1e-12 or abs(round(got, 1) - printed) < 1e-9 or abs(round(got) - printed) < 1e-9, (kind, p, got, printed)


def test_intensity_limits():
    # decoding (q = 1) moves about one byte per flop; many candidates approach the head dimension
    assert abs(S.attention_intensity(1, 10 ** 6, 128) - 1.0) < 0.01
    assert S.attention_intensity(10 ** 6, 10 ** 6, 128) > 127.0
    # a linear layer with one row is a matrix-vector product: one flop per weight byte
    assert abs(S.linear_intensity(1, 4096, 11008) - 1.0) < 1e-3
    assert S.linear_intensity(64, 6656, 17920) < 64


def test_acceleration_rate_fit():
    assert abs(S.acceleration_rate(64) - 0.477 * 6) < 1e-12          # 2.86 tokens per step at 64 candidates
    assert S.acceleration_rate(1) == 0.0
    assert S.acceleration_rate(16) < S.acceleration_rate(32) < S.acceleration_rate(64)


def test_speedup_definition_closed_forms():
    qs = [1, 16, 32, 64, 128]
    flat = S.simulate_speedup(lambda q: 1.0, qs)                     # free candidates: speedup = acceleration rate
    assert all(abs(r["speedup"] - S.acceleration_rate(r["candidates"])) < 1e-12 for r in flat)
    assert S.best_candidates(flat) == 128
    linear = S.simulate_speedup(lambda q: float(q), qs)              # latency proportional to q: log2(q)/q decreases
    assert S.best_candidates(linear) == 16
    # latency = 1 + q/64: log2(q) / (1 + q/64) is 3.2, 3.33, 3.19, 3.0 at q = 16, 32, 48, 64: an interior optimum
    knee = S.simulate_speedup(lambda q: 1.0 + q / 64.0, [1, 16, 32, 48, 64, 80, 96, 112, 256, 1024])
    assert S.best_candidates(knee) == 32
    assert abs(knee[2]["speedup"] - 0.477 * 5.0 * (65 / 64) / 1.5) < 1e-12 and abs(knee[2]["normalized_latency"] - 1.5 / (65 / 64)) < 1e-12


def test_roofline_latency_regimes():
    # one token, batch 1: every operator is memory-bound, latency = bytes / bandwidth
    shp = S.LLAMA_7B
    ops = shp.operators(1, 1, 1024)
    lat = S.roofline_latency(shp, 1, 1, 1024, 312e12, 1935e9)
    assert abs(lat - sum(o["bytes"] for o in ops.values()) / 1935e9) < 1e-12
    # many rows: compute-bound, latency = flops / peak
    lat = S.roofline_latency(shp, 64, 112, 1024, 312e12, 1935e9)
    ops = shp.operators(64, 112, 1024)
    assert lat >= sum(o["flops"] for o in ops.values()) / 312e12 - 1e-12
    # the appendix's third claim: at a fixed candidate count longer sequences cost more (attention only)
    assert S.roofline_latency(shp, 4, 64, 8192, 312e12, 1935e9) > S.roofline_latency(shp, 4, 64, 1024, 312e12, 1935e9)
    # weights of the seven linear operators of Llama-7B: 2 bytes each, read once
    w = 2 * (3 * 4096 * 4096 + 3 * 4096 * 11008)
    assert abs(sum(o["bytes"] for n, o in shp.operators(1, 1, 0).items() if n != "QK^T, PV") - w) < 1e6
