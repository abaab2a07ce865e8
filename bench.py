#!/usr/bin/env python3
"""Benchmark of the Medusa verification step on one MI355X.

A step is one pass of the whole hot path (heads, top-k/tree, tree attention on one cache layer,
LM-head logits of the tree tokens, acceptance, KV commit of all layers) over one batch of seeded
synthetic inputs that are already resident in HBM.  Prints ONE JSON line with the step rate, the
roofline of the dominant kernel (the W2 vocabulary projection of medusa_heads, timed live with
HIP events inside the timed region) and the CPU oracle timed on the host cores as a baseline.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth

# HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE (two runs), each scaled by what the same counter reads for a plain 1 GiB copy
# (FETCH_SIZE counts 2 KiB units on this chip, WRITE_SIZE 1 KiB units).  bench.py cannot run the
# profiler itself; the figure is the recorded measurement for the workload it was taken on.
MEASURED_TRAFFIC_BYTES = {"C2": 512192 * 2 * 1024 + 505 * 1024, "C3": 512192 * 2 * 1024 + 505 * 1024}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="C2", help="workload name (C1..C5); the headline metric is quoted on C2")
    ap.add_argument("--event-every", type=int, default=8,
                    help="time the dominant kernel with a HIP event pair in every N-th timed step (a pair costs the "
                         "step about 5 us of dispatch gaps, so not every step carries one)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--breakdown", action="store_true", help="also time every library call on its own (stderr)")
    ap.add_argument("--block", action="store_true",
                    help="time the simplified decoder block of App. G on the tree tokens instead of the verification "
                         "step (its own JSON line; the headline metric stays the verification step)")
    ap.add_argument("--speed-model", action="store_true",
                    help="measure the simplified block at 1..112 candidate tokens and print the appendix's simulated "
                         "speedup for this GPU (its own JSON line)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run three plain 1 GiB device copies (reference kernel of known size for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


class HipEvents:
    """Raw hipEvent_t handles for the library's profiling hook (timed on whatever stream the hook records on)."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.pairs = []
        for _ in range(n):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(a)) == 0 and self.hip.hipEventCreate(ctypes.byref(b)) == 0
            self.pairs.append((a, b))

    def elapsed_ms(self, i):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.pairs[i][0], self.pairs[i][1])
        assert rc == 0, f"hipEventElapsedTime failed ({rc})"
        return ms.value

    def close(self):
        for a, b in self.pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(b)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2401_10774_amd as M
    from paper_2401_10774_amd.step import VerificationStep
    from workloads import get_config, make_step_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    cfg = get_config(args.config)
    torch.cuda.set_device(0)
    if args.block:
        bench_block(args, cfg)
        return
    if args.speed_model:
        bench_speed_model(args, cfg)
        return

    t0 = time.time()
    x = make_step_inputs(cfg)

    def dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
        return torch.from_numpy(a).cuda()

    tensors = {k: dev(v) for k, v in x.items()}
    tree = M.MedusaTree(branching=cfg.branching)
    step = VerificationStep(tensors, tree, cfg.accept, cfg.temperature, cfg.eps, cfg.delta)
    step.prepare()
    torch.cuda.synchronize()
    print(f"[bench] {cfg.name}: inputs drawn and uploaded in {time.time() - t0:.1f} s", file=sys.stderr, flush=True)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    L = M.lib()
    K, W = args.steps, args.warmup
    step.commit_out_of_place()   # every timed step sees the same prefix lengths; no reset between steps
    plant_accepted_paths(step, tensors, tree, cfg)
    for i in range(W):
        step.run(i % cfg.NL)
    torch.cuda.synchronize()

    every = max(1, args.event_every)
    timed = [i for i in range(K) if i % every == 0]
    events = HipEvents(len(timed))
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for i in range(K):
        if i % every == 0:
            L.medusa_profile_set_events(events.pairs[i // every][0], events.pairs[i // every][1])
        else:
            L.medusa_profile_set_events(None, None)
        step.run((W + i) % cfg.NL)
    stop.record()
    torch.cuda.synchronize()
    L.medusa_profile_set_events(None, None)
    ms_per_step = start.elapsed_time(stop) / K
    kern_ms = sum(events.elapsed_ms(j) for j in range(len(timed))) / len(timed)
    events.close()
    accept_len = step.accept_out[0].cpu().numpy()

    e = 2 if cfg.dtype == "bf16" else 4
    mean_prefix = float(np.mean(x["prefix_len"]))
    parts = step.algorithmic_bytes(mean_prefix, float(accept_len.mean()))
    steps_per_s = 1e3 / ms_per_step
    step_gbs = parts["total"] / (ms_per_step * 1e-3) / 1e9
    # dominant kernel: the W2 stream of medusa_heads (M = B rows): weights once + activations + fp32 logits
    dom_bytes = parts["heads_w2"]
    dom_gbs = dom_bytes / (kern_ms * 1e-3) / 1e9

    out = {
        "metric": "verification steps/sec + achieved HBM GB/s vs peak, 7B shapes, 64-node tree",
        "value": round(steps_per_s, 2),
        "unit": "steps/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {
            "workload": f"{cfg.name}: B={cfg.B} d={cfg.d} heads={cfg.Hq}/{cfg.Hkv}x{cfg.D} V={cfg.V} K={cfg.K} "
                        f"tree={cfg.branching} T={cfg.T} prefix=[{cfg.L_min},{cfg.L_max}] NL={cfg.NL} "
                        f"accept={cfg.accept}",
            "seed": cfg.seed,
            "launch": "eager, one stream, attended cache layer rotates every step",
        },
        "step_hbm": {"algorithmic_bytes": int(parts["total"]), "achieved_GBps": round(step_gbs, 1),
                     "frac_of_peak": round(step_gbs / HBM_PEAK_GBS, 4)},
        "roofline": {
            "kernel": "gemv_bf16_kernel<1, EPI_LOGITS> (medusa_heads W2 projection, M=B)" if cfg.dtype == "bf16" and cfg.B <= 4
                      else "medusa_heads W2 projection",
            "bound": "hbm",
            "achieved": round(dom_gbs, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(dom_gbs / HBM_PEAK_GBS, 4),
            "bytes_per_launch": int(dom_bytes),
            "avg_launch_us": round(kern_ms * 1e3, 2),
            "launches_timed": len(timed),
            "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name),
        },
        "mean_accept_len": round(float(accept_len.mean()), 3),
    }

    if args.breakdown:
        breakdown(step, cfg, parts)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, x)
    print(json.dumps(out), flush=True)


def plant_accepted_paths(step, tensors, tree, cfg):
    """Input preparation, before any timing.  Random hidden states accept nothing beyond the root,
    which would leave acceptance and kv_commit their minimum work.  The paper's steps emit about
    three tokens (Sec. 3; 0.477 log2(64) = 2.86 in the appendix's model), so per sequence one tree
    path of 1..3 nodes below the root (two at batch 1; seeded) is made acceptable: the hidden
    state of each node on it is replaced by 40x the LM-head row of the path's next token, whose
    logit (about 65) then towers over the rest (about N(0, 1)).  The row norm (about 51) stays close
    to that of the random rows (64).  The tree tokens come from one untimed step on these inputs."""
    import numpy as np
    import torch

    step.run(0)
    torch.cuda.synchronize()
    tok = step.tree_tokens.view(cfg.B, tree.T).cpu().numpy()
    rng = np.random.default_rng(cfg.seed)
    rows, toks = [], []
    for b in range(cfg.B):
        dep = 2 if cfg.B == 1 else int(rng.integers(1, min(3, tree.K) + 1))
        at_depth = np.flatnonzero(tree.depth == dep)
        n = int(at_depth[rng.integers(len(at_depth))])
        while n > 0:
            rows.append(b * tree.T + int(tree.parent[n]))
            toks.append(int(tok[b, n]))
            n = int(tree.parent[n])
    hidden = tensors["hidden_tree"].view(cfg.B * tree.T, cfg.d)
    w = tensors["w_lm"][torch.tensor(toks, device="cuda")].float() * 40.0
    hidden[torch.tensor(rows, device="cuda")] = w.to(hidden.dtype)
    torch.cuda.synchronize()


def bench_block(args, cfg):
    """One step = one simplified decoder block (X W_Q, X W_K, X W_V, rotary embedding, tree attention,
    X W_u, X W_g, X W_d) on the B*T tree tokens of the named workload's shapes; weights and cache of
    the layer rotate over several distinct sets so that every step streams them from HBM."""
    import torch

    import paper_2401_10774_amd as M
    from paper_2401_10774_amd.block import SimplifiedBlock

    inter = {4096: 11008, 5120: 13824}.get(cfg.d, ((cfg.d * 8 // 3 + 255) // 256) * 256)      # Llama-family widths
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    es = 2 if cfg.dtype == "bf16" else 4
    tree = M.MedusaTree(branching=cfg.branching)
    B, T, h, Hq, Hkv, D = cfg.B, tree.T, cfg.d, cfg.Hq, cfg.Hkv, cfg.D
    gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
    layer_bytes = (Hq * D * h + 2 * Hkv * D * h + 2 * inter * Hq * D + h * inter) * es + 2 * B * Hkv * cfg.Lcap * D * es
    n_sets = max(2, min(16, int(3e9 // layer_bytes)))
    rnd = lambda *shape, std=1.0: (torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32) * std).to(dt)
    sets = []
    for _ in range(n_sets):
        wqkv = rnd((Hq + 2 * Hkv) * D, h, std=h ** -0.5)     # one allocation: the block fuses the three projections at B = 1
        sets.append(dict(wq=wqkv[:Hq * D], wk=wqkv[Hq * D:(Hq + Hkv) * D], wv=wqkv[(Hq + Hkv) * D:],
                         wu=rnd(inter, Hq * D, std=h ** -0.5), wg=rnd(inter, Hq * D, std=h ** -0.5),
                         wd=rnd(h, inter, std=inter ** -0.5), kc=rnd(B, Hkv, cfg.Lcap, D), vc=rnd(B, Hkv, cfg.Lcap, D)))
        # bf16: gate and up in one call over interleaved weights (the separate matrices are then not read)
        sets[-1]["wgu"] = M.interleave_gate_up(sets[-1]["wg"], sets[-1]["wu"]) if dt == torch.bfloat16 else None
    x = rnd(B * T, h)
    pl = torch.randint(cfg.L_min, cfg.L_max + 1, (B,), generator=gen, device="cuda", dtype=torch.int32)
    depth = torch.from_numpy(tree.depth).to(device="cuda", dtype=torch.int32)
    pos = (pl[:, None] + depth[None, :]).to(torch.int32).contiguous()
    blk = SimplifiedBlock(tree, B, h, Hq, Hkv, D, inter, cfg.Lcap, dt)
    scale = 1.0 / math.sqrt(D)

    def run(i):
        w = sets[i % n_sets]
        blk.run(x, w["wq"], w["wk"], w["wv"], w["wu"], w["wg"], w["wd"], w["kc"], w["vc"], pl, pos, scale, w["wgu"])

    K, W = args.steps, args.warmup
    for i in range(W):
        run(i)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for i in range(K):
        run(i)
    stop.record()
    torch.cuda.synchronize()
    ms = start.elapsed_time(stop) / K
    mean_L = float(pl.float().mean())
    M_rows = B * T
    fused_gate_up = any(c[0] == "tree_linear_swiglu" for c in next(iter(blk._plans.values())))
    w_bytes = (Hq * D * h + 2 * Hkv * D * h + 2 * inter * Hq * D + h * inter) * es
    act_bytes = (3 * M_rows * h + 2 * M_rows * (Hq + 2 * Hkv) * D + 2 * M_rows * Hq * D + 3 * M_rows * Hq * D
                 + (2 if fused_gate_up else 4) * M_rows * inter + M_rows * h) * es   # (fused gate/up: no `up` round trip)
    kv_bytes = int(2 * B * Hkv * mean_L * D * es)
    total = w_bytes + act_bytes + kv_bytes
    flops = 2.0 * M_rows * (Hq * D * h + 2 * Hkv * D * h + 2 * inter * Hq * D + h * inter) + 4.0 * B * Hq * T * (mean_L + T) * D
    if args.breakdown:
        stream = torch.cuda.current_stream().cuda_stream
        plans = [blk._calls(x, w["wq"], w["wk"], w["wv"], w["wu"], w["wg"], w["wd"], w["kc"], w["vc"], pl, pos, scale, w["wgu"])
                 for w in sets]
        names = [{"tree_rope": "rotary", "tree_attention": "QK^T, PV", "tree_linear_swiglu": "X W_u, W_g"}.get(c[0], c[0])
                 for c in plans[0]]
        n_proj = names.index("rotary")                 # projection calls in front of the rotary embedding: 1, 2 or 3
        lin_names = {1: ["X W_QKV"], 2: ["X W_Q", "X W_KV"], 3: ["X W_Q", "X W_K", "X W_V"]}[n_proj] + (
            ["X W_d"] if "X W_u, W_g" in names else ["X W_u", "X W_g", "X W_d"])
        names = [lin_names.pop(0) if nm in ("tree_linear", "tree_linear_segments") else nm for nm in names]
        for j, name in enumerate(names):
            for i in range(5):
                _, fn, a = plans[i % n_sets][j]
                fn(*a, stream)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(56):
                _, fn, a = plans[i % n_sets][j]
                fn(*a, stream)
            e1.record()
            torch.cuda.synchronize()
            print(f"[bench]   {name:10s} {e0.elapsed_time(e1) / 56 * 1e3:8.1f} us", file=sys.stderr, flush=True)
    print(json.dumps({
        "metric": "simplified decoder block (App. G) on the tree tokens", "value": round(1e3 / ms, 2), "unit": "blocks/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name} shapes: B={B} T={T} h={h} inter={inter} heads={Hq}/{Hkv}x{D} prefix=[{cfg.L_min},{cfg.L_max}]",
                   "weight_sets_rotated": n_sets},
        "block_hbm": {"algorithmic_bytes": total, "achieved_GBps": round(total / ms / 1e6, 1),
                      "frac_of_peak": round(total / ms / 1e6 / HBM_PEAK_GBS, 4)},
        "block_flops": {"useful_TFLOPs": round(flops / ms / 1e9, 1)},
    }), flush=True)


def bench_speed_model(args, cfg):
    """The simulation of the appendix on hardware constraints with measured MI355X latencies: one
    simplified block at q = 1, 16, ..., 112 candidate tokens (q = 1 is plain decoding), speedup(q) =
    0.477 log2(q) * latency(1) / latency(q); batch and prefix length sweeps as in the appendix's
    three experiments.  Trees: the greedy sparse tree of q - 1 nodes on the synthetic accuracy table."""
    import torch

    import paper_2401_10774_amd as M
    from paper_2401_10774_amd import speed_model as S
    from paper_2401_10774_amd.block import SimplifiedBlock
    from workloads import synthetic_accuracy_table

    h, Hq, Hkv, D = cfg.d, cfg.Hq, cfg.Hkv, cfg.D
    inter = {4096: 11008, 5120: 13824}.get(h, ((h * 8 // 3 + 255) // 256) * 256)
    shape = S.BlockShape(h=h, inter=inter, n_heads=Hq, n_kv_heads=Hkv, d=D)
    dt = torch.bfloat16
    gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
    rnd = lambda *shp, std=1.0: (torch.randn(shp, generator=gen, device="cuda", dtype=torch.float32) * std).to(dt)
    n_sets = 6
    qkv = [rnd((Hq + 2 * Hkv) * D, h, std=h ** -0.5) for _ in range(n_sets)]      # one allocation per set (fused at batch 1)
    wsets = [dict(wq=qkv[i][:Hq * D], wk=qkv[i][Hq * D:(Hq + Hkv) * D], wv=qkv[i][(Hq + Hkv) * D:],
                  wu=rnd(inter, Hq * D, std=h ** -0.5), wg=rnd(inter, Hq * D, std=h ** -0.5), wd=rnd(h, inter, std=inter ** -0.5))
             for i in range(n_sets)]
    for w in wsets:
        w["wgu"] = M.interleave_gate_up(w["wg"], w["wu"])
    qs = [1, 16, 32, 48, 64, 80, 96, 112]
    acc = synthetic_accuracy_table(5, 10)
    trees = {q: (M.MedusaTree(nodes=[]) if q == 1 else M.MedusaTree(accuracy=acc, n_nodes=q - 1)) for q in qs}
    scale = 1.0 / math.sqrt(D)
    experiments = [("batch 1, prefix 1024", 1, 1024), ("batch 4, prefix 1024", 4, 1024), ("batch 16, prefix 1024", 16, 1024),
                   ("batch 32, prefix 1024", 32, 1024), ("batch 4, prefix 4096", 4, 4096)]
    results = {}
    for label, B, s_len in experiments:
        Lcap = s_len + 128
        caches = [(rnd(B, Hkv, Lcap, D), rnd(B, Hkv, Lcap, D)) for _ in range(max(2, min(n_sets, int(1.5e9 // (4 * B * Hkv * Lcap * D)))))]
        pl = torch.full((B,), s_len, dtype=torch.int32, device="cuda")
        lat = {}
        for q in qs:
            tree = trees[q]
            T = tree.T
            blk = SimplifiedBlock(tree, B, h, Hq, Hkv, D, inter, Lcap, dt)
            x = rnd(B * T, h)
            pos = (pl[:, None] + torch.from_numpy(tree.depth).to(device="cuda", dtype=torch.int32)[None, :]).to(torch.int32).contiguous()

            def run(i):
                w = wsets[i % n_sets]
                kc, vc = caches[i % len(caches)]
                blk.run(x, w["wq"], w["wk"], w["wv"], w["wu"], w["wg"], w["wd"], kc, vc, pl, pos, scale,
                        w["wgu"] if B * T > 4 else None)      # (plain decoding keeps the wave-per-row kernels; the block itself decides where the fused pass pays)

            for i in range(12):
                run(i)
            torch.cuda.synchronize()
            # three timed groups of 20 blocks, the median group counts (a stray stall of the box,
            # seen once as a 4x outlier of one point, would otherwise bend the curve)
            groups = []
            for g in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(20):
                    run(20 * g + i)
                e1.record()
                torch.cuda.synchronize()
                groups.append(e0.elapsed_time(e1) / 20 * 1e-3)
            lat[q] = sorted(groups)[1]
            del blk
        rows = S.simulate_speedup(lambda q: lat[q], qs)
        roof = S.simulate_speedup(lambda q: S.roofline_latency(shape, B, q, s_len, 2.5e15, 8e12), qs)
        results[label] = {"best_candidates": S.best_candidates(rows), "best_speedup": round(max(r["speedup"] for r in rows), 3),
                          "latency_us": {str(q): round(lat[q] * 1e6, 1) for q in qs},
                          "speedup": {str(r["candidates"]): round(r["speedup"], 3) for r in rows},
                          "roofline_best_candidates": S.best_candidates(roof)}
        print(f"[bench] {label}:", file=sys.stderr)
        for r, rr in zip(rows, roof):
            print(f"[bench]   q={r['candidates']:4d}  block {r['latency'] * 1e6:8.1f} us  x{r['normalized_latency']:5.2f}  "
                  f"acc_rate {r['acc_rate']:5.2f}  speedup {r['speedup']:5.2f}   (roofline-only speedup {rr['speedup']:5.2f})",
                  file=sys.stderr, flush=True)
        del caches
    print(json.dumps({
        "metric": "simulated Medusa speedup of the simplified decoder block (appendix model, measured latencies)",
        "value": results[experiments[0][0]]["best_speedup"], "unit": "x vs. one token per block", "n_gpus": 1, "steps": 60, "warmup": 12,
        "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name} block shapes h={h} inter={inter} heads={Hq}/{Hkv}x{D}; candidates {qs}"},
        "experiments": results}), flush=True)


def breakdown(step, cfg, parts):
    """Per-call timings (each call 50x back to back, attended layer rotating); informational, stderr only."""
    import torch
    pre, post = step._calls(0)
    names = ["heads (W1+W2)", "topk_tree", "attention", "verify GEMM", "accept", "commit"]
    keys = [("heads_w1", "heads_w2"), ("topk",), ("attention",), ("verify",), ("accept",), ("commit",)]
    stream = torch.cuda.current_stream().cuda_stream
    n = 50
    for idx, name in enumerate(names):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for i in range(n):
            calls = step._calls(i % cfg.NL)
            _, fn, fargs = (calls[0] + calls[1])[idx]
            fn(*fargs, stream)
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) / n * 1e3
        nbytes = sum(parts[k] for k in keys[idx])
        print(f"[bench]   {name:14s} {us:9.1f} us  {nbytes / 1e6:9.1f} MB  {nbytes / us / 1e3:8.1f} GB/s", file=sys.stderr)


def cpu_baseline(cfg, x):
    """The CPU oracle, as it stands, on one full step of the same inputs (host cores of this machine)."""
    from oracle import medusa_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    otree = O.tree_cartesian(cfg.branching)
    pl0 = x["prefix_len"].copy()
    n, t0 = 0, time.time()
    while True:                                  # whole steps until about 10 s of CPU work are on the clock
        x["prefix_len"][:] = pl0
        O.verification_step_ref(x, otree, cfg.dtype, 1.0 / math.sqrt(cfg.D), cfg.accept, cfg.temperature, cfg.eps,
                                cfg.delta)
        n += 1
        dt = time.time() - t0
        if dt >= 10.0 or n >= 50:
            break
    return {"value": round(n / dt, 4), "unit": "steps/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{n} full step(s) of {cfg.name} (all heads, all tree rows, all {cfg.NL} committed layers), "
                      f"{dt:.1f} s wall, numpy float64"}


if __name__ == "__main__":
    main()
