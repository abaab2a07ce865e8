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

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "heads_w2_hbm_traffic.md")


def measured_traffic(workload):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc (FETCH_SIZE and
    WRITE_SIZE in two runs, each scaled by what the same counter reads for a plain 1 GiB copy), read
    from the tracked summary of those runs: lines `traffic_bytes <workload> <bytes> commit <hash>`.
    bench.py cannot run the profiler itself; None when the summary has no line for the workload."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                w = line.split()
                if len(w) >= 5 and w[0] == "traffic_bytes" and w[1] == workload and w[3] == "commit":
                    return {"bytes": int(w[2]), "commit": w[4]}
    except OSError:
        pass
    return None


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
    ap.add_argument("--breakdown", action="store_true", help="also print the per-call timings of the JSON line to stderr")
    ap.add_argument("--block", action="store_true",
                    help="time the simplified decoder block of App. G on the tree tokens instead of the verification "
                         "step (its own JSON line; the headline metric stays the verification step)")
    ap.add_argument("--forward", action="store_true",
                    help="time the whole verification pass with a stack of --layers simplified decoder blocks in place "
                         "of the single attention call (heads -> top-k/tree -> blocks -> LM head -> acceptance -> commit)")
    ap.add_argument("--layers", type=int, default=0, help="--forward: decoder blocks in the stack (default: the workload's layer count)")
    ap.add_argument("--batch", type=int, default=0, help="sequences in the batch instead of the workload's (C4 with --batch 1: the 13B shapes on one 89-token tree)")
    ap.add_argument("--speed-model", action="store_true",
                    help="measure the simplified block at 1..112 candidate tokens and print the appendix's simulated "
                         "speedup for this GPU (its own JSON line)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run three plain 1 GiB device copies (reference kernel of known size for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


class HipEvents:
    """Raw hipEvent_t handles for the library's timed entry (recorded on the stream the call is given)."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.handles = []
        for _ in range(n):
            a = ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(a)) == 0
            self.handles.append(a)

    def elapsed_ms(self, i, j):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.handles[i], self.handles[j])
        assert rc == 0, f"hipEventElapsedTime failed ({rc})"
        return ms.value

    def close(self):
        for a in self.handles:
            self.hip.hipEventDestroy(a)


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
    if args.batch > 0:
        import dataclasses
        cfg = dataclasses.replace(cfg, B=args.batch)
    if args.block:
        bench_block(args, cfg)
        return
    if args.speed_model:
        bench_speed_model(args, cfg)
        return
    if args.forward:
        bench_forward(args, cfg)
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

    K, W = args.steps, args.warmup
    step.commit_out_of_place()   # every timed step sees the same prefix lengths; no reset between steps
    plant_accepted_paths(step, tensors, tree, cfg)
    # Between two verification steps a decoder streams its whole backbone, so nothing of this step's
    # weights is left in the 256 MB last-level cache.  The timed loop reproduces that: the W1 stack and
    # the LM head rotate over copies (W2, 1 GB, and the KV layers, which rotate too, evict themselves).
    w1_bytes = tensors["w1"].numel() * tensors["w1"].element_size()
    lm_bytes = tensors["w_lm"].numel() * tensors["w_lm"].element_size()
    n_w1 = max(2, min(4, int(math.ceil(600e6 / w1_bytes))))
    n_lm = max(2, min(4, int(math.ceil(700e6 / lm_bytes))))
    step.add_weight_copies(n_w1, n_lm)
    every = max(1, args.event_every)

    def timed_loop(cold):
        for i in range(W):
            step.run(i % cfg.NL, wset=i if cold else 0)
        timed = [i for i in range(K) if i % every == 0]
        events = HipEvents(3 * len(timed))
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        start.record()
        for i in range(K):
            ev = events.handles[3 * (i // every):3 * (i // every) + 3] if i % every == 0 else None
            step.run((W + i) % cfg.NL, wset=(W + i) if cold else 0, heads_events=ev)
        stop.record()
        torch.cuda.synchronize()
        ms = start.elapsed_time(stop) / K
        w1_ms = sum(events.elapsed_ms(3 * j, 3 * j + 1) for j in range(len(timed))) / len(timed)
        w2_ms = sum(events.elapsed_ms(3 * j + 1, 3 * j + 2) for j in range(len(timed))) / len(timed)
        events.close()
        return ms, w1_ms, w2_ms, len(timed)

    ms_per_step, w1_ms, kern_ms, n_timed = timed_loop(cold=True)
    accept_len = step.accept_out[0].cpu().numpy()
    warm_ms, _, _, _ = timed_loop(cold=False)

    mean_prefix = float(np.mean(x["prefix_len"]))
    parts = step.algorithmic_bytes(mean_prefix, float(accept_len.mean()))
    steps_per_s = 1e3 / ms_per_step
    step_gbs = parts["total"] / (ms_per_step * 1e-3) / 1e9
    warm_gbs = parts["total"] / (warm_ms * 1e-3) / 1e9
    # dominant kernel: the W2 stream of medusa_heads (M = B rows): weights once + activations + fp32 logits
    dom_bytes = parts["heads_w2"]
    dom_gbs = dom_bytes / (kern_ms * 1e-3) / 1e9
    kernels = per_call_timings(step, cfg, parts, w1_ms, kern_ms)
    traffic = None if args.batch > 0 else measured_traffic(cfg.name)      # (the profiled figure belongs to the workload's own batch size)

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
                        f"accept={cfg.accept}, accepted paths planted in the hidden states",
            "planted": True,
            "seed": cfg.seed,
            "launch": f"eager, one stream; every step streams its weights from HBM: attended cache layer, W1 ({n_w1} "
                      f"copies) and LM head ({n_lm} copies) rotate every step",
        },
        "step_hbm": {"algorithmic_bytes": int(parts["total"]), "achieved_GBps": round(step_gbs, 1),
                     "frac_of_peak": round(step_gbs / HBM_PEAK_GBS, 4),
                     "cold_lm_head": {"steps_per_s": round(steps_per_s, 2), "frac_of_peak": round(step_gbs / HBM_PEAK_GBS, 4),
                                      "note": "the headline: W1 and LM head rotate over copies, nothing is cache-resident"},
                     "warm_lm_head": {"steps_per_s": round(1e3 / warm_ms, 2), "frac_of_peak": round(warm_gbs / HBM_PEAK_GBS, 4),
                                      "note": "same step with one copy of W1 and of the LM head re-read every step "
                                              "(they stay in the last-level cache); not what a decoder sees"}},
        "roofline": {
            "kernel": ("gemv_bf16_kernel<%d, EPI_LOGITS>" % cfg.B if cfg.dtype == "bf16" and cfg.B <= 2
                       else "gemm_ring_bf16_kernel<1, 8, 8, EPI_LOGITS>" if cfg.dtype == "bf16" and cfg.B <= 16
                       else "medusa_heads W2 kernel") + " (medusa_heads W2 projection, M=B)",
            "bound": "hbm",
            "achieved": round(dom_gbs, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(dom_gbs / HBM_PEAK_GBS, 4),
            "bytes_per_launch": int(dom_bytes),
            "avg_launch_us": round(kern_ms * 1e3, 2),
            "launches_timed": n_timed,
            "traffic": None if traffic is None else traffic["bytes"],
            "traffic_measured_at_commit": None if traffic is None else traffic["commit"],
        },
        "kernels": kernels,
        "kernels_note": "call durations between two events on the stream, in instrumented steps after the timed region (W1, W2: "
                        "inside it); an event pair adds about 2 us to a call -- the profiler's kernel durations are in "
                        "profiles/bench_kernel_traces.md",
        "mean_accept_len": round(float(accept_len.mean()), 3),
    }

    if args.breakdown:
        for name, k in kernels.items():
            print(f"[bench]   {name:16s} {k['us']:9.1f} us  {k['MB']:9.1f} MB  {k['GBps']:8.1f} GB/s", file=sys.stderr)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, x)
    print(json.dumps(out), flush=True)


def per_call_timings(step, cfg, parts, w1_ms, w2_ms, n=48):
    """Every library call of the step timed with an event pair around it, in steps of their own
    after the timed region (a pair costs the step several microseconds of dispatch gaps), with the
    same rotation of layers and weight copies; the two kernels of the heads call keep the figures
    measured inside the timed region.  us = average duration of the call on the stream (a call is
    one kernel, except attention: split kernel + merge); MB = its algorithmic bytes."""
    import torch
    stream = torch.cuda.current_stream().cuda_stream
    names = ["heads", "topk_tree", "attention", "verify_lm_head", "accept", "commit"]   # (verify + accept may be the fused pair)
    pairs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in names] for _ in range(n)]
    for i in range(n):
        pre, post = step._calls(i % cfg.NL, i)
        for j, (name, fn, fargs) in enumerate(pre + post):
            pairs[i][j][0].record()
            rc = fn(*fargs, stream)
            pairs[i][j][1].record()
            assert rc == 0, (name, rc)
    torch.cuda.synchronize()
    us = {nm: sum(p[j][0].elapsed_time(p[j][1]) for p in pairs[8:]) / (n - 8) * 1e3 for j, nm in enumerate(names)}
    keys = {"topk_tree": ("topk",), "attention": ("attention",), "verify_lm_head": ("verify",), "accept": ("accept",),
            "commit": ("commit",)}
    out = {}

    def entry(t_us, nbytes):
        return {"us": round(t_us, 2), "MB": round(nbytes / 1e6, 2), "GBps": round(nbytes / t_us / 1e3, 1),
                "frac_of_hbm_peak": round(nbytes / t_us / 1e3 / HBM_PEAK_GBS, 4)}

    out["heads_w1"] = entry(w1_ms * 1e3, parts["heads_w1"])
    out["heads_w2"] = entry(w2_ms * 1e3, parts["heads_w2"])
    for nm in names[1:]:
        out[nm] = entry(us[nm], sum(parts[k] for k in keys[nm]))
    flops = 2.0 * cfg.B * cfg.T * cfg.d * cfg.V
    out["verify_lm_head"]["useful_TFLOPs"] = round(flops / us["verify_lm_head"] / 1e6, 1)
    out["verify_lm_head"]["frac_of_bf16_mfma_peak"] = round(flops / us["verify_lm_head"] / 1e6 / 2500.0, 4)
    out["heads_w1"]["note"] = out["heads_w2"]["note"] = "timed inside the timed region (medusa_heads_timed)"
    return out


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


def bench_forward(args, cfg):
    """One step = one whole verification pass of a backbone-shaped stack: medusa_heads, top-k and tree,
    NL simplified decoder blocks on the tree tokens (each streaming its own weights, attending its own
    cache layer and leaving the tree tokens' K and V for the commit), the LM head on the last block's
    output, acceptance, and the commit of all NL layers.  Synthetic weights; no embedding, norms or
    residual stream (out of scope), so the accept lengths are those of random logits."""
    import numpy as np
    import torch

    import paper_2401_10774_amd as M
    from paper_2401_10774_amd.forward import TreeBackbone, alloc_qkv
    from paper_2401_10774_amd.step import VerificationStep
    from workloads import make_step_inputs, scaled_config

    NL = args.layers or cfg.NL
    if NL != cfg.NL:
        cfg = scaled_config(cfg.name, NL=NL)
    inter = {4096: 11008, 5120: 13824}.get(cfg.d, ((cfg.d * 8 // 3 + 255) // 256) * 256)
    dt, es = torch.bfloat16, 2
    if cfg.dtype != "bf16":
        print("bench.py --forward: bf16 workloads only", file=sys.stderr)
        sys.exit(2)
    tree = M.MedusaTree(branching=cfg.branching)
    B, T, h, Hq, Hkv, D, V = cfg.B, tree.T, cfg.d, cfg.Hq, cfg.Hkv, cfg.D, cfg.V
    x = make_step_inputs(cfg, names=[n for n in ("h_last", "hidden_tree", "w1", "w2", "w_lm", "k_cache", "v_cache", "prefix_len")])

    def dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
        return torch.from_numpy(a).cuda()

    tensors = {k: dev(v) for k, v in x.items()}
    q, k_tree, v_tree = alloc_qkv(NL, B, Hq, Hkv, T, D, dt)
    tensors["q"], tensors["k_tree"], tensors["v_tree"] = q[0], k_tree, v_tree
    step = VerificationStep(tensors, tree, cfg.accept, cfg.temperature, cfg.eps, cfg.delta)
    step.prepare()
    step.commit_out_of_place()
    gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
    rnd = lambda *shape, std=1.0: (torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32) * std).to(dt)
    weights = []
    for _ in range(NL):
        wg, wu = rnd(inter, Hq * D, std=(Hq * D) ** -0.5), rnd(inter, Hq * D, std=(Hq * D) ** -0.5)
        weights.append({"w_qkv": rnd((Hq + 2 * Hkv) * D, h, std=h ** -0.5), "w_gu": M.interleave_gate_up(wg, wu),
                        "wd": rnd(h, inter, std=inter ** -0.5)})
        if not (B * T <= 160 or M.medusa_gemm_plan(B * T, 2 * inter, Hq * D, 1, False)["kind"] == "big"):
            weights[-1]["wu"], weights[-1]["wg"] = wu, wg
        del wg, wu
    bb = TreeBackbone(tree, B, h, Hq, Hkv, D, inter, cfg.Lcap, weights, q, k_tree, v_tree, tensors["k_cache"], tensors["v_cache"],
                      tensors["prefix_len"], step.position_ids)
    x0 = rnd(B * T, h)
    hidden_rows = tensors["hidden_tree"].view(B * T, h)
    backbone = lambda: bb.run(x0, hidden_rows)
    K, W = args.steps, args.warmup
    for _ in range(W):
        step.run(backbone=backbone)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(K):
        step.run(backbone=backbone)
    stop.record()
    torch.cuda.synchronize()
    ms = start.elapsed_time(stop) / K
    accept_len = step.accept_out[0].cpu().numpy()
    finite = bool(torch.isfinite(step.verify_logits).all())
    mean_L = float(np.mean(x["prefix_len"]))
    M_rows = B * T
    layer_w = ((Hq + 2 * Hkv) * D * h + 2 * inter * Hq * D + h * inter) * es
    layer_act = (M_rows * h + M_rows * (Hq + 2 * Hkv) * D * 3 + M_rows * Hq * D * 2 + 2 * M_rows * inter + M_rows * h) * es
    layer_kv = int(2 * B * Hkv * mean_L * D * es)
    step_parts = step.algorithmic_bytes(mean_L, float(accept_len.mean()))
    total = NL * (layer_w + layer_act + layer_kv) + step_parts["total"] - step_parts["attention"]
    print(json.dumps({
        "metric": "verification passes/s of a backbone-shaped stack (heads, tree, NL simplified blocks, LM head, acceptance, commit)",
        "value": round(1e3 / ms, 2), "unit": "passes/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name} shapes, {NL} layers: B={B} T={T} h={h} inter={inter} heads={Hq}/{Hkv}x{D} V={V} "
                               f"prefix=[{cfg.L_min},{cfg.L_max}]",
                   "note": "every layer has its own weights (no rotation needed: the stack is larger than any cache); no "
                           "embedding, norms, output projection or residual stream"},
        "pass_hbm": {"algorithmic_bytes": int(total), "achieved_GBps": round(total / ms / 1e6, 1),
                     "frac_of_peak": round(total / ms / 1e6 / HBM_PEAK_GBS, 4)},
        "mean_accept_len": round(float(accept_len.mean()), 3), "logits_finite": finite,
        "tokens_per_s_at_accept_len": {"measured (random weights)": round(float(accept_len.mean()) * 1e3 / ms, 1),
                                       "3.0 (the paper's trained heads, for scale)": round(3.0 * 1e3 / ms, 1)},
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
                   ("batch 32, prefix 1024", 32, 1024), ("batch 64, prefix 1024", 64, 1024), ("batch 4, prefix 256", 4, 256), ("batch 4, prefix 4096", 4, 4096),
                   ("batch 4, prefix 8192", 4, 8192)]
    results = {}
    for label, B, s_len in experiments:
        Lcap = s_len + 128
        caches = [(rnd(B, Hkv, Lcap, D), rnd(B, Hkv, Lcap, D)) for _ in range(max(2, min(n_sets, int(1.5e9 // (4 * B * Hkv * Lcap * D)))))]
        pl = torch.full((B,), s_len, dtype=torch.int32, device="cuda")
        lat = {}
        qs_here = [q for q in qs if B * trees[q].T <= 16384]         # (the library takes up to 16384 tree tokens per call)
        for q in qs_here:
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
        rows = S.simulate_speedup(lambda q: lat[q], qs_here)
        roof = S.simulate_speedup(lambda q: S.roofline_latency(shape, B, q, s_len, 2.5e15, 8e12), qs_here)
        results[label] = {"best_candidates": S.best_candidates(rows), "best_speedup": round(max(r["speedup"] for r in rows), 3),
                          "latency_us": {str(q): round(lat[q] * 1e6, 1) for q in qs_here},
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


def cpu_baseline(cfg, x):
    """The CPU oracle, as it stands, on whole steps of the same inputs (host cores of this machine): at the
    thread count numpy's BLAS takes by itself, and limited to one thread."""
    from oracle import medusa_oracle as O
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threadpool_limits = None
        cores = os.cpu_count() or 1
    otree = O.tree_cartesian(cfg.branching)
    pl0 = x["prefix_len"].copy()

    def run(budget_s, max_steps):
        n, t0 = 0, time.time()
        while True:                              # whole steps until the budget of CPU work is on the clock
            x["prefix_len"][:] = pl0
            O.verification_step_ref(x, otree, cfg.dtype, 1.0 / math.sqrt(cfg.D), cfg.accept, cfg.temperature, cfg.eps,
                                    cfg.delta)
            n += 1
            dt = time.time() - t0
            if dt >= budget_s or n >= max_steps:
                return n, dt

    n, dt = run(10.0, 50)
    out = {"value": round(n / dt, 4), "unit": "steps/s", "cores": int(cores), "kind": "oracle",
           "sample": f"{n} full step(s) of {cfg.name} (all heads, all tree rows, all {cfg.NL} committed layers), "
                     f"{dt:.1f} s wall, numpy float64"}
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            n1, dt1 = run(8.0, 3)
        out["one_thread"] = {"value": round(n1 / dt1, 4), "unit": "steps/s", "cores": 1,
                             "sample": f"{n1} full step(s), {dt1:.1f} s wall"}
    return out


if __name__ == "__main__":
    main()
