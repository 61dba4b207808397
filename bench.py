#!/usr/bin/env python3
"""Benchmark of the placement-aware MoE layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config NAME]

A step is one call of prism_moe_layer (route -> dispatch -> grouped SwiGLU FFN
over the local experts -> combine) on one batch of seeded synthetic input that
is already resident in HBM.  Prints ONE JSON line: whole-job tokens/s, the
roofline fraction of the dominant kernel (timed with HIP events recorded by the
library around that kernel on the launch stream) and the CPU oracle timed on a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_BF16_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E peak
DEFAULT_CONFIG = "cfg2_mixtral_prefill"
DECODE_WEIGHT_COPIES = 4           # rotate weight copies so the 256 MB last-level cache cannot help


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def read_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch"):
            return float(line.split("=")[1])
    return None


def measured_ceilings(torch, P):
    """Second denominators measured on this very GPU: a pure bf16 MFMA loop (constant and
    random operand values: the sustained clock depends on them) and a streaming HBM read."""
    n_wg, iters = 1024, 4000
    out = torch.empty(n_wg * 256, dtype=torch.float32, device="cuda")
    res = {}
    gen = torch.Generator(device="cuda").manual_seed(7)
    for name, ops in (("mfma_bf16_constant_operands_tflops",
                       torch.full((n_wg * 256 * 16,), 1.5, dtype=torch.bfloat16, device="cuda")),
                      ("mfma_bf16_random_operands_tflops",
                       torch.randn(n_wg * 256 * 16, generator=gen, device="cuda").to(torch.bfloat16))):
        P.prism_ceiling_mfma_bf16(ops, out, n_wg, iters)          # warm-up
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flop = sum(P.prism_ceiling_mfma_bf16(ops, out, n_wg, iters) for _ in range(3))
        e1.record()
        torch.cuda.synchronize()
        res[name] = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    src = torch.zeros(4 << 30, dtype=torch.uint8, device="cuda")   # 16x the last-level cache
    n_rd = 32768
    sink = torch.empty(n_rd * 256 * 16, dtype=torch.uint8, device="cuda")
    P.prism_ceiling_hbm_read(src, sink, n_rd)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    nbytes = sum(P.prism_ceiling_hbm_read(src, sink, n_rd) for _ in range(5))
    e1.record()
    torch.cuda.synchronize()
    res["hbm_read_gbs"] = nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
    return res


def cpu_baseline(inp, n_sample: int):
    """Time the CPU oracle, as it stands, on the first n_sample tokens of the workload."""
    from oracle import prism_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    c = inp.cfg
    f = inp.f32
    n = min(n_sample, c.T)
    xs = f(inp.x)[:n]
    t0 = time.perf_counter()
    O.moe_layer(xs, f(inp.w_router), inp.bias, lambda e: tuple(f(w) for w in inp.expert(e)),
                [tuple(f(w) for w in inp.shared(s)) for s in range(c.S)], inp.mask, c.k, c.dtype,
                c.bias_group_tokens, np.arange(n))
    dt = time.perf_counter() - t0
    return {"value": n / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {n} of {c.T} tokens of {c.name}, whole layer, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", default=DEFAULT_CONFIG)
    ap.add_argument("--cpu-sample-tokens", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--trace-all", action="store_true", help="also time every stage (stderr)")
    ap.add_argument("--weight-layout", choices=("row_major", "tiled"), default="tiled",
                    help="expert weight layout in HBM; tiled (16 x 32 tiles) is packed once, outside the "
                         "timed region, as a server does when it loads or receives an expert")
    ap.add_argument("--mask", choices=("top", "random"), default="top",
                    help="hosted experts: the most popular ones (what the first loop of Alg. 2 hosts) or a "
                         "seeded uniformly random subset of the same size (the uniform baseline of Sec. IV)")
    ap.add_argument("--tokens", type=int, default=None,
                    help="another batch size for the chosen workload's layer (not the benchmark line: "
                         "config.workload then says so)")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the measured MFMA / HBM ceilings of this GPU")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1")
        sys.exit(2)

    import torch
    import paper_2508_12851_amd as P
    from prism_inputs import CONFIGS, make_config, make_inputs

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)
    cfg = CONFIGS[args.config]
    overrides = {}
    if args.mask == "random":
        overrides["mask_kind"] = "random"
    if args.tokens is not None:
        if args.tokens < 1:
            log("bench.py: --tokens must be at least 1")
            sys.exit(2)
        overrides["T"] = args.tokens
    if overrides:
        cfg = make_config(args.config, **overrides)
    workload = cfg.name if args.tokens is None else f"{cfg.name} layer with {cfg.T} tokens"
    # up to 512 tokens the dominant kernel streams the hosted weights once: HBM roofline
    decode = cfg.T <= (64 if args.tokens is None else 512)
    steps = args.steps if args.steps is not None else (200 if decode else 30)
    warmup = args.warmup if args.warmup is not None else (20 if decode else 5)

    t0 = time.perf_counter()
    inp = make_inputs(cfg, weights="local", threads=16)
    log(f"[bench] generated {cfg.name} inputs in {time.perf_counter() - t0:.1f} s")

    def dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
        return torch.from_numpy(a).cuda()

    desc = P.make_desc(cfg.H, cfg.F, cfg.E, cfg.k, cfg.S, cfg.dtype, cfg.bias_group_tokens,
                       weight_layout=args.weight_layout)
    wdev = (lambda a: P.prism_pack_weights(dev(a))) if args.weight_layout == "tiled" else dev
    experts = [tuple(wdev(w) for w in inp.expert(e)) if inp.mask[e] else None for e in range(cfg.E)]
    shared = [tuple(wdev(w) for w in inp.shared(s)) for s in range(cfg.S)]
    tables = [P.WeightTable(experts, shared)]
    if decode:
        for _ in range(DECODE_WEIGHT_COPIES - 1):
            ex = [None if t is None else tuple(w.clone() for w in t) for t in experts]
            sh = [tuple(w.clone() for w in t) for t in shared]
            tables.append(P.WeightTable(ex, sh))
    x, w_router, bias, mask = dev(inp.x), dev(inp.w_router), dev(inp.bias), dev(inp.mask)
    ws = P.alloc_workspace(desc, cfg.T)
    out = P.alloc_layer_out(desc, cfg.T)
    torch.cuda.synchronize()

    # one HIP event pair per timed step around the dominant kernel (gate/up grouped GEMM)
    n_st = len(P.STAGES)
    traced = range(n_st) if args.trace_all else (P.STAGES.index("ffn_up"),)
    events = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(n_st)] for _ in range(steps)]
    handle_arrays = []
    for step_ev in events:
        arr = (ctypes.c_void_p * (2 * n_st))()
        for s in traced:
            for j in (0, 1):
                step_ev[s][j].record()               # materialise the hipEvent_t
                arr[2 * s + j] = step_ev[s][j].cuda_event
        handle_arrays.append(arr)
    torch.cuda.synchronize()

    def step(i, ev=None):
        P.prism_moe_layer(desc, x, w_router, bias, tables[i % len(tables)], mask, ws, out,
                          stage_events=ev)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i, handle_arrays[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / steps
    tokens_per_s = cfg.T * steps / elapsed

    # per-step times from separate, individually bracketed calls (outside the timed region)
    n_ind = min(steps, 50)
    ind = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(n_ind)]
    for i, (e0, e1) in enumerate(ind):
        e0.record()
        step(i)
        e1.record()
    torch.cuda.synchronize()
    step_ms = sorted(e0.elapsed_time(e1) for e0, e1 in ind)

    stage_ms = {}
    for s in traced:
        stage_ms[P.STAGES[s]] = float(np.mean([events[i][s][0].elapsed_time(events[i][s][1])
                                               for i in range(steps)]))
    n_local, n_remote = out.n_local_remote.cpu().tolist()
    counts = out.counts.cpu().numpy()
    # tokens with at least one remote slot: what a sender that ships a token once per peer, not
    # once per assignment, would at least have to send (the byte counts are per assignment)
    remote_tokens = int((inp.mask[out.topk_idx.cpu().numpy()] == 0).any(axis=1).sum())
    share = np.sort(counts.astype(np.float64) / max(1, counts.sum()))[::-1]
    zipf = np.arange(1, cfg.E + 1, dtype=np.float64) ** -cfg.zipf_s
    log(f"[bench] realised expert shares (sorted) {np.round(share[:8], 3).tolist()} ... against Zipf(s={cfg.zipf_s}) "
        f"{np.round((zipf / zipf.sum())[:8], 3).tolist()}; tokens with a remote slot: {remote_tokens} of {cfg.T}")
    rows = n_local + cfg.S * cfg.T
    es = cfg.es
    dom_ms = stage_ms["ffn_up"]
    if decode:
        touched = int(np.sum((inp.mask == 1) & (counts > 0))) + cfg.S
        alg_bytes = touched * 2 * cfg.H * cfg.F * es + cfg.T * cfg.H * es + rows * cfg.F * es
        achieved = alg_bytes / (dom_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": achieved / PEAK_HBM_GBS, "traffic": read_traffic(cfg.name) if args.tokens is None else None,
                    "kernel": "grouped_gemm_kernel<gated> (gate/up projection + silu*up)",
                    "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": dom_ms}
    else:
        alg_flop = 4.0 * cfg.H * cfg.F * rows
        achieved = alg_flop / (dom_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": achieved, "peak": PEAK_MFMA_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": achieved / PEAK_MFMA_BF16_TFLOPS,
                    "traffic": read_traffic(cfg.name) if args.tokens is None else None,
                    "kernel": "grouped_gemm_kernel<gated> (gate/up projection + silu*up)",
                    "algorithmic_flop_per_launch": alg_flop, "kernel_ms": dom_ms}
    layer_flop = 2.0 * cfg.T * cfg.H * cfg.E + 6.0 * cfg.H * cfg.F * rows
    log(f"[bench] {cfg.name}: {ms_per_step:.3f} ms/step, {tokens_per_s:.4g} tokens/s, "
        f"n_local={n_local} n_remote={n_remote} local ratio={n_local / max(1, cfg.A):.3f}, "
        f"layer {layer_flop / (ms_per_step * 1e-3) / 1e12:.1f} TFLOP/s; stage ms: "
        + ", ".join(f"{k}={v:.4f}" for k, v in stage_ms.items()))

    result = {
        "metric": "moe_layer_tokens_per_sec", "value": tokens_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": workload, "tokens": cfg.T, "hidden": cfg.H, "ffn": cfg.F,
                   "experts": cfg.E, "top_k": cfg.k, "shared_experts": cfg.S,
                   "local_experts": int(inp.mask.sum()), "n_local": n_local, "n_remote": n_remote,
                   "remote_bytes_each_way": int(out.remote_bytes[0]),
                   "tokens_with_a_remote_slot": remote_tokens, "mask": args.mask,
                   "weight_copies_rotated": len(tables),
                   "weight_layout": args.weight_layout + (" (packed once at load, not timed)"
                                                          if args.weight_layout == "tiled" else "")},
        "roofline": roofline,
        "layer_tflops": layer_flop / (ms_per_step * 1e-3) / 1e12,
        "step_ms_median": step_ms[len(step_ms) // 2], "step_ms_min": step_ms[0],
    }
    if not args.no_ceilings:
        ceil = measured_ceilings(torch, P)
        result["measured_ceilings"] = ceil
        ref = ceil["hbm_read_gbs"] if decode else ceil["mfma_bf16_random_operands_tflops"]
        roofline["frac_of_measured_ceiling"] = roofline["achieved"] / ref
        log("[bench] measured ceilings: " + ", ".join(f"{k}={v:.1f}" for k, v in ceil.items()))
    if not args.no_cpu_baseline:
        n_sample = args.cpu_sample_tokens or cfg.T      # the whole batch: a few seconds of numpy
        result["cpu_baseline"] = cpu_baseline(inp, n_sample)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
