#!/usr/bin/env python3
"""Benchmark of the placement-aware MoE layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config NAME] [--phase P]

A step is one call of prism_moe_layer (route -> dispatch -> grouped SwiGLU FFN
over the local experts -> combine) on one batch of seeded synthetic input that
is already resident in HBM.  Prints ONE JSON line: whole-job tokens/s, the
roofline fraction of the dominant kernel (timed with HIP events recorded by the
library around that kernel on the launch stream) and of the whole layer, and the
CPU oracle timed on a bounded sample of the same workload.

The default run times the Mixtral-shaped prefill batch (the line's `value`) and,
under the key `decode`, the decode batch of the same layer -- the two halves of
the headline metric: fraction of the bf16 MFMA peak and fraction of the HBM
bandwidth.  `--config cfg5_dsv2lite_migration` times both phases of the
migration scenario (`phases`), `--phase 0|1` one of them.
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
DECODE_CONFIG = "cfg3_mixtral_decode"
DECODE_WEIGHT_COPIES = 4           # rotate weight copies so the 256 MB last-level cache cannot help
GEMM1 = "grouped_gemm_kernel<gated> (gate/up projection + silu*up)"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def read_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary,
    and the commit it was measured at -- or (None, reason) when the summary is missing or was
    measured on kernel sources other than the ones this run uses."""
    from paper_2508_12851_amd.profile_summary import kernel_source_hash
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None, "no committed counter summary for this workload"
    fields = {}
    for line in open(path):
        for key in ("traffic_bytes_per_launch", "kernel_source_sha256", "commit"):
            if line.startswith(key):
                fields[key] = line.split("=", 1)[1].strip()
    if fields.get("kernel_source_sha256") != kernel_source_hash():
        return None, "the committed counter summary was measured on other kernel sources"
    return float(fields["traffic_bytes_per_launch"]), fields.get("commit", "")


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
    # the same read with loads marked non-temporal, in the pattern the ceiling study found fastest
    # (256 workgroups, 256 KiB spans, 16 loads in flight per thread): what the decode GEMMs' weight
    # loads, marked the same way, are up against
    pattern = dict(n_workgroups=256, loads_in_flight=16, span_bytes=256 << 10, mode=2)
    P.prism_ceiling_hbm_read_pattern(src, sink, **pattern)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    nbytes = sum(P.prism_ceiling_hbm_read_pattern(src, sink, **pattern) for _ in range(5))
    e1.record()
    torch.cuda.synchronize()
    res["hbm_read_nontemporal_gbs"] = nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
    return res


def cpu_baseline(inp, n_sample: int):
    """Time the CPU oracle, as it stands, on the first n_sample tokens of the workload."""
    from oracle import prism_oracle as O
    cores = len(os.sched_getaffinity(0))        # the cores this process (and numpy under it) may use
    c = inp.cfg
    f = inp.f32
    n = min(n_sample, c.T)
    xs = f(inp.x)[:n]
    # whole passes over the sample until about 10 s of CPU work are on the clock (4 passes at most)
    passes, dt = 0, 0.0
    while passes < 4 and dt < 10.0:
        t0 = time.perf_counter()
        O.moe_layer(xs, f(inp.w_router), inp.bias, lambda e: tuple(f(w) for w in inp.expert(e)),
                    [tuple(f(w) for w in inp.shared(s)) for s in range(c.S)], inp.mask, c.k, c.dtype,
                    c.bias_group_tokens, np.arange(n))
        dt += time.perf_counter() - t0
        passes += 1
    return {"value": n * passes / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {n} of {c.T} tokens of {c.name}, whole layer, {passes} passes, {dt:.1f} s"}


class DeviceWeights:
    """Expert weights uploaded once per (expert, layout) and shared by the workloads of a run
    that use the same layer (the decode batch runs on the prefill batch's layer)."""

    def __init__(self, torch, P, layout, values="real"):
        self.torch, self.P, self.layout, self.values = torch, P, layout, values
        self.cache = {}

    def dev(self, a):
        torch = self.torch
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
        return torch.from_numpy(a).cuda()

    def triple(self, key, arrays):
        if key not in self.cache:
            up = (lambda a: self.P.prism_pack_weights(self.dev(a))) if self.layout == "tiled" else self.dev
            t = tuple(up(w) for w in arrays)
            if self.values == "zero":
                t = tuple(w.zero_() for w in t)
            elif self.values == "constant":
                t = tuple(w.fill_(2.0 ** -6) for w in t)
            self.cache[key] = t
        return self.cache[key]


def run_workload(torch, P, cfg, inp, args, dw, *, steps, warmup, decode, label, rotate):
    """Times `steps` layer calls on one workload; returns its record and the last outputs."""
    desc = P.make_desc(cfg.H, cfg.F, cfg.E, cfg.k, cfg.S, cfg.dtype, cfg.bias_group_tokens,
                       weight_layout=args.weight_layout)
    experts = [dw.triple((cfg.seed, "e", e), inp.expert(e)) if inp.mask[e] else None for e in range(cfg.E)]
    shared = [dw.triple((cfg.seed, "s", s), inp.shared(s)) for s in range(cfg.S)]
    tables = [P.WeightTable(experts, shared)]
    for _ in range(rotate - 1):
        ex = [None if t is None else tuple(w.clone() for w in t) for t in experts]
        sh = [tuple(w.clone() for w in t) for t in shared]
        tables.append(P.WeightTable(ex, sh))
    x, w_router, bias, mask = dw.dev(inp.x), dw.dev(inp.w_router), dw.dev(inp.bias), dw.dev(inp.mask)
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

    # An event between two kernels costs about 6 us on the stream (a kernel trace of the decode
    # step shows it: back-to-back launches otherwise), 4 % of a decode step for the pair around
    # the dominant kernel.  Decode-sized workloads therefore carry the pair on every 8th timed
    # step; the kernel time is the mean over those steps, inside the timed region all the same.
    event_every = 8 if decode and steps >= 16 and not args.trace_all else 1
    timed = [i for i in range(steps) if i % event_every == 0]
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i, handle_arrays[i] if i % event_every == 0 else None)
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
                                               for i in timed]))
    n_local, n_remote = out.n_local_remote.cpu().tolist()
    counts = out.counts.cpu().numpy()
    # tokens with at least one remote slot: what a sender that ships a token once per peer, not
    # once per assignment, would at least have to send (the byte counts are per assignment)
    remote_tokens = int((inp.mask[out.topk_idx.cpu().numpy()] == 0).any(axis=1).sum())
    share = np.sort(counts.astype(np.float64) / max(1, counts.sum()))[::-1]
    zipf = np.arange(1, cfg.E + 1, dtype=np.float64) ** -cfg.zipf_s
    log(f"[bench] {label}: realised expert shares (sorted) {np.round(share[:8], 3).tolist()} ... against "
        f"Zipf(s={cfg.zipf_s}) {np.round((zipf / zipf.sum())[:8], 3).tolist()}; tokens with a remote slot: "
        f"{remote_tokens} of {cfg.T}")
    rows = n_local + cfg.S * cfg.T
    es = cfg.es
    dom_ms = stage_ms["ffn_up"]
    step_s = ms_per_step * 1e-3
    # the committed counter summaries were taken on the benchmark workloads as bench.py runs them by default
    as_profiled = (label == cfg.name and args.mask == "top" and args.weight_layout == "tiled" and
                   args.expert_weights == "real")
    traffic, traffic_note = read_traffic(cfg.name) if as_profiled else (None, "not the profiled workload")
    if decode:
        # the dominant kernel streams W_gate and W_up of every hosted expert that received a token
        touched = int(np.sum((inp.mask == 1) & (counts > 0))) + cfg.S
        alg_bytes = touched * 2 * cfg.H * cfg.F * es + cfg.T * cfg.H * es + rows * cfg.F * es
        achieved = alg_bytes / (dom_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "scope": "dominant kernel", "achieved": achieved, "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS, "traffic": traffic,
                    "traffic_source": traffic_note, "kernel": GEMM1,
                    "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": dom_ms,
                    "kernel_ms_from": f"HIP events around the kernel on every {event_every}th of the timed steps"
                                      if event_every > 1 else "HIP events around the kernel on every timed step"}
        # the whole layer: all three weight matrices of those experts, the tokens, the router, the output
        layer_bytes = (touched * 3 * cfg.H * cfg.F * es + cfg.T * cfg.H * es + cfg.E * cfg.H * es +
                       cfg.T * cfg.H * es)
        layer = {"bound": "hbm", "scope": "whole layer (all kernels, launch gaps included)",
                 "achieved": layer_bytes / step_s / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                 "frac": layer_bytes / step_s / 1e9 / PEAK_HBM_GBS, "algorithmic_bytes_per_step": layer_bytes}
    else:
        alg_flop = 4.0 * cfg.H * cfg.F * rows
        achieved = alg_flop / (dom_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "scope": "dominant kernel", "achieved": achieved,
                    "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_MFMA_BF16_TFLOPS,
                    "traffic": traffic, "traffic_source": traffic_note, "kernel": GEMM1,
                    "algorithmic_flop_per_launch": alg_flop, "kernel_ms": dom_ms,
                    "kernel_ms_from": "HIP events around the kernel on every timed step"}
        layer_flop = 2.0 * cfg.T * cfg.H * cfg.E + 6.0 * cfg.H * cfg.F * rows
        layer = {"bound": "mfma", "scope": "whole layer (all kernels, launch gaps included)",
                 "achieved": layer_flop / step_s / 1e12, "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
                 "frac": layer_flop / step_s / 1e12 / PEAK_MFMA_BF16_TFLOPS,
                 "algorithmic_flop_per_step": layer_flop}
    log(f"[bench] {label}: {ms_per_step:.3f} ms/step, {tokens_per_s:.4g} tokens/s, "
        f"n_local={n_local} n_remote={n_remote} local ratio={n_local / max(1, cfg.A):.3f}, "
        f"dominant kernel {roofline['frac']:.3f} / whole layer {layer['frac']:.3f} of the {roofline['bound']} peak; "
        "stage ms: " + ", ".join(f"{k}={v:.4f}" for k, v in stage_ms.items()))
    rec = {
        "workload": label, "tokens": cfg.T, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "tokens_per_s": tokens_per_s, "elapsed_s": elapsed,
        "step_ms_median": step_ms[len(step_ms) // 2], "step_ms_min": step_ms[0],
        "roofline": roofline, "layer_roofline": layer,
        "config": {"workload": label, "tokens": cfg.T, "hidden": cfg.H, "ffn": cfg.F,
                   "experts": cfg.E, "top_k": cfg.k, "shared_experts": cfg.S,
                   "local_experts": int(inp.mask.sum()), "n_local": n_local, "n_remote": n_remote,
                   "local_compute_ratio": n_local / max(1, cfg.A),
                   "remote_bytes_each_way": int(out.remote_bytes[0]),
                   "tokens_with_a_remote_slot": remote_tokens, "mask": args.mask,
                   "weight_copies_rotated": len(tables),
                   "weight_layout": args.weight_layout + (" (packed once at load, not timed)"
                                                          if args.weight_layout == "tiled" else "")},
        "counts": counts.tolist(),
    }
    if args.trace_all:
        rec["stage_ms"] = stage_ms
    del tables, ws, out
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", default=DEFAULT_CONFIG)
    ap.add_argument("--phase", choices=("0", "1", "both"), default="both",
                    help="two-phase (migration) workloads: time phase 0, phase 1 or both (the default; "
                         "the line's value is then the throughput over both phases, `phases` holds each)")
    ap.add_argument("--no-decode", action="store_true",
                    help="default workload only: skip the decode batch of the same layer")
    ap.add_argument("--cpu-sample-tokens", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--trace-all", action="store_true", help="also time every stage (stage_ms)")
    ap.add_argument("--weight-layout", choices=("row_major", "tiled"), default="tiled",
                    help="expert weight layout in HBM; tiled (16 x 32 tiles) is packed once, outside the "
                         "timed region, as a server does when it loads or receives an expert")
    ap.add_argument("--mask", choices=("top", "random"), default="top",
                    help="hosted experts: the most popular ones (what the first loop of Alg. 2 hosts) or a "
                         "seeded uniformly random subset of the same size (the uniform baseline of Sec. IV)")
    ap.add_argument("--tokens", type=int, default=None,
                    help="another batch size for the chosen workload's layer (not the benchmark line: "
                         "config.workload then says so)")
    ap.add_argument("--expert-weights", choices=("real", "zero", "constant"), default="real",
                    help="a measurement, not the benchmark line: overwrite the expert weights in HBM with zeros or "
                         "with one constant after loading them -- same routing, same kernels, same memory traffic, "
                         "but operands that barely toggle the matrix cores, which shows how much of the GEMM time "
                         "is the chip's data-dependent, power-limited clock")
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
    phases = [0] if cfg.n_phases == 1 else ([0, 1] if args.phase == "both" else [int(args.phase)])

    dw = DeviceWeights(torch, P, args.weight_layout, args.expert_weights)
    if args.expert_weights != "real":
        workload += f" with {args.expert_weights} expert weights (a power measurement, not the benchmark)"
    recs, inputs = [], []
    for phase in phases:
        t0 = time.perf_counter()
        inp = make_inputs(cfg, phase=phase)
        if inputs:                                   # same layer in every phase: share the host copies
            inp._experts, inp._shared = inputs[0]._experts, inputs[0]._shared
        inp.materialize([int(e) for e in np.flatnonzero(inp.mask)], threads=16)
        log(f"[bench] generated {cfg.name} inputs (phase {phase}) in {time.perf_counter() - t0:.1f} s")
        label = workload if cfg.n_phases == 1 else f"{workload} phase {phase}"
        recs.append(run_workload(torch, P, cfg, inp, args, dw, steps=steps, warmup=warmup, decode=decode,
                                 label=label, rotate=DECODE_WEIGHT_COPIES if decode else 1))
        inputs.append(inp)
    main_rec = recs[0]
    total_tokens = sum(r["tokens"] * r["steps"] for r in recs)
    total_s = sum(r["elapsed_s"] for r in recs)

    result = {
        "metric": "moe_layer_tokens_per_sec", "value": total_tokens / total_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": 1e3 * total_s / (steps * len(recs)),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": dict(main_rec["config"], workload=workload),
        "roofline": main_rec["roofline"], "layer_roofline": main_rec["layer_roofline"],
        "layer_tflops": main_rec["layer_roofline"]["achieved"] if not decode else None,
        "step_ms_median": main_rec["step_ms_median"], "step_ms_min": main_rec["step_ms_min"],
    }
    if args.trace_all:
        result["stage_ms"] = main_rec["stage_ms"]
    if len(recs) > 1:
        # per phase: counts, split, remote bytes, throughput (the mask and the popularity ranking change
        # between the phases; the migration itself is the mask change, 16 experts = 277 MB to load)
        result["phases"] = [{k: r[k] for k in ("workload", "ms_per_step", "tokens_per_s", "roofline",
                                               "layer_roofline", "config", "counts")} for r in recs]
        m0, m1 = inputs[0].mask, inputs[1].mask
        result["migration"] = {"experts_admitted": int(np.sum((m1 == 1) & (m0 == 0))),
                               "experts_evicted": int(np.sum((m1 == 0) & (m0 == 1))),
                               "bytes_loaded": int(np.sum((m1 == 1) & (m0 == 0))) * 3 * cfg.H * cfg.F * cfg.es,
                               "changed_entries_eq3": int(np.sum(m0 != m1))}

    if args.config == DEFAULT_CONFIG and args.tokens is None and not args.no_decode:
        # the other half of the headline metric: the decode batch of the same layer (same weights, already
        # in HBM), rotating through distinct copies of them so that the last-level cache cannot serve any
        dcfg = CONFIGS[DECODE_CONFIG] if args.mask == "top" else make_config(DECODE_CONFIG, mask_kind="random")
        dinp = make_inputs(dcfg)
        dinp._experts, dinp._shared = inputs[0]._experts, inputs[0]._shared
        d = run_workload(torch, P, dcfg, dinp, args, dw, steps=200, warmup=20, decode=True,
                         label=dcfg.name, rotate=DECODE_WEIGHT_COPIES)
        result["decode"] = {k: d[k] for k in ("workload", "steps", "warmup", "ms_per_step", "tokens_per_s",
                                              "step_ms_median", "step_ms_min", "roofline", "layer_roofline",
                                              "config")}
    dw.cache.clear()
    torch.cuda.empty_cache()
    if not args.no_ceilings:
        ceil = measured_ceilings(torch, P)
        result["measured_ceilings"] = ceil
        for rec in [result] + ([result["decode"]] if "decode" in result else []):
            rf = rec["roofline"]
            ref = (max(ceil["hbm_read_gbs"], ceil["hbm_read_nontemporal_gbs"]) if rf["bound"] == "hbm"
                   else ceil["mfma_bf16_random_operands_tflops"])
            rf["frac_of_measured_ceiling"] = rf["achieved"] / ref
        log("[bench] measured ceilings: " + ", ".join(f"{k}={v:.1f}" for k, v in ceil.items()))
    if not args.no_cpu_baseline:
        n_sample = args.cpu_sample_tokens or cfg.T      # the whole batch: a few seconds of numpy
        result["cpu_baseline"] = cpu_baseline(inputs[0], n_sample)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
