"""What is the fastest this GPU streams from HBM, and with which access pattern?

    python -m paper_2508_12851_amd.ceiling_study [--gib 4] [--reps 3]
    python -m paper_2508_12851_amd.ceiling_study --single-launch-mib 1120

The second form times ONE launch that reads the given number of MiB (the weights one decode
GEMM streams), start-up and tail of the launch included, on buffers that rotate so that no
launch finds its data in the last-level cache: what a kernel of that size can reach at best.

Sweeps prism_ceiling_hbm_read_pattern over workgroups per launch, loads in flight per thread,
contiguous span per workgroup and load kind, on a zero-filled buffer 16x the last-level cache,
and prints every point and the best ones (GB/s).  The decode path of the layer is judged
against 8 TB/s nominal; this says how much of that any kernel can reach on the machine at hand.
"""
import argparse
import itertools
import json

import torch

import paper_2508_12851_amd as P

MODES = {0: "registers", 1: "direct-to-LDS", 2: "non-temporal", 3: "LDS non-temporal"}


def single_launch(nbytes):
    import numpy as np
    bufs = [torch.zeros(nbytes, dtype=torch.uint8, device="cuda") for _ in range(4)]
    sink = torch.empty(65536 * 4096, dtype=torch.uint8, device="cuda")
    print(f"one launch reading {nbytes / 1e6:.0f} MB, median of 10 launches on 4 rotating buffers")
    for grid, mode, u, span in itertools.product((224, 256), (1, 3, 2), (8, 16), (256 << 10, 512 << 10, 1 << 20)):
        ts = []
        for i in range(12):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            n = P.prism_ceiling_hbm_read_pattern(bufs[i % 4], sink, grid, u, span, mode)
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        t = float(np.median(ts[2:]))
        print(f"{MODES[mode]:<16} workgroups {grid}  in flight {u:>2}  span {span >> 10:>5} KiB: {t * 1e3:7.1f} us  "
              f"{n / t / 1e6:7.1f} GB/s", flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gib", type=int, default=4)
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--json", default=None, help="also write all points to this file")
    ap.add_argument("--single-launch-mib", type=int, default=None)
    args = ap.parse_args()
    if args.single_launch_mib is not None:
        return single_launch(args.single_launch_mib << 20)
    nbytes = args.gib << 30
    src = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    sink = torch.empty(65536 * 4096, dtype=torch.uint8, device="cuda")
    points = []
    spans = [16 << 10, 64 << 10, 256 << 10, 1 << 20, 4 << 20, 16 << 20]
    grids = [256, 512, 1024, 2048, 4096, 16384, 65536]
    for mode, u, span, grid in itertools.product(MODES, (2, 4, 8, 16), spans, grids):
        if span % (4096 * u) or nbytes // span < grid // 4:
            continue                      # spans must hold whole trips; most workgroups need a span
        P.prism_ceiling_hbm_read_pattern(src, sink, grid, u, span, mode)            # warm-up
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        n = sum(P.prism_ceiling_hbm_read_pattern(src, sink, grid, u, span, mode) for _ in range(args.reps))
        e1.record()
        torch.cuda.synchronize()
        gbs = n / (e0.elapsed_time(e1) * 1e-3) / 1e9
        points.append(dict(mode=MODES[mode], loads_in_flight=u, span_kib=span >> 10, workgroups=grid, gbs=gbs))
        print(f"{MODES[mode]:<16} in flight {u:>2}  span {span >> 10:>6} KiB  workgroups {grid:>6}  {gbs:8.1f} GB/s",
              flush=True)
    # the committed ceiling kernel (grid-strided 16-byte loads, 4 in flight) for comparison
    out = torch.empty(32768 * 256 * 16, dtype=torch.uint8, device="cuda")
    P.prism_ceiling_hbm_read(src, out, 32768)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    n = sum(P.prism_ceiling_hbm_read(src, out, 32768) for _ in range(args.reps))
    e1.record()
    torch.cuda.synchronize()
    base = n / (e0.elapsed_time(e1) * 1e-3) / 1e9
    print(f"\nprism_ceiling_hbm_read (what bench.py reports): {base:.1f} GB/s")
    points.sort(key=lambda p: -p["gbs"])
    print("best patterns:")
    for p in points[:12]:
        print(f"  {p['gbs']:8.1f} GB/s  {p['mode']:<16} in flight {p['loads_in_flight']:>2}  span {p['span_kib']:>6} KiB  "
              f"workgroups {p['workgroups']:>6}")
    for mode in MODES.values():
        best = max((p for p in points if p["mode"] == mode), key=lambda p: p["gbs"])
        print(f"best {mode}: {best['gbs']:.1f} GB/s ({best})")
    if args.json:
        json.dump(dict(points=points, baseline_gbs=base), open(args.json, "w"))


if __name__ == "__main__":
    main()
