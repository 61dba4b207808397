"""Asynchronous expert migration next to a running layer (Sec. III-C "Expert Migration").

Adopting a new placement means loading the admitted experts' weights onto the server while it
keeps serving under the old placement, then switching the mask.  Here the load is a host-to-
device copy on a second HIP stream (default priority) that overlaps the layer's kernels; the
switch is a copy of the new mask enqueued on the compute stream behind an event of the copy
stream, so every layer call enqueued before it runs under the old mask with the old weights and
every call after it under the new mask with all admitted weights in place.  Eq. 3 prices the
migration as (changed placement entries) x m_e / speed; the measured copy time gives the speed.

    python -m paper_2508_12851_amd.migration        # config 5 at full size, prints one JSON line
"""
from __future__ import annotations

import json
import time
from typing import Dict, Iterable, Sequence

import numpy as np


class Migrator:
    """Loads experts into a WeightTable on a copy stream and flips the mask stream-ordered."""

    def __init__(self):
        import torch
        self.torch = torch
        self.copy_stream = torch.cuda.Stream()            # default priority
        self.done = torch.cuda.Event(enable_timing=True)
        self.begun = torch.cuda.Event(enable_timing=True)
        self.bytes = 0
        self._staged_mask = None

    def start(self, table, host_experts: Dict[int, Sequence], new_mask: np.ndarray) -> None:
        """host_experts: expert id -> (w_gate, w_up, w_down) PINNED host tensors of the admitted
        experts.  Enqueues their upload and the pointer-table update on the copy stream."""
        torch = self.torch
        experts = table.keep[0]
        self.bytes = 0
        ptrs = [t.cpu().clone() for t in table.tables[:3]]
        # destination buffers are allocated up front (allocation is not part of the overlap)
        dst = {e: tuple(torch.empty(w.shape, dtype=w.dtype, device="cuda") for w in ws)
               for e, ws in host_experts.items()}
        self.copy_stream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(self.copy_stream):
            self.begun.record()
            for e, ws in host_experts.items():
                for i, w in enumerate(ws):
                    if not w.is_pinned():
                        raise ValueError("migration sources must be pinned host tensors")
                    dst[e][i].copy_(w, non_blocking=True)
                    self.bytes += w.numel() * w.element_size()
                    ptrs[i][e] = dst[e][i].data_ptr()
                experts[e] = dst[e]
            # entries of the admitted experts only change here; running layers never read them
            self._ptr_host = [p.pin_memory() for p in ptrs]
            for i in range(3):
                table.tables[i].copy_(self._ptr_host[i], non_blocking=True)
            self.done.record()
        self._staged_mask = torch.from_numpy(np.ascontiguousarray(new_mask, dtype=np.uint8)).pin_memory()

    def commit(self, mask_dev, stream=None) -> None:
        """Switches mask_dev to the new placement at this point of `stream` (the compute stream):
        waits there for the uploads, then overwrites the mask."""
        torch = self.torch
        s = torch.cuda.current_stream() if stream is None else stream
        s.wait_event(self.done)
        with torch.cuda.stream(s):
            mask_dev.copy_(self._staged_mask, non_blocking=True)

    def copy_seconds(self) -> float:
        self.done.synchronize()
        return self.begun.elapsed_time(self.done) * 1e-3


def run_migration_demo(config: str = "cfg5_dsv2lite_migration", steps_each: int = 6, **overrides) -> Dict:
    """Phase-1 traffic of the migration workload: steps under the stale phase-0 mask, the same
    steps while the 16 admitted experts upload, then steps under the phase-1 mask."""
    import torch

    from prism_inputs import make_config, make_inputs

    from . import binding as B
    from . import placement as PL

    def dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).cuda()
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    def host_pinned(a):
        t = torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16) if a.dtype == np.uint16 \
            else torch.from_numpy(np.ascontiguousarray(a))
        return t.pin_memory()

    cfg = make_config(config, **overrides)
    p0 = make_inputs(cfg, phase=0)
    p1 = make_inputs(cfg, phase=1, weights="all", threads=16)
    admitted = [e for e in range(cfg.E) if p1.mask[e] and not p0.mask[e]]
    desc = B.make_desc(cfg.H, cfg.F, cfg.E, cfg.k, cfg.S, cfg.dtype, cfg.bias_group_tokens)
    experts = [tuple(dev(w) for w in p1.expert(e)) if p0.mask[e] else None for e in range(cfg.E)]
    shared = [tuple(dev(w) for w in p1.shared(s)) for s in range(cfg.S)]
    table = B.WeightTable(experts, shared)
    host = {e: tuple(host_pinned(w) for w in p1.expert(e)) for e in admitted}
    x, w_r, bias = dev(p1.x), dev(p1.w_router), dev(p1.bias)
    mask = dev(p0.mask.copy())
    ws = B.alloc_workspace(desc, cfg.T)
    out = B.alloc_layer_out(desc, cfg.T)

    def timed(n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            B.prism_moe_layer(desc, x, w_r, bias, table, mask, ws, outputs=out)
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t0) / n

    timed(3)
    ms_before = timed(steps_each)
    stale_local = int(out.n_local_remote[0])
    mig = Migrator()
    mig.start(table, host, p1.mask)
    ms_during = timed(steps_each)                       # overlaps the upload
    still_stale = int(out.n_local_remote[0])
    copy_s = mig.copy_seconds()
    mig.commit(mask)
    ms_after = timed(steps_each)
    new_local = int(out.n_local_remote[0])

    expert_bytes = 3.0 * cfg.H * cfg.F * cfg.es
    speed = mig.bytes / copy_s
    eq3_s, flips = PL.migration_cost(p0.mask.reshape(1, 1, -1), p1.mask.reshape(1, 1, -1),
                                     expert_bytes, [speed])
    return {
        "workload": cfg.name, "admitted_experts": len(admitted), "bytes_loaded": mig.bytes,
        "copy_ms": copy_s * 1e3, "measured_speed_gbs": speed / 1e9,
        "eq3_flips": flips, "eq3_seconds_at_measured_speed": eq3_s,
        "ms_per_step_before": ms_before, "ms_per_step_during_upload": ms_during,
        "ms_per_step_after": ms_after,
        "local_ratio_stale_mask": stale_local / cfg.A, "local_ratio_during": still_stale / cfg.A,
        "local_ratio_new_mask": new_local / cfg.A,
    }


if __name__ == "__main__":
    print(json.dumps(run_migration_demo()))
