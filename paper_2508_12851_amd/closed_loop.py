"""The feedback loop of Sec. III-A/III-C on one GPU: N simulated edge servers x L MoE layers.

Window 1: every server runs its layers under a uniform placement and the layer accumulates the
activation counts f_n^l(e).  The scheduler-side pipeline (entropy, Alg. 1, Alg. 2) turns them
into a new placement; Eq. 3/4 price the migration.  Window 2: fresh tokens with the same
popularity run under both placements; the remote assignments the layer lists are Eq. 2's
proxy cost of the placement on that window's counts.

Everything on the GPU goes through the C ABI (prism_moe_layer); the planning is the native host
code of prism_placement.h.  Inputs are the seeded synthetic workloads of prism_inputs: one
weight seed per layer, one popularity (bias) draw per server.

    python -m paper_2508_12851_amd.closed_loop [--servers 4] [--layers 4] [--config cfg5_dsv2lite_migration]
"""
from __future__ import annotations

import argparse
import json
from typing import Dict

import numpy as np


def uniform_placement(n_servers: int, n_layers: int, n_experts: int) -> np.ndarray:
    """Expert e of every layer on server e * N // E (the 'Uniform' split of Sec. IV-A)."""
    place = np.zeros((n_servers, n_layers, n_experts), np.uint8)
    for e in range(n_experts):
        place[e * n_servers // n_experts, :, e] = 1
    return place


def run_closed_loop(config: str = "cfg5_dsv2lite_migration", n_servers: int = 4, n_layers: int = 4,
                    mem_fraction: float = 0.5, link_bytes_per_s: float = 62.5e6,
                    io_bytes_per_s: float = 25e9, **overrides) -> Dict:
    """mem_fraction: a server's memory as a fraction of the whole model (L * E experts).
    link_bytes_per_s: server-to-server bandwidth used to turn a remote call into seconds
    (500 Mbps, the paper's emulated edge link); io_bytes_per_s: expert load bandwidth (Eq. 3)."""
    import torch

    from prism_inputs import make_config, make_inputs

    from . import binding as B
    from . import placement as PL

    def dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).cuda()
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    overrides = {**overrides, "n_phases": max(n_servers, 2)}    # one popularity draw per server
    base = make_config(config, **overrides)
    N, L, E = n_servers, n_layers, base.E
    cfgs = [make_config(config, **{**overrides, "seed": base.seed + 7919 * l}) for l in range(L)]
    desc = B.make_desc(base.H, base.F, E, base.k, base.S, base.dtype, base.bias_group_tokens)
    ws = B.alloc_workspace(desc, base.T)

    tables = []
    for l in range(L):                                   # the model: all experts of every layer
        inp = make_inputs(cfgs[l], weights="all")
        tables.append(B.WeightTable([tuple(dev(w) for w in inp.expert(e)) for e in range(E)],
                                    [tuple(dev(w) for w in inp.shared(s)) for s in range(base.S)]))

    def window(placement: np.ndarray, tokens_seed: int):
        """One pass of every (server, layer) under `placement`: counts and remote assignments."""
        f = np.zeros((N, L, E), np.int64)
        remote = np.zeros((N, L), np.int64)
        for n in range(N):
            for l in range(L):
                c = make_config(config, **{**overrides, "seed": cfgs[l].seed,
                                           "tokens_seed": tokens_seed})
                inp = make_inputs(c, phase=n)            # phase n: server n's own popularity draw
                accum = torch.zeros(E, dtype=torch.int64, device="cuda")
                o = B.prism_moe_layer(desc, dev(inp.x), dev(inp.w_router), dev(inp.bias), tables[l],
                                      dev(placement[n, l]), ws, counts_accum=accum)
                f[n, l] = accum.cpu().numpy()
                remote[n, l] = int(o.n_local_remote[1])
        return f, remote

    uniform = uniform_placement(N, L, E)
    f1, remote1 = window(uniform, tokens_seed=10_001)
    server_mem = [mem_fraction * L * E] * N              # in experts (m_e = 1)
    v, counts, planned, ok = PL.placement_plan(f1, server_mem, 1.0)

    f2, remote_uniform = window(uniform, tokens_seed=10_002)
    _, remote_planned = window(planned, tokens_seed=10_002)

    expert_bytes = 3.0 * base.H * base.F * base.es
    t_mig, flips = PL.migration_cost(uniform, planned, expert_bytes, [io_bytes_per_s] * N)
    seconds_per_remote_call = 2.0 * base.H * base.es / link_bytes_per_s      # one row each way
    cost_old, cost_new = PL.proxy_cost(f1, uniform), PL.proxy_cost(f1, planned)
    adopt = PL.migration_decision(cost_old, cost_new, t_mig, seconds_per_remote_call)
    total = int(f2.sum())
    return {
        "servers": N, "layers": L, "experts": E, "plan_ok": ok,
        "entropy_bits_mean": float(v.mean()), "experts_per_server": counts.sum(axis=1).tolist(),
        "window1_proxy_cost_uniform": cost_old, "window1_proxy_cost_planned": cost_new,
        "window2_remote_uniform": int(remote_uniform.sum()),
        "window2_remote_planned": int(remote_planned.sum()),
        "window2_eq2_uniform": PL.proxy_cost(f2, uniform),
        "window2_eq2_planned": PL.proxy_cost(f2, planned),
        "local_ratio_uniform": float(1.0 - remote_uniform.sum() / total),
        "local_ratio_planned": float(1.0 - remote_planned.sum() / total),
        "migration_flips": flips, "migration_seconds": t_mig,
        "seconds_per_remote_call": seconds_per_remote_call, "adopt": adopt,
        "window1_remote_uniform": int(remote1.sum()),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg5_dsv2lite_migration")
    ap.add_argument("--servers", type=int, default=4)
    ap.add_argument("--layers", type=int, default=4)
    ap.add_argument("--mem-fraction", type=float, default=0.5)
    ap.add_argument("--tokens", type=int, default=2048)
    ap.add_argument("--hidden", type=int, default=512)
    ap.add_argument("--ffn", type=int, default=512)
    a = ap.parse_args()
    print(json.dumps(run_closed_loop(a.config, a.servers, a.layers, a.mem_fraction,
                                     T=a.tokens, H=a.hidden, F=a.ffn)))


if __name__ == "__main__":
    main()
