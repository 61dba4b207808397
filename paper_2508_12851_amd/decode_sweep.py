"""Multi-layer decode loop and local-fraction sweep on one GPU (one simulated edge server).

L stacked MoE layers, each with its own weights, its own expert popularity (layer-wise
variation, Sec. II-B) and its own placement mask; a decode step runs the layers one after the
other (x <- x + layer(x)), so the hosted experts' weights stream from HBM layer after layer as
in a real decode step.  Sweeping the number of hosted experts per layer from 0 to E gives this
build's analogue of the paper's Fig. 4: time of the local part of a layer and bytes that would
cross the network, against the proportion of expert calls served remotely.

    python -m paper_2508_12851_amd.decode_sweep [--layers 16] [--tokens 32] [--graph]

Weights are synthetic (N(0, 1/H), drawn on the GPU), popularity bias is the seeded Zipf bias of
prism_inputs with one rank permutation per layer, masks host the most popular experts.
"""
from __future__ import annotations

import argparse
import json
import time
from typing import Dict, List

import numpy as np


class Stack:
    """L layers resident in HBM: router, bias, all E experts (so any mask can be swept)."""

    def __init__(self, n_layers: int, T: int, H: int, F: int, E: int, k: int, zipf_s: float = 1.0,
                 seed: int = 0):
        import torch

        from prism_inputs import zipf_bias

        from . import binding as B

        self.B, self.torch = B, torch
        self.L, self.T, self.H, self.F, self.E, self.k = n_layers, T, H, F, E, k
        self.desc = B.make_desc(H, F, E, k, 0, "bf16", 0)
        gen = torch.Generator(device="cuda").manual_seed(seed)

        def normal(shape, std):
            return (torch.randn(shape, generator=gen, device="cuda") * std).to(torch.bfloat16)

        rng = np.random.default_rng(seed)
        self.w_router, self.bias, self.tables, self.ranks = [], [], [], []
        for _ in range(n_layers):
            self.w_router.append(normal((E, H), H ** -0.5))
            ranks = np.empty(E, np.int64)
            ranks[rng.permutation(E)] = np.arange(1, E + 1)
            self.ranks.append(ranks)
            self.bias.append(torch.from_numpy(zipf_bias(ranks, zipf_s).reshape(1, E)
                                              .astype(np.float32)).cuda())
            experts = [(normal((F, H), H ** -0.5), normal((F, H), H ** -0.5), normal((H, F), F ** -0.5))
                       for _ in range(E)]
            self.tables.append(B.WeightTable(experts, []))
        self.x0 = normal((T, H), 1.0)
        self.ws = B.alloc_workspace(self.desc, T)
        self.outs = [B.alloc_layer_out(self.desc, T) for _ in range(n_layers)]
        self.accum = [torch.zeros(E, dtype=torch.int64, device="cuda") for _ in range(n_layers)]

    def masks_hosting(self, n_local: int):
        """Per layer: the n_local most popular experts of that layer."""
        torch = self.torch
        masks = []
        for ranks in self.ranks:
            m = np.zeros(self.E, np.uint8)
            m[np.argsort(ranks, kind="stable")[:n_local]] = 1
            masks.append(torch.from_numpy(m).cuda())
        return masks

    def step(self, masks, x=None, stream=None):
        """One decode step through all layers; returns the final hidden state."""
        B = self.B
        x = self.x0 if x is None else x
        for l in range(self.L):
            o = B.prism_moe_layer(self.desc, x, self.w_router[l], self.bias[l], self.tables[l],
                                  masks[l], self.ws, outputs=self.outs[l],
                                  counts_accum=self.accum[l], stream=stream)
            x = x + o.out
        return x


def sweep(n_layers: int = 16, T: int = 32, H: int = 4096, F: int = 14336, E: int = 8, k: int = 2,
          steps: int = 20, warmup: int = 3, use_graph: bool = False, seed: int = 0) -> List[Dict]:
    import torch

    st = Stack(n_layers, T, H, F, E, k, seed=seed)
    rows = []
    es = 2
    for n_local in range(E + 1):
        masks = st.masks_hosting(n_local)
        for _ in range(warmup):
            st.step(masks)
        torch.cuda.synchronize()
        graph = None
        if use_graph:
            side = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    st.step(masks, stream=side)
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay() if graph is not None else st.step(masks)
        torch.cuda.synchronize()
        ms = 1e3 * (time.perf_counter() - t0) / steps
        n_loc = sum(int(o.n_local_remote[0]) for o in st.outs)
        n_rem = sum(int(o.n_local_remote[1]) for o in st.outs)
        remote_bytes = sum(int(o.remote_bytes.sum()) for o in st.outs)
        touched = sum(int(((o.counts > 0) & (m > 0)).sum()) for o, m in zip(st.outs, masks))
        weight_bytes = touched * 3 * H * F * es
        rows.append({
            "hosted_experts_per_layer": n_local, "layers": n_layers, "tokens": T,
            "remote_fraction": n_rem / max(1, n_loc + n_rem),
            "ms_per_step": ms, "ms_per_layer": ms / n_layers, "tokens_per_s": T / (ms * 1e-3),
            "remote_bytes_per_step": remote_bytes,
            "weight_bytes_streamed_per_step": weight_bytes,
            "hbm_gbs": weight_bytes / (ms * 1e-3) / 1e9,
            "graph": bool(use_graph),
        })
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=16)
    ap.add_argument("--tokens", type=int, default=32)
    ap.add_argument("--hidden", type=int, default=4096)
    ap.add_argument("--ffn", type=int, default=14336)
    ap.add_argument("--experts", type=int, default=8)
    ap.add_argument("--top-k", type=int, default=2)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--graph", action="store_true", help="replay each step from a captured graph")
    a = ap.parse_args()
    for row in sweep(a.layers, a.tokens, a.hidden, a.ffn, a.experts, a.top_k, a.steps,
                     use_graph=a.graph):
        print(json.dumps(row), flush=True)


if __name__ == "__main__":
    main()
