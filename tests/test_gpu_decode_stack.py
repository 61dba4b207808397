"""Stacked layers in a decode loop: per-layer masks and counts, the chain against the oracle,
the sweep's bookkeeping, and replay of a captured graph against eager execution."""
import numpy as np
import pytest
import torch

import paper_2508_12851_amd as P
from oracle import prism_oracle as O
from paper_2508_12851_amd.decode_sweep import Stack, sweep

from gpu_util import TOL, rel_err, to_f32

pytestmark = pytest.mark.gpu


def _host(t):
    return t.detach().float().cpu().numpy()


def test_stack_matches_oracle_chain_layer_by_layer():
    st = Stack(n_layers=3, T=24, H=256, F=192, E=8, k=2, seed=5)
    masks = st.masks_hosting(5)
    x = st.x0
    for l in range(st.L):
        o = P.prism_moe_layer(st.desc, x, st.w_router[l], st.bias[l], st.tables[l], masks[l], st.ws,
                              outputs=st.outs[l])
        torch.cuda.synchronize()
        experts = lambda e: tuple(_host(w) for w in st.tables[l].keep[0][e])
        ref = O.moe_layer(_host(x), _host(st.w_router[l]), _host(st.bias[l]), experts, [],
                          masks[l].cpu().numpy(), st.k, "bf16", 0)
        assert np.array_equal(o.topk_idx.cpu().numpy(), ref.route.topk_idx)
        assert np.array_equal(o.counts.cpu().numpy(), ref.route.counts)
        assert o.n_local_remote.cpu().tolist() == [ref.dispatch.n_local, ref.dispatch.n_remote]
        assert rel_err(to_f32(o.out), ref.out) <= TOL["bf16"]
        x = x + o.out                         # the GPU's own hidden state feeds the next layer
    # the layers differ: popularity (hence masks and counts) varies layer by layer
    assert len({tuple(m.cpu().tolist()) for m in masks}) > 1


def test_sweep_bookkeeping_small():
    rows = sweep(n_layers=2, T=16, H=256, F=192, E=8, k=2, steps=2, warmup=1)
    assert [r["hosted_experts_per_layer"] for r in rows] == list(range(9))
    assert rows[0]["remote_fraction"] == 1.0 and rows[-1]["remote_fraction"] == 0.0
    fr = [r["remote_fraction"] for r in rows]
    assert all(a >= b for a, b in zip(fr, fr[1:]))                # hosting more never sends more
    for r in rows:
        n_rem = round(r["remote_fraction"] * 2 * 16 * 2)
        assert r["remote_bytes_per_step"] == 2 * n_rem * 256 * 2  # one bf16 row each way per call
    assert rows[0]["weight_bytes_streamed_per_step"] == 0


def test_graph_replay_equals_eager():
    """A decode step captured in a graph (no allocation, no memset node inside the library) and
    replayed several times, with eager work in between, gives the eager result every time."""
    st = Stack(n_layers=3, T=32, H=256, F=448, E=8, k=2, seed=9)
    masks = st.masks_hosting(5)
    eager = st.step(masks).clone()
    eager_counts = [o.counts.clone() for o in st.outs]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            y = st.step(masks, stream=side)
    torch.cuda.synchronize()
    for i in range(4):
        for o in st.outs:                      # eager work between replays: poison the outputs
            o.out.fill_(float("nan"))
            o.counts.fill_(-1)
        st.ws.fill_(0x7F)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, eager), i
        for o, c in zip(st.outs, eager_counts):
            assert torch.equal(o.counts, c)
