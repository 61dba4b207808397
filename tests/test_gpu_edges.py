"""GPU parity at the edges of the launch configurations: batch sizes around the decode /
prefill switch and around the tile heights, the shortest contractions the tile rings
accept, one expert taking every token, a non-default stream with accumulated counts and
stage events, and a workspace sized for a larger batch."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2508_12851_amd as P
from prism_inputs import make_config, make_inputs

from gpu_util import check_layer, desc_of, oracle_layer, run_layer, to_dev, weight_table

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T", [2, 15, 16, 17, 63, 64, 65, 255, 256, 257, 513])
def test_batch_sizes_around_tile_and_path_boundaries(T):
    cfg = make_config("cfg2_mixtral_prefill", T=T, H=256, F=448)
    inp = make_inputs(cfg)
    err = check_layer(cfg, run_layer(cfg, inp), oracle_layer(inp))
    print(f"T={T}: out err {err:.3g}")


@pytest.mark.parametrize("T", [64, 65, 127, 128, 129, 257, 512, 513])
def test_batch_sizes_of_a_wide_layer_around_the_tile_and_path_boundaries(T):
    """H >= 256 and F >= 1024: batches of 65..512 tokens take 128 x 256 tiles and a split down
    projection; 64 and 513 are the neighbouring paths."""
    cfg = make_config("cfg2_mixtral_prefill", T=T, H=256, F=1024)
    inp = make_inputs(cfg)
    err = check_layer(cfg, run_layer(cfg, inp), oracle_layer(inp))
    print(f"T={T}: out err {err:.3g}")


@pytest.mark.parametrize("T", [24, 300])
@pytest.mark.parametrize("H,F", [(64, 64), (128, 64), (64, 192), (192, 128), (128, 1024), (256, 1024)])
def test_shortest_contractions(T, H, F):
    """H or F of 64..192: the k-tile ring is as long as the whole contraction."""
    cfg = make_config("cfg4_finegrained", T=T, H=H, F=F, E=12, k=3, S=1, n_local=7,
                      bias_group_tokens=0)
    inp = make_inputs(cfg)
    err = check_layer(cfg, run_layer(cfg, inp), oracle_layer(inp))
    print(f"T={T} H={H} F={F}: out err {err:.3g}")


@pytest.mark.parametrize("T,F", [(40, 448), (700, 448), (400, 1024)])
def test_one_expert_takes_every_token(T, F):
    """A +1000 bias sends slot 0 of every token to expert 3: one group with T rows (several
    row tiles), the other hosted experts nearly empty."""
    cfg = make_config("cfg2_mixtral_prefill", T=T, H=256, F=F)
    inp = make_inputs(cfg)
    inp.bias[:, 3] += 1000.0
    inp.mask[3] = 1
    o = run_layer(cfg, inp)
    check_layer(cfg, o, oracle_layer(inp))
    assert int(o.counts[3]) == T and torch.all(o.topk_idx[:, 0] == 3)


def test_other_stream_accumulated_counts_and_stage_events():
    cfg = make_config("cfg5_dsv2lite_migration", T=300, H=128, F=192)
    inp = make_inputs(cfg)
    ref = oracle_layer(inp)
    desc = desc_of(cfg)
    ws = P.alloc_workspace(desc, cfg.T)
    wt = weight_table(inp)
    args = (desc, to_dev(inp.x), to_dev(inp.w_router), to_dev(inp.bias), wt, to_dev(inp.mask), ws)
    accum = torch.zeros(cfg.E, dtype=torch.int64, device="cuda")
    n_st = len(P.STAGES)
    events = [torch.cuda.Event(enable_timing=True) for _ in range(2 * n_st)]
    handles = (ctypes.c_void_p * (2 * n_st))()
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for i, ev in enumerate(events):
            ev.record()                      # materialise the hipEvent_t
            handles[i] = ev.cuda_event
        o = None
        for _ in range(3):
            o = P.prism_moe_layer(*args, counts_accum=accum, stream=side, stage_events=handles)
    side.synchronize()
    check_layer(cfg, o, ref)
    assert np.array_equal(accum.cpu().numpy(), 3 * ref.route.counts.astype(np.int64))
    # stages were recorded in launch order on that stream: every interval is >= 0
    for s in range(n_st):
        assert events[2 * s].elapsed_time(events[2 * s + 1]) >= 0.0
        if s:
            assert events[2 * s - 1].elapsed_time(events[2 * s]) >= 0.0


@pytest.mark.parametrize("T,H,F", [(20, 128, 192), (300, 128, 192), (300, 256, 1088)])
def test_workspace_sized_for_a_larger_batch(T, H, F):
    cfg = make_config("cfg4_finegrained", T=T, H=H, F=F, bias_group_tokens=64)
    inp = make_inputs(cfg)
    ws = P.alloc_workspace(desc_of(cfg), 2048)
    ws.fill_(0xA5)
    check_layer(cfg, run_layer(cfg, inp, ws=ws), oracle_layer(inp))


def test_unsupported_shapes_and_small_workspaces_are_refused_before_any_launch():
    with pytest.raises(P.PrismError, match="supported limits"):
        P.workspace_bytes(P.make_desc(96, 128, 8, 2, 0, "bf16"), 16)      # H % 64 != 0 (bf16 FFN)
    d = P.make_desc(128, 128, 8, 2, 0, "bf16")
    small = P.alloc_workspace(d, 4)
    bf = dict(dtype=torch.bfloat16, device="cuda")
    hosted = [tuple(torch.zeros(s, **bf) for s in ((128, 128), (128, 128), (128, 128)))] * 8
    with pytest.raises(P.PrismError, match="workspace too small"):
        P.prism_moe_layer(d, torch.zeros((4096, 128), **bf), torch.zeros((8, 128), **bf), None,
                          P.WeightTable(hosted, []), torch.ones(8, dtype=torch.uint8, device="cuda"),
                          small)


def test_debug_check_finds_a_hosted_expert_without_weights():
    cfg = make_config("cfg4_finegrained", T=16, H=128, F=192, bias_group_tokens=0)
    inp = make_inputs(cfg)
    desc = desc_of(cfg)
    mask = to_dev(inp.mask)
    P.prism_debug_check_weights(desc, weight_table(inp), mask)            # hosted ones are all there
    hosted = int(np.flatnonzero(inp.mask)[3])
    holes = inp.mask.copy()
    holes[hosted] = 0                                                     # table without that expert ...
    with pytest.raises(P.PrismError, match=f"expert {hosted}"):
        P.prism_debug_check_weights(desc, weight_table(inp, holes), mask)  # ... but the mask hosts it
    P.prism_debug_check_weights(desc, weight_table(inp, holes), to_dev(holes))


@pytest.mark.parametrize("T,H,F", [(2500, 128, 192), (300, 256, 1088)])
def test_prefill_layer_graph_replay_equals_eager(T, H, F):
    """A prefill layer (staged router, two-launch dispatch with the schedule workgroups, both GEMMs,
    combine) and one of a few hundred tokens (single dispatch workgroup, schedule launch, split down
    projection, slice-summing combine) captured in a graph and replayed with the workspace and
    outputs poisoned in between give the eager result every time: the library allocates nothing
    and needs no memset node."""
    cfg = make_config("cfg4_finegrained", T=T, H=H, F=F, bias_group_tokens=512)
    inp = make_inputs(cfg)
    desc = desc_of(cfg)
    ws = P.alloc_workspace(desc, cfg.T)
    out = P.alloc_layer_out(desc, cfg.T)
    wt = weight_table(inp)
    x, wr, b, m = to_dev(inp.x), to_dev(inp.w_router), to_dev(inp.bias), to_dev(inp.mask)
    P.prism_moe_layer(desc, x, wr, b, wt, m, ws, out)
    torch.cuda.synchronize()
    eager = {k: getattr(out, k).clone() for k in ("out", "topk_idx", "counts", "remote_src", "remote_bytes")}
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            P.prism_moe_layer(desc, x, wr, b, wt, m, ws, out, stream=side)
    torch.cuda.synchronize()
    for i in range(3):
        out.out.fill_(float("nan"))
        out.counts.fill_(-1)
        out.remote_src.fill_(-7)
        ws.fill_(0x7F)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        nr = int(out.n_local_remote[1])
        assert torch.equal(out.out, eager["out"]) and torch.equal(out.topk_idx, eager["topk_idx"]), i
        assert torch.equal(out.counts, eager["counts"]) and torch.equal(out.remote_bytes, eager["remote_bytes"])
        assert torch.equal(out.remote_src[:nr], eager["remote_src"][:nr])


@pytest.mark.parametrize("T,S", [(37, 0), (333, 2), (901, 1)])
def test_expert_ffn_with_local_src_at_the_very_end_of_its_allocation(T, S):
    """prism_expert_ffn is handed a local_src of exactly T*k ints (T*k odd, so its last 16-byte
    piece is cut short) that ends where its allocation ends: the kernel's prefetch of a row
    tile's source rows must neither depend on anything past that end nor change a result.
    Shared-expert tiles (S > 0) take no source rows at all."""
    from oracle import prism_oracle as O

    from gpu_util import TOL, rel_err, to_f32

    cfg = make_config("cfg4_finegrained", T=T, H=256, F=448, E=6, k=3, S=S, n_local=4,
                      bias_group_tokens=0)
    inp = make_inputs(cfg)
    f = inp.f32
    desc = desc_of(cfg)
    ws = P.alloc_workspace(desc, cfg.T)
    r = O.route(f(inp.x), f(inp.w_router), inp.bias, cfg.k, cfg.bias_group_tokens)
    d = O.dispatch(r.topk_idx, inp.mask, cfg.H, cfg.es)
    A = cfg.A
    assert A % 4 != 0
    src = np.full(A, -1, np.int32)
    src[:d.n_local] = d.local_src
    # the list occupies the last A ints of a larger buffer whose front is poisoned
    buf = torch.full((4096 + A,), 0x7FFFFFF0, dtype=torch.int32, device="cuda")
    tail = buf[4096:]
    tail.copy_(torch.from_numpy(src))
    offsets = to_dev(d.local_offsets)
    wt = weight_table(inp)
    x = to_dev(inp.x)
    y_tail = P.prism_expert_ffn(desc, x, wt, tail, offsets, ws)
    y_plain = P.prism_expert_ffn(desc, x, wt, to_dev(src), offsets, ws)
    torch.cuda.synchronize()
    assert torch.equal(y_tail, y_plain)
    y_ref = O.expert_ffn(f(inp.x), lambda e: tuple(f(w) for w in inp.expert(e)),
                         [tuple(f(w) for w in inp.shared(s)) for s in range(S)], d.local_src,
                         d.local_offsets, cfg.k)
    got = to_f32(y_tail)
    assert rel_err(np.concatenate([got[:d.n_local], got[A:]]), y_ref) <= TOL[cfg.dtype]


@pytest.mark.parametrize("T,H,F,E,n_local", [(513, 128, 4096, 8, 5), (700, 256, 4160, 8, 5), (1100, 512, 4096, 4, 3),
                                               (2300, 256, 4096, 2, 2), (900, 768, 5120, 16, 9),
                                               (600, 256, 4032, 8, 5)])
def test_prefill_batches_whose_last_round_of_the_down_projection_is_cut(T, H, F, E, n_local):
    """More than 512 tokens of a layer with a long down-projection contraction (F >= 4096; the last
    case is just below and takes the plain path): the
    items of the partly filled last round are cut along the contraction into slice entries, run
    by a launch of their own and summed in slice order.  Row-major and tiled weights."""
    cfg = make_config("cfg2_mixtral_prefill", T=T, H=H, F=F, E=E, k=2, n_local=n_local)
    inp = make_inputs(cfg)
    ref = oracle_layer(inp)
    for tiled in (False, True):
        o = run_layer(cfg, inp, wt=weight_table(inp, tiled=tiled), weight_layout="tiled" if tiled else "row_major")
        err = check_layer(cfg, o, ref)
        print(f"T={T} H={H} F={F} tiled={tiled}: out err {err:.3g}")
