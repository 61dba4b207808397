"""GPU parity of the whole layer on seeded random layer shapes, batch sizes, masks, gate
conventions and weight layouts (all within the documented limits): what the hand-picked cases
of the other files might miss.  Every case prints its parameters before it runs.

The output error is max |a - ref| / (|ref| + rms(ref)) with the rms of the whole batch, for every
stage of every case but one: the layer output of the cases in random_cases.PER_ROW_CASES is
measured against the rms of the token's own row, because the bf16 roundings the layer is defined
with exceed the bar against the batch rms there in exact arithmetic (shown on the CPU by
tests/test_error_measure.py, which also shows that no other case needs it)."""
import numpy as np
import pytest

from prism_inputs import make_config, make_inputs
from random_cases import N_CASES, PER_ROW_CASES, draw_case

from gpu_util import check_layer, oracle_layer, run_layer, weight_table

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("i", range(N_CASES))
def test_layer_parity_on_a_random_shape(i):
    kw, gate_mode, tiled = draw_case(i)
    print(f"case {i}: {kw} gates={gate_mode} tiled={tiled}", flush=True)
    cfg = make_config("cfg4_finegrained", **kw)
    inp = make_inputs(cfg)
    ref = oracle_layer(inp, renormalize=gate_mode == "renormalized")
    o = run_layer(cfg, inp, wt=weight_table(inp, tiled=tiled), gate_mode=gate_mode,
                  weight_layout="tiled" if tiled else "row_major")
    err = check_layer(cfg, o, ref, per_row=i in PER_ROW_CASES)
    print(f"case {i}: out err {err:.3g}, n_local {ref.dispatch.n_local}, n_remote {ref.dispatch.n_remote}")


@pytest.mark.parametrize("i", range(0, N_CASES, 2))
def test_separate_calls_parity_on_a_random_shape(i):
    """The same shapes through prism_route, prism_dispatch, prism_expert_ffn, prism_combine,
    prism_pack_remote and prism_combine_remote one by one, each against its oracle function."""
    import torch

    import paper_2508_12851_amd as P
    from oracle import prism_oracle as O

    from gpu_util import TOL, desc_of, rel_err, to_dev, to_f32

    kw, gate_mode, tiled = draw_case(i)
    print(f"case {i}: {kw} gates={gate_mode} tiled={tiled}", flush=True)
    cfg = make_config("cfg4_finegrained", **kw)
    inp = make_inputs(cfg)
    f = inp.f32
    desc = desc_of(cfg, gate_mode, "tiled" if tiled else "row_major")
    ws = P.alloc_workspace(desc, cfg.T)
    x = to_dev(inp.x)

    r_ref = O.route(f(inp.x), f(inp.w_router), inp.bias, cfg.k, cfg.bias_group_tokens,
                    renormalize=gate_mode == "renormalized")
    r = P.prism_route(desc, x, to_dev(inp.w_router), to_dev(inp.bias))
    assert np.array_equal(r.topk_idx.cpu().numpy(), r_ref.topk_idx)
    assert np.array_equal(r.counts.cpu().numpy(), r_ref.counts)
    assert np.max(np.abs(r.topk_gate.cpu().numpy() - r_ref.topk_gate), initial=0.0) <= 1e-6

    d_ref = O.dispatch(r_ref.topk_idx, inp.mask, cfg.H, cfg.es)
    d = P.prism_dispatch(desc, r.topk_idx, to_dev(inp.mask), ws)
    nl, nr = d.n_local_remote.cpu().tolist()
    assert (nl, nr) == (d_ref.n_local, d_ref.n_remote)
    assert np.array_equal(d.local_src.cpu().numpy()[:nl], d_ref.local_src)
    assert np.array_equal(d.remote_src.cpu().numpy()[:nr], d_ref.remote_src)
    assert np.array_equal(d.local_offsets.cpu().numpy(), d_ref.local_offsets)
    assert np.array_equal(d.remote_offsets.cpu().numpy(), d_ref.remote_offsets)
    assert np.array_equal(d.remote_bytes.cpu().numpy(), d_ref.remote_bytes)

    wt = weight_table(inp, all_experts=True, tiled=tiled)
    experts = lambda e: tuple(f(w) for w in inp.expert(e))
    shared = [tuple(f(w) for w in inp.shared(s)) for s in range(cfg.S)]
    y_ref = O.expert_ffn(f(inp.x), experts, shared, d_ref.local_src, d_ref.local_offsets, cfg.k)
    y = P.prism_expert_ffn(desc, x, wt, d.local_src, d.local_offsets, ws)
    torch.cuda.synchronize()
    yg = to_f32(y)
    y_got = np.concatenate([yg[:nl], yg[cfg.A:]])                 # shared rows start at T*k
    assert rel_err(y_got, y_ref) <= TOL[cfg.dtype]

    out_ref = O.combine(y_ref, d_ref.local_src, r_ref.topk_gate, cfg.T, cfg.S, cfg.dtype)
    out = P.prism_combine(desc, y, d.local_src, d.local_offsets, r.topk_gate, ws)
    torch.cuda.synchronize()
    assert rel_err(to_f32(out), out_ref, per_row=i in PER_ROW_CASES) <= TOL[cfg.dtype]

    # the remote call: ship, execute on a peer that hosts everything, add the returned rows
    packed = P.prism_pack_remote(desc, x, d.remote_src, d.remote_offsets)
    torch.cuda.synchronize()
    got = packed.view(torch.int16).cpu().numpy().view(np.uint16) if cfg.dtype == "bf16" \
        else packed.cpu().numpy()
    assert np.array_equal(got[:nr], O.pack_remote(inp.x, d_ref.remote_src, cfg.k))
    if nr > 0:
        peer = P.make_desc(cfg.H, cfg.F, cfg.E, 1, 0, cfg.dtype,
                           weight_layout="tiled" if tiled else "row_major")
        rows = torch.arange(nr, dtype=torch.int32, device="cuda")
        y_rem = P.prism_expert_ffn(peer, packed[:nr].contiguous(), wt, rows, d.remote_offsets,
                                   P.alloc_workspace(peer, nr))
        y_rem_ref = O.expert_ffn(f(inp.x), experts, [], d_ref.remote_src, d_ref.remote_offsets, cfg.k)
        assert rel_err(to_f32(y_rem), y_rem_ref) <= TOL[cfg.dtype]
        P.prism_combine_remote(desc, y_rem, d.remote_src, d.remote_offsets, r.topk_gate, out, ws)
        torch.cuda.synchronize()
        done_ref = O.combine_remote(out_ref, y_rem_ref, d_ref.remote_src, r_ref.topk_gate, cfg.dtype)
        err = rel_err(to_f32(out), done_ref)
        assert err <= 1.5 * TOL[cfg.dtype], err                   # one more bf16 rounding on the way
    print(f"case {i}: n_local {nl}, n_remote {nr}: all stages agree")


@pytest.mark.parametrize("i", range(12))
def test_layer_parity_on_a_random_wide_shape(i):
    """Prefill batches whose down projection may have its last round of items cut along the
    contraction (F >= 4096): whole layer against the oracle, whole-batch error measure."""
    from random_cases import draw_wide_case
    kw, tiled = draw_wide_case(i)
    print(f"wide case {i}: {kw} tiled={tiled}", flush=True)
    cfg = make_config("cfg2_mixtral_prefill", **kw)
    inp = make_inputs(cfg)
    ref = oracle_layer(inp)
    o = run_layer(cfg, inp, wt=weight_table(inp, tiled=tiled), weight_layout="tiled" if tiled else "row_major")
    err = check_layer(cfg, o, ref)
    print(f"wide case {i}: out err {err:.3g}, n_local {ref.dispatch.n_local}, n_remote {ref.dispatch.n_remote}")


@pytest.mark.parametrize("i", range(24))
def test_layer_parity_on_a_random_streaming_shape(i):
    """Batches of 1 to 352 tokens of wide layers, where the expert FFN streams the weights once and
    splits the down projection's contraction by a count chosen on the device: whole layer against
    the oracle, whole-batch error measure."""
    from random_cases import draw_streaming_case
    kw, tiled = draw_streaming_case(i)
    print(f"streaming case {i}: {kw} tiled={tiled}", flush=True)
    cfg = make_config("cfg3_mixtral_decode", **kw)
    inp = make_inputs(cfg)
    ref = oracle_layer(inp)
    o = run_layer(cfg, inp, wt=weight_table(inp, tiled=tiled), weight_layout="tiled" if tiled else "row_major")
    err = check_layer(cfg, o, ref)
    print(f"streaming case {i}: out err {err:.3g}, n_local {ref.dispatch.n_local}, n_remote {ref.dispatch.n_remote}")

