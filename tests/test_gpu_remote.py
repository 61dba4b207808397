"""The remote call end to end on one GPU: the requesting server's layer, the rows it ships
(prism_pack_remote), the hosting side's grouped FFN on the shipped rows (prism_expert_ffn with
one slot per row and no shared experts), and the aggregation of the returned rows
(prism_combine_remote).  Local partial + returned rows must give the layer with every expert
hosted."""
import numpy as np
import pytest
import torch

import paper_2508_12851_amd as P
from oracle import prism_oracle as O
from prism_inputs import make_config, make_inputs

from gpu_util import TOL, check_layer, desc_of, oracle_layer, rel_err, run_layer, to_dev, to_f32, weight_table

pytestmark = pytest.mark.gpu

CASES = {
    "tiny_f32": dict(name="cfg1_tiny_f32"),
    "mixtral_small": dict(name="cfg2_mixtral_prefill", T=333, H=256, F=448),
    "mixtral_decode": dict(name="cfg3_mixtral_decode", T=32, H=256, F=448),
    "finegrained_small": dict(name="cfg4_finegrained", T=700, H=128, F=192, bias_group_tokens=128),
    "dsv2_small": dict(name="cfg5_dsv2lite_migration", T=515, H=128, F=192),
}


@pytest.mark.parametrize("case", list(CASES))
def test_remote_call_completes_the_layer(case):
    kw = dict(CASES[case])
    cfg = make_config(kw.pop("name"), **kw)
    inp = make_inputs(cfg)
    f = inp.f32
    desc = desc_of(cfg)
    ws = P.alloc_workspace(desc, cfg.T)
    wt_all = weight_table(inp, all_experts=True)
    x = to_dev(inp.x)

    # requesting server: local partial sum and the remote list
    part_ref = oracle_layer(inp)
    o = run_layer(cfg, inp, wt=wt_all, ws=ws)
    check_layer(cfg, o, part_ref)
    R = int(o.n_local_remote[1])
    assert R == part_ref.dispatch.n_remote and R > 0

    # rows it ships: bit-exact copies of the remote assignments' tokens
    packed = P.prism_pack_remote(desc, x, o.remote_src, o.remote_offsets)
    torch.cuda.synchronize()
    shipped_ref = O.pack_remote(inp.x, part_ref.dispatch.remote_src, cfg.k)
    got = packed.view(torch.int16).cpu().numpy().view(np.uint16) if cfg.dtype == "bf16" \
        else packed.cpu().numpy()
    assert np.array_equal(got[:R], shipped_ref)
    assert not got[R:].any()

    # hosting side: grouped FFN over the shipped rows, one slot per row, no shared experts
    peer = P.make_desc(cfg.H, cfg.F, cfg.E, 1, 0, cfg.dtype)
    ws_peer = P.alloc_workspace(peer, R)
    rows = torch.arange(R, dtype=torch.int32, device="cuda")
    y_remote = P.prism_expert_ffn(peer, packed[:R].contiguous(), wt_all, rows, o.remote_offsets, ws_peer)
    torch.cuda.synchronize()
    experts = lambda e: tuple(f(w) for w in inp.expert(e))
    y_ref = O.expert_ffn(f(inp.x), experts, [], part_ref.dispatch.remote_src,
                         part_ref.dispatch.remote_offsets, cfg.k)
    assert rel_err(to_f32(y_remote), y_ref) <= TOL[cfg.dtype]

    # requesting server again: add the returned rows to the local partial sum
    out = o.out.clone()
    P.prism_combine_remote(desc, y_remote, o.remote_src, o.remote_offsets, o.topk_gate, out, ws)
    torch.cuda.synchronize()
    done_ref = O.combine_remote(part_ref.out, y_ref, part_ref.dispatch.remote_src,
                                part_ref.route.topk_gate, cfg.dtype)
    err = rel_err(to_f32(out), done_ref)
    assert err <= TOL[cfg.dtype], err
    # = the layer with every expert hosted, computed in one go (one rounding fewer)
    ones = np.ones(cfg.E, np.uint8)
    full_ref = oracle_layer(inp, ones)
    full = run_layer(cfg, inp, mask=ones, wt=wt_all, ws=ws)
    assert rel_err(to_f32(out), full_ref.out) <= 1.5 * TOL[cfg.dtype]
    assert rel_err(to_f32(out), to_f32(full.out)) <= 1.5 * TOL[cfg.dtype]
    print(f"{case}: R={R}, completed-layer err {err:.3g}")


def test_nothing_remote_leaves_out_untouched():
    cfg = make_config("cfg2_mixtral_prefill", T=100, H=128, F=128)
    inp = make_inputs(cfg)
    desc = desc_of(cfg)
    ws = P.alloc_workspace(desc, cfg.T)
    ones = np.ones(cfg.E, np.uint8)
    o = run_layer(cfg, inp, mask=ones, wt=weight_table(inp, all_experts=True), ws=ws)
    assert o.n_local_remote.cpu().tolist() == [cfg.A, 0]
    before = o.out.clone()
    y_none = torch.zeros((1, cfg.H), dtype=torch.bfloat16, device="cuda")
    P.prism_combine_remote(desc, y_none, o.remote_src, o.remote_offsets, o.topk_gate, o.out, ws)
    packed = P.prism_pack_remote(desc, to_dev(inp.x), o.remote_src, o.remote_offsets)
    torch.cuda.synchronize()
    assert torch.equal(o.out, before) and not packed.any()
