"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Every output of the layer is compared with the oracle for EVERY token: routing, counts, the
local / remote split, the permutation the layer call builds (read back from its workspace),
the remote list and its byte counts bit for bit, the gates to 1e-6, and the layer output
element by element within the bf16 bar.  Each workload runs with the expert weights in the
16 x 32 tiles bench.py uses and with row-major weights, against one oracle result.
"""
import time

import numpy as np
import pytest
import torch

import paper_2508_12851_amd as P
from prism_inputs import CONFIGS, make_config, make_inputs

from gpu_util import TOL, check_permutation, desc_of, oracle_layer, rel_err, to_dev, to_f32, weight_table

pytestmark = pytest.mark.gpu

LAYOUTS = ("tiled", "row_major")


def _run(cfg, inp, layout):
    desc = desc_of(cfg, weight_layout=layout)
    ws = P.alloc_workspace(desc, cfg.T)
    wt = weight_table(inp, tiled=layout == "tiled")
    o = P.prism_moe_layer(desc, to_dev(inp.x), to_dev(inp.w_router), to_dev(inp.bias), wt,
                          to_dev(inp.mask), ws)
    o.perm = P.prism_layer_permutation(desc, cfg.T, ws)
    torch.cuda.synchronize()
    return o


def _check_all(cfg, inp, o, ref):
    """Every output of one layer call against the oracle's result for the whole batch."""
    r, d = ref.route, ref.dispatch
    assert np.array_equal(o.topk_idx.cpu().numpy(), r.topk_idx)
    assert np.array_equal(o.counts.cpu().numpy(), r.counts)
    assert int(o.counts.sum()) == cfg.T * cfg.k
    gate = o.topk_gate.cpu().numpy()
    assert np.max(np.abs(gate - r.topk_gate)) <= 1e-6
    assert np.max(np.abs(gate.astype(np.float64).sum(axis=1) - 1.0)) <= 1e-6
    nl, nr = o.n_local_remote.cpu().tolist()
    assert (nl, nr) == (d.n_local, d.n_remote) and nl + nr == cfg.A
    assert nr == int(r.counts[inp.mask == 0].sum())            # Eq. 2 with raw f, one server/layer
    assert np.array_equal(o.remote_src.cpu().numpy()[:nr], d.remote_src)
    assert np.array_equal(o.remote_offsets.cpu().numpy(), d.remote_offsets)
    assert o.remote_bytes.cpu().tolist() == [nr * cfg.H * cfg.es] * 2
    check_permutation(o.perm, d, cfg.A)
    got = to_f32(o.out)
    assert got.shape == ref.out.shape == (cfg.T, cfg.H)
    assert np.all(np.isfinite(got))
    err = rel_err(got, ref.out)                                # every token, every element
    assert err <= TOL[cfg.dtype], err
    if cfg.S == 0:   # tokens with no local slot and no shared expert must be exactly zero
        no_local = ~np.any(inp.mask[r.topk_idx] == 1, axis=1)
        assert np.all(got[no_local] == 0)
    return err


def _full_parity(cfg, inp, label, layouts=LAYOUTS):
    t0 = time.perf_counter()
    ref = oracle_layer(inp)                                    # all cfg.T tokens
    dt = time.perf_counter() - t0
    outs = {}
    for layout in layouts:
        o = _run(cfg, inp, layout)
        err = _check_all(cfg, inp, o, ref)
        outs[layout] = o
        print(f"{label} [{layout}]: all {cfg.T} tokens, out err {err:.3g} (oracle {dt:.1f} s)", flush=True)
    return ref, outs


def test_cfg2_mixtral_prefill_full_size():
    cfg = CONFIGS["cfg2_mixtral_prefill"]
    inp = make_inputs(cfg, weights="local", threads=16)
    _, outs = _full_parity(cfg, inp, "cfg2")
    # the prefill kernels form every sum in the same order in both layouts
    assert torch.equal(outs["tiled"].out, outs["row_major"].out)


def test_cfg3_mixtral_decode_full_size():
    cfg = CONFIGS["cfg3_mixtral_decode"]
    inp = make_inputs(cfg, weights="local", threads=16)
    _full_parity(cfg, inp, "cfg3")


@pytest.mark.parametrize("n_local", [1, 3, 8])
def test_mixtral_decode_with_other_numbers_of_hosted_experts(n_local):
    """The decode batch with 1, 3 and all 8 experts hosted: the schedule builder splits the down
    projection's contraction into a number of slices that depends on how many experts received
    tokens (from one workgroup per item to eight)."""
    cfg = make_config("cfg3_mixtral_decode", n_local=n_local)
    inp = make_inputs(cfg, weights="local", threads=16)
    _full_parity(cfg, inp, f"Mixtral decode, {n_local} hosted", layouts=("tiled",))


@pytest.mark.parametrize("T", [96, 128, 200, 300, 512, 1024, 1536, 2048])
def test_mixtral_shape_other_batch_sizes_full_size(T):
    """The full Mixtral layer shape between the decode and the benchmark batch: 128 x 128 tiles
    up to 256 tokens (one row tile per expert up to 128, two for the popular experts at 200),
    128 x 256 tiles up to 352, both with the split down projection; prefill tiles whose last
    round of work items is only partly filled above."""
    cfg = make_config("cfg2_mixtral_prefill", T=T)
    inp = make_inputs(cfg, weights="local", threads=16)
    _full_parity(cfg, inp, f"Mixtral shape, {T} tokens", layouts=("tiled",))


def test_cfg4_finegrained_full_size():
    cfg = CONFIGS["cfg4_finegrained"]
    inp = make_inputs(cfg, weights="local", threads=16)
    _full_parity(cfg, inp, "cfg4")


def test_cfg5_migration_full_size_both_phases():
    cfg = CONFIGS["cfg5_dsv2lite_migration"]
    ratios = []
    for phase in (0, 1):
        inp = make_inputs(cfg, phase=phase, weights="local", threads=16)
        ref, _ = _full_parity(cfg, inp, f"cfg5 phase {phase}")
        ratios.append(ref.dispatch.n_local / cfg.A)
        print(f"cfg5 phase {phase}: local ratio {ratios[-1]:.3f}")
    # keeping the phase-0 mask for phase-1 traffic lowers the local compute ratio (Fig. 6a analogue)
    p0 = make_inputs(cfg, phase=0)
    p1 = make_inputs(cfg, phase=1, weights="all", threads=16)
    desc = desc_of(cfg)
    ws = P.alloc_workspace(desc, cfg.T)
    stale = P.prism_moe_layer(desc, to_dev(p1.x), to_dev(p1.w_router), to_dev(p1.bias),
                              weight_table(p1, all_experts=True), to_dev(p0.mask), ws)
    torch.cuda.synchronize()
    assert int(stale.n_local_remote[0]) / cfg.A < ratios[1]


def test_large_ragged_batch():
    """Many more tokens than any benchmark config (79 dispatch chunks, ~800 row tiles, a
    ragged last tile everywhere), every token against the oracle."""
    cfg = make_config("cfg4_finegrained", T=40001, H=512, F=640, E=32, k=4, S=1, n_local=19,
                      bias_group_tokens=4096)
    inp = make_inputs(cfg, weights="local", threads=16)
    _full_parity(cfg, inp, "large ragged batch")


def test_cfg2_full_size_properties_that_hold_at_any_size():
    """Without the oracle: local partial + remote partial = the layer with every expert hosted
    (Sec. III-A: what the hosting servers return is added to the local partial sum), and
    permuting the tokens permutes the outputs and leaves the activation counts unchanged."""
    cfg = CONFIGS["cfg2_mixtral_prefill"]
    inp = make_inputs(cfg, weights="all", threads=16)
    desc = desc_of(cfg)
    ws = P.alloc_workspace(desc, cfg.T)
    wt = weight_table(inp, all_experts=True)
    x, w_r, bias = to_dev(inp.x), to_dev(inp.w_router), to_dev(inp.bias)

    def run(xx, mask):
        o = P.prism_moe_layer(desc, xx, w_r, bias, wt, to_dev(mask), ws)
        torch.cuda.synchronize()
        return o

    ones = np.ones(cfg.E, np.uint8)
    local, remote, full = run(x, inp.mask), run(x, 1 - inp.mask), run(x, ones)
    assert torch.equal(local.topk_idx, full.topk_idx) and torch.equal(local.counts, full.counts)
    assert int(local.n_local_remote[0]) == int(remote.n_local_remote[1])
    assert full.n_local_remote.cpu().tolist() == [cfg.A, 0]
    summed = to_f32(local.out).astype(np.float64) + to_f32(remote.out)
    assert rel_err(summed, to_f32(full.out)) <= 2 * TOL[cfg.dtype]

    perm = torch.from_numpy(np.random.default_rng(12).permutation(cfg.T)).cuda()
    shuffled = run(x[perm].contiguous(), inp.mask)
    assert torch.equal(shuffled.counts, local.counts)
    assert torch.equal(shuffled.topk_idx, local.topk_idx[perm])
    assert torch.equal(shuffled.topk_gate, local.topk_gate[perm])
    assert shuffled.n_local_remote.cpu().tolist() == local.n_local_remote.cpu().tolist()
    # rows meet other rows in the MFMA tiles, but every row's sums are formed in the same order
    assert rel_err(to_f32(shuffled.out), to_f32(local.out[perm])) <= 1e-6
