"""Helpers shared by the GPU parity tests: upload seeded inputs, run the oracle."""
import numpy as np
import torch

import paper_2508_12851_amd as P
from oracle import prism_oracle as O


def to_dev(a: np.ndarray) -> torch.Tensor:
    """numpy -> device tensor; uint16 arrays are bf16 bit patterns."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def desc_of(cfg, gate_mode="renormalized", weight_layout="row_major"):
    return P.make_desc(cfg.H, cfg.F, cfg.E, cfg.k, cfg.S, cfg.dtype, cfg.bias_group_tokens, gate_mode,
                       weight_layout)


def weight_table(inp, mask=None, all_experts=False, tiled=False):
    """Upload hosted experts (None for the others) and the shared experts; tiled: re-laid
    into 16 x 32 tiles by the library's own pack kernel."""
    c = inp.cfg
    mask = inp.mask if mask is None else mask
    up = (lambda w: P.prism_pack_weights(to_dev(w))) if tiled else to_dev
    experts = []
    for e in range(c.E):
        if all_experts or mask[e]:
            experts.append(tuple(up(w) for w in inp.expert(e)))
        else:
            experts.append(None)
    shared = [tuple(up(w) for w in inp.shared(s)) for s in range(c.S)]
    return P.WeightTable(experts, shared)


def oracle_layer(inp, mask=None, x=None, token_pos=None, renormalize=True):
    c = inp.cfg
    f = inp.f32
    return O.moe_layer(f(inp.x) if x is None else x, f(inp.w_router), inp.bias,
                       lambda e: tuple(f(w) for w in inp.expert(e)),
                       [tuple(f(w) for w in inp.shared(s)) for s in range(c.S)],
                       inp.mask if mask is None else mask, c.k, c.dtype, c.bias_group_tokens,
                       token_pos, renormalize)


def rel_err(a, ref, per_row=False):
    """max |a - ref| / (|ref| + rms(ref)): the layer-output error measure.  per_row: the rms of
    the element's own row (token) instead of the whole array -- for batches whose tokens differ
    widely in magnitude (a zero row of ref then demands an exactly zero row of a)."""
    a = np.asarray(a, np.float64)
    ref = np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0
    if per_row:
        rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
    else:
        rms = np.sqrt(np.mean(ref ** 2))
    diff = np.abs(a - ref)
    return float(np.max(np.where(diff == 0, 0.0, diff / (np.abs(ref) + rms + 1e-300))))


TOL = {"f32": 1e-4, "bf16": 2e-2}


def run_layer(cfg, inp, mask=None, wt=None, ws=None, gate_mode="renormalized",
              weight_layout="row_major", **kw):
    desc = desc_of(cfg, gate_mode, weight_layout)
    ws = P.alloc_workspace(desc, cfg.T) if ws is None else ws
    mask = inp.mask if mask is None else mask
    wt = weight_table(inp, mask) if wt is None else wt
    o = P.prism_moe_layer(desc, to_dev(inp.x), to_dev(inp.w_router), to_dev(inp.bias), wt,
                          to_dev(mask), ws, **kw)
    # the permutation the layer call itself built (it lives in the workspace)
    o.perm = P.prism_layer_permutation(desc, cfg.T, ws, stream=kw.get("stream"))
    torch.cuda.synchronize()
    return o


def check_permutation(perm, dispatch_ref, A):
    """local_src / local_offsets / inverse of a layer call, bit for bit against oracle.dispatch."""
    nl = dispatch_ref.n_local
    assert np.array_equal(perm.local_offsets.cpu().numpy(), dispatch_ref.local_offsets)
    assert np.array_equal(perm.local_src.cpu().numpy()[:nl], dispatch_ref.local_src)
    inv = np.full(A, -1, dtype=np.int32)
    inv[dispatch_ref.local_src] = np.arange(nl, dtype=np.int32)
    assert np.array_equal(perm.inv.cpu().numpy(), inv)


def check_layer(cfg, o, ref, per_row=False):
    """Integer outputs bit-exact, gates to 1e-6, layer output within the dtype's tolerance."""
    nl, nr = o.n_local_remote.cpu().tolist()
    assert np.array_equal(o.topk_idx.cpu().numpy(), ref.route.topk_idx)
    assert np.array_equal(o.counts.cpu().numpy(), ref.route.counts)
    assert np.max(np.abs(o.topk_gate.cpu().numpy() - ref.route.topk_gate), initial=0.0) <= 1e-6
    assert (nl, nr) == (ref.dispatch.n_local, ref.dispatch.n_remote)
    assert np.array_equal(o.remote_src.cpu().numpy()[:nr], ref.dispatch.remote_src)
    assert np.array_equal(o.remote_offsets.cpu().numpy(), ref.dispatch.remote_offsets)
    assert np.array_equal(o.remote_bytes.cpu().numpy(), ref.dispatch.remote_bytes)
    if getattr(o, "perm", None) is not None:
        check_permutation(o.perm, ref.dispatch, cfg.A)
    err = rel_err(to_f32(o.out), ref.out, per_row)
    assert err <= TOL[cfg.dtype], err
    return err
