"""Pins for the CPU oracle: things the paper's definitions and plain mathematics fix.

The paper prints no worked numeric example of a layer forward, so the pins are
closed forms, brute force written differently, library routines on the special
cases that reduce to them, and the invariants that follow from the local /
remote indicator (Sec. III-B), the aggregation of local and remote results
(Sec. III-A), the proxy objective (Eq. 2) and the local compute ratio (Sec. IV,
Fig. 5).
"""
import numpy as np
import pytest
import torch

from oracle import prism_oracle as O
from prism_inputs import make_config, make_inputs


def _tiny(**kw):
    cfg = make_config("cfg1_tiny_f32", **kw)
    inp = make_inputs(cfg, weights="all")
    return cfg, inp


def _layer(inp, mask=None, k=None, dtype=None, x=None, token_pos=None, scale_down=1.0):
    c = inp.cfg
    f = inp.f32

    def experts(e):
        wg, wu, wd = inp.expert(e)
        return f(wg), f(wu), f(wd) * np.float32(scale_down)

    shared = []
    for s in range(c.S):
        wg, wu, wd = inp.shared(s)
        shared.append((f(wg), f(wu), f(wd) * np.float32(scale_down)))
    return O.moe_layer(f(inp.x) if x is None else x, f(inp.w_router), inp.bias, experts, shared,
                       inp.mask if mask is None else mask, c.k if k is None else k,
                       c.dtype if dtype is None else dtype, c.bias_group_tokens, token_pos)


# ---------------------------------------------------------------------------
# routing: brute force and closed forms
# ---------------------------------------------------------------------------

def _brute_route(x, w, bias_rows, k):
    """Full sort of all E logits per token with key (-logit, index); python loops."""
    T, H = x.shape
    E = w.shape[0]
    idx = np.zeros((T, k), dtype=np.int32)
    gate = np.zeros((T, k), dtype=np.float64)
    logits = np.zeros((T, E), dtype=np.float32)
    for t in range(T):
        lg = []
        for e in range(E):
            acc = 0.0
            for h in range(H):
                acc += float(x[t, h]) * float(w[e, h])
            v = np.float32(acc)
            if bias_rows is not None:
                v = np.float32(v + np.float32(bias_rows[t][e]))
            lg.append(v)
        logits[t] = lg
        order = sorted(range(E), key=lambda e: (-float(lg[e]), e))[:k]
        full = np.exp(np.array([float(v) for v in lg]) - max(float(v) for v in lg))
        full = full / full.sum()           # full softmax over all E experts ...
        sel = full[order]
        gate[t] = sel / sel.sum()          # ... renormalised over the k picked
        idx[t] = order
    return idx, gate, logits


def test_route_matches_brute_force_full_sort():
    rng = np.random.default_rng(11)
    T, H, E, k = 24, 40, 10, 3
    x = rng.standard_normal((T, H)).astype(np.float32)
    w = rng.standard_normal((E, H)).astype(np.float32) * 0.2
    bias = rng.standard_normal((3, E)).astype(np.float32)
    r = O.route(x, w, bias, k, bias_group_tokens=8)
    rows = [bias[t // 8] for t in range(T)]
    bidx, bgate, blogits = _brute_route(x, w, rows, k)
    assert np.array_equal(r.logits, blogits)           # same sum order: the same fp32 bits
    assert np.array_equal(r.topk_idx, bidx)
    assert np.max(np.abs(r.topk_gate - bgate)) < 1e-6


def test_route_k1_gate_is_exactly_one():
    cfg, inp = _tiny()
    r = O.route(inp.x, inp.w_router, inp.bias, 1)
    assert np.all(r.topk_gate == np.float32(1.0))
    assert np.array_equal(r.topk_idx[:, 0], np.argmax(r.logits, axis=1))


def test_route_k_equals_E_is_full_softmax():
    cfg, inp = _tiny()
    r = O.route(inp.x, inp.w_router, inp.bias, cfg.E)
    sm = torch.softmax(torch.from_numpy(r.logits).double(), dim=1).numpy()
    got = np.zeros_like(sm)
    for t in range(cfg.T):
        got[t, r.topk_idx[t]] = r.topk_gate[t]
    assert np.max(np.abs(got - sm)) < 1e-6
    # slots are in descending logit order
    sel = np.take_along_axis(r.logits, r.topk_idx.astype(np.int64), axis=1)
    assert np.all(sel[:, :-1] >= sel[:, 1:])


def test_route_zero_router_picks_first_k_with_equal_gates():
    T, H, E, k = 17, 32, 8, 4
    x = np.random.default_rng(0).standard_normal((T, H)).astype(np.float32)
    r = O.route(x, np.zeros((E, H), np.float32), None, k)
    assert np.array_equal(r.topk_idx, np.tile(np.arange(k, dtype=np.int32), (T, 1)))
    assert np.all(r.topk_gate == np.float32(1.0 / k))
    assert np.array_equal(r.counts, np.array([T] * k + [0] * (E - k), dtype=np.int32))


def test_route_duplicated_rows_tie_goes_to_lower_index():
    rng = np.random.default_rng(5)
    T, H, E = 50, 16, 6
    x = rng.standard_normal((T, H)).astype(np.float32)
    w = rng.standard_normal((E, H)).astype(np.float32)
    w[4] = w[1]                      # experts 1 and 4 always tie exactly
    r = O.route(x, w, None, 2)
    for t in range(T):
        row = list(r.topk_idx[t])
        if 4 in row:
            assert 1 in row and row.index(1) < row.index(4)
    # and the tie does occur as the top pair somewhere
    assert any(list(r.topk_idx[t]) == [1, 4] for t in range(T))
    tie = [t for t in range(T) if list(r.topk_idx[t]) == [1, 4]]
    assert np.all(r.topk_gate[tie] == np.float32(0.5))


def test_route_huge_bias_forces_slot0():
    cfg, inp = _tiny()
    bias = inp.bias.copy()
    bias[0, 6] += np.float32(1000.0)
    r = O.route(inp.x, inp.w_router, bias, 2)
    assert np.all(r.topk_idx[:, 0] == 6)
    assert np.all(r.topk_gate[:, 0] == np.float32(1.0))   # exp(-~1000) underflows in fp32 sum


def test_route_against_torch_topk_softmax_tie_free():
    rng = np.random.default_rng(3)
    T, H, E, k = 200, 64, 16, 4
    x = rng.standard_normal((T, H)).astype(np.float32)
    w = rng.standard_normal((E, H)).astype(np.float32) / 8
    r = O.route(x, w, None, k)
    lg = torch.from_numpy(r.logits)
    assert all(len(set(row.tolist())) == E for row in lg)     # no exact ties
    vals, idx = torch.topk(lg, k, dim=1)
    assert np.array_equal(r.topk_idx, idx.numpy().astype(np.int32))
    full = torch.softmax(lg.double(), dim=1)
    g = torch.gather(full, 1, idx)
    g = g / g.sum(dim=1, keepdim=True)
    assert np.max(np.abs(r.topk_gate - g.numpy())) < 1e-6
    # logits agree with a library matmul in a different precision path
    ref = (torch.from_numpy(x).double() @ torch.from_numpy(w).double().T).float().numpy()
    assert np.array_equal(r.logits, ref)


def test_route_bias_row_selection_uses_token_position():
    rng = np.random.default_rng(9)
    T, H, E = 12, 8, 5
    x = rng.standard_normal((T, H)).astype(np.float32)
    w = rng.standard_normal((E, H)).astype(np.float32)
    bias = np.zeros((3, E), np.float32)
    bias[1, 3] = 1000.0
    bias[2, 0] = 1000.0
    r = O.route(x, w, bias, 1, bias_group_tokens=4)
    assert np.all(r.topk_idx[4:8, 0] == 3) and np.all(r.topk_idx[8:12, 0] == 0)
    # a subset evaluated with explicit positions gives the same rows
    sub = np.array([9, 2, 5])
    rs = O.route(x[sub], w, bias, 1, bias_group_tokens=4, token_pos=sub)
    assert np.array_equal(rs.topk_idx, r.topk_idx[sub])
    assert np.array_equal(rs.logits, r.logits[sub])


def test_gates_sum_to_one_and_counts_sum_to_Tk():
    cfg, inp = _tiny()
    r = O.route(inp.x, inp.w_router, inp.bias, cfg.k)
    assert np.max(np.abs(r.topk_gate.astype(np.float64).sum(axis=1) - 1.0)) < 1e-6
    assert int(r.counts.sum()) == cfg.T * cfg.k
    assert np.array_equal(r.counts, np.bincount(r.topk_idx.reshape(-1), minlength=cfg.E))
    # every token picks k distinct experts
    assert all(len(set(row)) == cfg.k for row in r.topk_idx.tolist())


def test_counts_invariant_under_token_permutation():
    cfg, inp = _tiny()
    perm = np.random.default_rng(1).permutation(cfg.T)
    r0 = O.route(inp.x, inp.w_router, inp.bias, cfg.k)
    r1 = O.route(inp.x[perm], inp.w_router, inp.bias, cfg.k)
    assert np.array_equal(r0.counts, r1.counts)
    assert np.array_equal(r0.topk_idx[perm], r1.topk_idx)


# ---------------------------------------------------------------------------
# dispatch: partition, ordering, proxy objective, bytes
# ---------------------------------------------------------------------------

def _check_dispatch(idx, mask, d, H, es):
    A = idx.size
    E = len(mask)
    flat = idx.reshape(-1)
    both = np.concatenate([d.local_src, d.remote_src])
    assert np.array_equal(np.sort(both), np.arange(A))                 # partition
    assert d.local_offsets[0] == 0 and d.remote_offsets[0] == 0
    assert d.local_offsets[E] == d.n_local == len(d.local_src)
    assert d.remote_offsets[E] == d.n_remote == len(d.remote_src)
    for e in range(E):
        for src, off, hosted in ((d.local_src, d.local_offsets, True),
                                 (d.remote_src, d.remote_offsets, False)):
            seg = src[off[e]:off[e + 1]]
            assert np.all(flat[seg] == e)
            assert np.all(np.diff(seg) > 0)                            # strictly ascending
            if bool(mask[e]) != hosted:
                assert len(seg) == 0
    counts = np.bincount(flat, minlength=E)
    # Eq. 2 for one server and layer, with raw f: remote invocations
    assert d.n_remote == int(counts[np.asarray(mask) == 0].sum())
    assert np.array_equal(d.remote_bytes, np.array([d.n_remote * H * es] * 2))


def test_dispatch_partition_and_order_tiny_config():
    cfg, inp = _tiny()
    r = O.route(inp.x, inp.w_router, inp.bias, cfg.k)
    d = O.dispatch(r.topk_idx, inp.mask, cfg.H, cfg.es)
    _check_dispatch(r.topk_idx, inp.mask, d, cfg.H, cfg.es)
    ratio = d.n_local / (cfg.T * cfg.k)                               # local compute ratio
    assert ratio == r.counts[inp.mask == 1].sum() / (cfg.T * cfg.k)


def test_dispatch_hand_example():
    idx = np.array([[2, 0], [1, 2], [0, 3], [2, 1]], dtype=np.int32)   # T=4, k=2
    mask = np.array([1, 0, 1, 0], dtype=np.uint8)
    d = O.dispatch(idx, mask, hidden=8, elem_size=2)
    assert d.local_src.tolist() == [1, 4, 0, 3, 6]       # expert 0: a=1,4 ; expert 2: a=0,3,6
    assert d.local_offsets.tolist() == [0, 2, 2, 5, 5]
    assert d.remote_src.tolist() == [2, 7, 5]            # expert 1: a=2,7 ; expert 3: a=5
    assert d.remote_offsets.tolist() == [0, 0, 2, 2, 3]
    assert (d.n_local, d.n_remote) == (5, 3)
    assert d.remote_bytes.tolist() == [3 * 8 * 2, 3 * 8 * 2]


def test_dispatch_all_ones_and_all_zero_masks():
    cfg, inp = _tiny()
    r = O.route(inp.x, inp.w_router, inp.bias, cfg.k)
    ones = np.ones(cfg.E, np.uint8)
    d1 = O.dispatch(r.topk_idx, ones, cfg.H, cfg.es)
    assert d1.n_remote == 0 and d1.remote_bytes.tolist() == [0, 0] and d1.n_local == cfg.A
    d0 = O.dispatch(r.topk_idx, np.zeros(cfg.E, np.uint8), cfg.H, cfg.es)
    assert d0.n_local == 0 and d0.n_remote == cfg.A
    assert int(d0.remote_bytes.sum()) == 2 * cfg.T * cfg.k * cfg.H * cfg.es
    # with complementary masks local and remote lists swap roles
    assert np.array_equal(d1.local_src, d0.remote_src)
    assert np.array_equal(d1.local_offsets, d0.remote_offsets)


def test_dispatch_random_masks_many_experts():
    rng = np.random.default_rng(2)
    T, E, k = 300, 37, 5
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    for _ in range(4):
        mask = (rng.random(E) < 0.5).astype(np.uint8)
        _check_dispatch(idx, mask, O.dispatch(idx, mask, 64, 2), 64, 2)


# ---------------------------------------------------------------------------
# FFN + combine
# ---------------------------------------------------------------------------

def _dense_reference(inp, mask, dtype):
    """Dense MoE: every expert on every token, times a T x E gate matrix (torch CPU)."""
    c = inp.cfg
    r = O.route(inp.f32(inp.x), inp.f32(inp.w_router), inp.bias, c.k, c.bias_group_tokens)
    G = torch.zeros(c.T, c.E, dtype=torch.float64)
    for t in range(c.T):
        for j in range(c.k):
            e = int(r.topk_idx[t, j])
            if mask[e]:
                G[t, e] = float(r.topk_gate[t, j])
    x = torch.from_numpy(inp.f32(inp.x)).double()
    out = torch.zeros(c.T, c.H, dtype=torch.float64)

    def mlp(tri):
        wg, wu, wd = (torch.from_numpy(inp.f32(w)).double() for w in tri)
        return (torch.nn.functional.silu(x @ wg.T) * (x @ wu.T)) @ wd.T

    for e in range(c.E):
        out += G[:, e:e + 1] * mlp(inp.expert(e))
    for s in range(c.S):
        out += mlp(inp.shared(s))
    return out.numpy()


def _err(a, ref):
    a = np.asarray(a, np.float64)
    ref = np.asarray(ref, np.float64)
    return np.max(np.abs(a - ref) / (np.abs(ref) + np.sqrt(np.mean(ref ** 2))))


def test_all_local_mask_reproduces_dense_moe():
    cfg, inp = _tiny()
    ones = np.ones(cfg.E, np.uint8)
    res = _layer(inp, mask=ones)
    assert _err(res.out, _dense_reference(inp, ones, "f32")) < 1e-6


def test_partial_mask_matches_masked_dense_moe_with_shared_experts():
    cfg = make_config("cfg4_finegrained", T=40, H=64, F=96, E=12, k=3, S=2, n_local=7,
                      bias_group_tokens=16)
    inp = make_inputs(cfg, weights="all")
    res = _layer(inp, dtype="f32")
    assert 0 < res.dispatch.n_remote < cfg.A
    assert _err(res.out, _dense_reference(inp, inp.mask, "f32")) < 1e-6


def test_mask_complement_adds_up_to_full_layer():
    # local partial + remote partial = full layer ("transmitted back ... aggregated")
    cfg = make_config("cfg4_finegrained", T=32, H=64, F=96, E=12, k=3, S=2, n_local=7,
                      bias_group_tokens=16)
    inp = make_inputs(cfg, weights="all")
    ones = np.ones(cfg.E, np.uint8)
    a = _layer(inp, mask=inp.mask, dtype="f32").out.astype(np.float64)
    b = _layer(inp, mask=1 - inp.mask, dtype="f32").out.astype(np.float64)
    full = _layer(inp, mask=ones, dtype="f32").out.astype(np.float64)
    shared_once = _layer(inp, mask=np.zeros(cfg.E, np.uint8), dtype="f32").out.astype(np.float64)
    assert _err(a + b - shared_once, full) < 1e-5


def test_linearity_in_w_down_and_zero_w_down():
    cfg, inp = _tiny()
    base = _layer(inp).out.astype(np.float64)
    scaled = _layer(inp, scale_down=4.0).out.astype(np.float64)      # power of two: exact
    assert _err(scaled, 4.0 * base) < 1e-6
    assert np.all(_layer(inp, scale_down=0.0).out == 0)


def test_single_expert_is_plain_swiglu_mlp():
    cfg = make_config("cfg1_tiny_f32", T=9, H=32, F=48, E=1, k=1, mask_given=(0,), n_local=1)
    inp = make_inputs(cfg, weights="all")
    res = _layer(inp)
    x = torch.from_numpy(inp.x).double()
    wg, wu, wd = (torch.from_numpy(w).double() for w in inp.expert(0))
    ref = (torch.nn.functional.silu(x @ wg.T) * (x @ wu.T)) @ wd.T
    assert _err(res.out, ref.numpy()) < 1e-6
    assert np.all(res.route.topk_gate == 1.0)


def test_swiglu_rows_hand_value():
    # one row, H=2, F=1: g = 1*2 + 0*5 = 2, u = 3*2 + 1*5 = 11, h = silu(2)*11, y = [h*0.5, -h]
    y = O.swiglu_rows(np.array([[2.0, 5.0]]), np.array([[1.0, 0.0]]), np.array([[3.0, 1.0]]),
                      np.array([[0.5], [-1.0]]))
    h = (2.0 / (1.0 + np.exp(-2.0))) * 11.0
    assert np.allclose(y, [[0.5 * h, -h]], rtol=1e-14)


def test_token_permutation_equivariance_of_output():
    cfg, inp = _tiny()
    perm = np.random.default_rng(4).permutation(cfg.T)
    a = _layer(inp).out
    b = _layer(inp, x=inp.x[perm]).out
    assert _err(b, a[perm]) < 1e-6


def test_token_subset_with_positions_matches_full_run():
    cfg = make_config("cfg4_finegrained", T=48, H=64, F=96, E=12, k=3, S=1, n_local=7,
                      bias_group_tokens=16)
    inp = make_inputs(cfg, weights="all")
    full = _layer(inp).out
    sub = np.array([40, 3, 17, 22])
    part = _layer(inp, x=inp.f32(inp.x)[sub], token_pos=sub).out
    assert np.array_equal(part, full[sub])


def test_expert_rows_are_in_local_src_order():
    cfg, inp = _tiny()
    f = inp.f32
    r = O.route(inp.x, inp.w_router, inp.bias, cfg.k)
    d = O.dispatch(r.topk_idx, inp.mask, cfg.H, cfg.es)
    y = O.expert_ffn(inp.x, lambda e: inp.expert(e), [], d.local_src, d.local_offsets, cfg.k)
    for row in (0, d.n_local // 2, d.n_local - 1):
        a = int(d.local_src[row])
        e = int(r.topk_idx.reshape(-1)[a])
        ref = O.swiglu_rows(inp.x[a // cfg.k][None], *inp.expert(e))[0]
        assert np.allclose(y[row], ref, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------------------
# output rounding
# ---------------------------------------------------------------------------

def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(8)
    v = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 6, 5000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 257.0, 3.0e-5]])
    got = O.round_to_dtype(v, "bf16")
    ref = torch.from_numpy(v).to(torch.bfloat16).float().numpy()
    assert np.array_equal(got, ref)


def test_bf16_layer_output_is_bf16_representable():
    cfg = make_config("cfg4_finegrained", T=16, H=64, F=96, E=12, k=3, S=1, n_local=7,
                      bias_group_tokens=0)
    inp = make_inputs(cfg, weights="all")
    out = _layer(inp).out
    assert np.array_equal(out, torch.from_numpy(out).to(torch.bfloat16).float().numpy())


# ---------------------------------------------------------------------------
# the remote call: ship rows, execute on the hosting server, add the returned rows
# ---------------------------------------------------------------------------

def test_remote_call_completes_the_layer():
    """local partial + returned remote rows = the layer with every expert hosted (the dense
    reference), and the shipped rows are the tokens of the remote assignments."""
    rng = np.random.default_rng(21)
    T, H, E, F, k, S = 23, 16, 6, 24, 3, 1
    x = rng.standard_normal((T, H))
    w_r = rng.standard_normal((E, H)) / 4
    experts = [tuple(rng.standard_normal(s) / 4 for s in ((F, H), (F, H), (H, F))) for _ in range(E)]
    shared = [tuple(rng.standard_normal(s) / 4 for s in ((F, H), (F, H), (H, F))) for _ in range(S)]
    mask = np.array([1, 0, 1, 0, 0, 1], np.uint8)
    part = O.moe_layer(x, w_r, None, lambda e: experts[e], shared, mask, k, "f32")
    full = O.moe_layer(x, w_r, None, lambda e: experts[e], shared, np.ones(E, np.uint8), k, "f32")
    d = part.dispatch
    shipped = O.pack_remote(x, d.remote_src, k)
    assert shipped.shape == (d.n_remote, H)
    for r, a in enumerate(d.remote_src):
        assert np.array_equal(shipped[r], x[a // k])
    # hosting side: the same grouped FFN over the shipped rows (one slot per row, no shared experts)
    y_remote = O.expert_ffn(shipped, lambda e: experts[e], [], np.arange(d.n_remote),
                            d.remote_offsets, 1)
    # ... equals running it on the requester's tokens through the remote list itself
    y_direct = O.expert_ffn(x, lambda e: experts[e], [], d.remote_src, d.remote_offsets, k)
    assert np.allclose(y_remote, y_direct, rtol=0, atol=1e-12)
    done = O.combine_remote(part.out, y_remote, d.remote_src, part.route.topk_gate, "f32")
    assert np.max(np.abs(done - full.out)) <= 1e-5 * (1 + np.max(np.abs(full.out)))
    # nothing remote: nothing added
    same = O.combine_remote(full.out, np.zeros((0, H)), np.zeros(0, np.int64), full.route.topk_gate, "f32")
    assert np.array_equal(same, full.out)


def test_combine_remote_rounds_once_to_the_layer_dtype():
    """Hand values: 1 + g*y with one bf16 rounding (bf16 spacing just above 1 is 2^-7)."""
    gate = np.array([[0.5, 0.5]], np.float32)
    src = np.array([1], np.int64)                       # slot 1 of token 0 is the remote one
    one = np.ones((1, 4))
    y = np.array([[2.0 ** -8, 3 * 2.0 ** -8, 2.0 ** -7, 5 * 2.0 ** -8]])   # added: half of these
    got = O.combine_remote(one, y, src, gate, "bf16")
    # 1 + 2^-9 -> 1;  1 + 3*2^-9 -> 1 + 2^-7;  1 + 2^-8 is a tie -> even (1);  1 + 5*2^-9 -> 1 + 2^-7
    assert np.array_equal(got, np.array([[1.0, 1.0 + 2.0 ** -7, 1.0, 1.0 + 2.0 ** -7]], np.float32))
    assert np.array_equal(O.combine_remote(one, y, src, gate, "f32"), (1.0 + 0.5 * y).astype(np.float32))


# ---------------------------------------------------------------------------
# gates without renormalisation: the picked entries of the softmax over all experts
# ---------------------------------------------------------------------------

def test_unrenormalised_gates():
    rng = np.random.default_rng(31)
    T, H, E, k = 40, 24, 10, 3
    x = rng.standard_normal((T, H)).astype(np.float32)
    w = rng.standard_normal((E, H)).astype(np.float32)
    b = rng.standard_normal((1, E)).astype(np.float32)
    a = O.route(x, w, b, k)
    u = O.route(x, w, b, k, renormalize=False)
    assert np.array_equal(a.topk_idx, u.topk_idx) and np.array_equal(a.counts, u.counts)
    # library value: torch softmax over all experts, gathered at the picks
    p = torch.softmax(torch.from_numpy(u.logits.astype(np.float64)), dim=1).numpy()
    assert np.max(np.abs(u.topk_gate - np.take_along_axis(p, u.topk_idx.astype(np.int64), 1))) <= 1e-7
    s = u.topk_gate.astype(np.float64).sum(axis=1)
    assert np.all(s < 1.0) and np.all(s > 0.0)                       # mass of the other experts is left out
    # dividing by their sum gives back the renormalised gates
    assert np.max(np.abs(u.topk_gate / s[:, None] - a.topk_gate)) <= 1e-6
    # k = E: nothing is left out, both conventions coincide
    full_a, full_u = O.route(x, w, b, E), O.route(x, w, b, E, renormalize=False)
    assert np.max(np.abs(full_a.topk_gate - full_u.topk_gate)) <= 1e-7
    # zero router, no bias: every expert has probability 1/E
    z = O.route(x, np.zeros_like(w), None, k, renormalize=False)
    assert np.allclose(z.topk_gate, 1.0 / E, rtol=0, atol=1e-7)
