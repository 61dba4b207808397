"""The seeded workload generator: determinism, storage format, masks, Zipf skew."""
import numpy as np
import torch

from prism_inputs import (CONFIGS, bf16_bits_to_f32, f32_to_bf16_bits, make_config, make_inputs,
                          top_popular_mask, zipf_bias)


def test_bf16_roundtrip_matches_torch():
    a = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 3
    bits = f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(bf16_bits_to_f32(bits), ref.float().numpy())
    assert np.array_equal(bits, ref.view(torch.int16).numpy().view(np.uint16))


def test_deterministic_and_tensor_independent():
    c = make_config("cfg2_mixtral_prefill", T=16, H=64, F=32)
    a = make_inputs(c)
    b = make_inputs(c)
    assert np.array_equal(a.x, b.x) and np.array_equal(a.w_router, b.w_router)
    assert np.array_equal(a.expert(3)[2], b.expert(3)[2])      # regenerated alone
    assert a.x.dtype == np.uint16 and a.expert(0)[0].shape == (32, 64)
    assert not np.array_equal(a.expert(0)[0], a.expert(1)[0])


def test_decode_config_shares_weights_with_prefill_config():
    p = make_inputs(make_config("cfg2_mixtral_prefill", T=8, H=64, F=32))
    d = make_inputs(make_config("cfg3_mixtral_decode", T=8, H=64, F=32))
    assert np.array_equal(p.w_router, d.w_router)
    assert np.array_equal(p.expert(2)[1], d.expert(2)[1])
    assert not np.array_equal(p.x, d.x)
    assert np.array_equal(p.mask, d.mask)


def test_given_and_top_masks():
    assert make_inputs("cfg1_tiny_f32").mask.tolist() == [1, 0, 1, 0, 0, 1, 0, 1]
    c = make_config("cfg2_mixtral_prefill", T=8, H=64, F=32)
    inp = make_inputs(c)
    assert int(inp.mask.sum()) == 5
    hosted_ranks = sorted(inp.ranks[0][inp.mask == 1].tolist())
    assert hosted_ranks == [1, 2, 3, 4, 5]
    assert np.allclose(inp.bias[0], -np.log(inp.ranks[0]))
    m = top_popular_mask(np.array([[1, 2, 3, 4]]), 1.0, 2)
    assert m.tolist() == [1, 1, 0, 0]
    assert zipf_bias(np.array([1, 2]), 2.0).tolist() == [0.0, np.float32(-2 * np.log(2.0))]


def test_per_block_rankings_and_two_phase_mask_swap():
    c4 = make_config("cfg4_finegrained", T=2048, H=32, F=32)
    i4 = make_inputs(c4)
    assert i4.bias.shape == (4, 60) and int(i4.mask.sum()) == 36
    assert not np.array_equal(i4.ranks[0], i4.ranks[1])
    c5 = make_config("cfg5_dsv2lite_migration", T=64, H=32, F=32)
    p0, p1 = make_inputs(c5, 0), make_inputs(c5, 1)
    assert int(p0.mask.sum()) == int(p1.mask.sum()) == 32
    assert int((p0.mask != p1.mask).sum()) == 32          # 16 evicted + 16 admitted
    assert not np.array_equal(p0.x, p1.x) and not np.array_equal(p0.ranks, p1.ranks)
    assert np.array_equal(p0.w_router, p1.w_router)


def test_all_named_configs_have_consistent_shapes():
    for name, c in CONFIGS.items():
        assert 1 <= c.k <= c.E and c.n_local <= c.E and c.dtype in ("f32", "bf16"), name
