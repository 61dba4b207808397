"""The tiled weight layout (16 x 32 tiles): the pack kernel against a plain numpy re-layout, and the
layer with tiled weights against the oracle and, bit for bit, against the row-major layer."""
import numpy as np
import pytest
import torch

import paper_2508_12851_amd as P
from prism_inputs import CONFIGS, make_config, make_inputs

from gpu_util import check_layer, oracle_layer, rel_err, run_layer, to_dev, to_f32, weight_table

pytestmark = pytest.mark.gpu


def _tiled_numpy(a):
    """[rows, cols] -> element (r, c) at ((r/16)(cols/32) + c/32) * 512 + (r%16) * 32 + c%32."""
    rows, cols = a.shape
    return a.reshape(rows // 16, 16, cols // 32, 32).transpose(0, 2, 1, 3).reshape(rows, cols)


@pytest.mark.parametrize("rows,cols", [(16, 32), (64, 64), (48, 160), (1408, 2048), (4096, 14336)])
def test_pack_kernel_matches_plain_relayout(rows, cols):
    a = np.random.default_rng(rows + cols).integers(0, 1 << 16, size=(rows, cols), dtype=np.uint16)
    packed = P.prism_pack_weights(to_dev(a))
    torch.cuda.synchronize()
    got = packed.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got.reshape(-1), _tiled_numpy(a).reshape(-1))


CASES = {
    "mixtral_small": dict(name="cfg2_mixtral_prefill", T=333, H=256, F=448),
    "mixtral_decode": dict(name="cfg3_mixtral_decode", T=32, H=256, F=448),
    "finegrained_small": dict(name="cfg4_finegrained", T=700, H=128, F=192, bias_group_tokens=128),
    "dsv2_decode": dict(name="cfg5_dsv2lite_migration", T=64, H=1024, F=256),
    "short_contraction": dict(name="cfg4_finegrained", T=300, H=64, F=192, E=12, k=3, S=1, n_local=7,
                              bias_group_tokens=0),
    "two_big_experts": dict(name="cfg2_mixtral_prefill", T=1100, H=256, F=448, E=2, k=2, n_local=1),
    "mixtral_mid": dict(name="cfg2_mixtral_prefill", T=200, H=256, F=1024),
    # decode batches whose shapes take the 32-wide k-tiles of the tiled layout (8-stage ring)
    "mixtral_decode_wide": dict(name="cfg3_mixtral_decode", T=32, H=512, F=1536),
    "finegrained_decode_wide": dict(name="cfg4_finegrained", T=50, H=256, F=1088, bias_group_tokens=16),
}


@pytest.mark.parametrize("case", list(CASES))
def test_layer_with_tiled_weights(case):
    kw = dict(CASES[case])
    cfg = make_config(kw.pop("name"), **kw)
    inp = make_inputs(cfg)
    ref = oracle_layer(inp)
    tiled = run_layer(cfg, inp, wt=weight_table(inp, tiled=True), weight_layout="tiled")
    err = check_layer(cfg, tiled, ref)
    plain = run_layer(cfg, inp)
    if "decode_wide" in case:    # other k-tile width: the same sums from another starting k-tile
        assert rel_err(to_f32(tiled.out), to_f32(plain.out)) <= 1e-2
    else:
        assert torch.equal(tiled.out, plain.out)        # same sums in the same order
    print(f"{case}: out err {err:.3g}")


def test_tiled_layout_is_refused_for_fp32_layers():
    d = P.make_desc(64, 64, 4, 2, 0, "f32", weight_layout="tiled")
    with pytest.raises(P.PrismError, match="supported limits"):
        P.workspace_bytes(d, 8)


@pytest.mark.parametrize("name", ["cfg2_mixtral_prefill", "cfg3_mixtral_decode"])
def test_full_size_tiled_equals_row_major(name):
    cfg = CONFIGS[name]
    inp = make_inputs(cfg, weights="local", threads=16)
    plain = run_layer(cfg, inp)
    tiled = run_layer(cfg, inp, wt=weight_table(inp, tiled=True), weight_layout="tiled")
    assert torch.equal(tiled.topk_idx, plain.topk_idx)
    if cfg.T <= 64:              # decode: 32-wide k-tiles, the sums start from another k-tile
        assert rel_err(to_f32(tiled.out), to_f32(plain.out)) <= 1e-2
    else:
        assert torch.equal(tiled.out, plain.out)
