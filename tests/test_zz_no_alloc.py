"""prism_moe_layer_static -- the entry point for callers that cannot allocate -- against
prism_moe_layer, through the C ABI: two calls in a row on the library's fixed scratch array,
the second with a smaller batch of another layer shape, every output bit for bit; sizes beyond
the array are refused before anything is launched."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2508_12851_amd as P
from prism_inputs import make_config, make_inputs

from gpu_util import desc_of, oracle_layer, check_layer, to_dev, weight_table

pytestmark = pytest.mark.gpu

FIELDS = ("out", "topk_idx", "topk_gate", "counts", "remote_offsets", "n_local_remote", "remote_bytes")


def _both(cfg, inp):
    desc = desc_of(cfg)
    assert P.workspace_bytes(desc, cfg.T) <= P.STATIC_SCRATCH_BYTES
    args = (desc, to_dev(inp.x), to_dev(inp.w_router), to_dev(inp.bias), weight_table(inp), to_dev(inp.mask))
    want = P.prism_moe_layer(*args, P.alloc_workspace(desc, cfg.T))
    got = P.alloc_layer_out(desc, cfg.T)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    reserved_before = torch.cuda.memory_reserved()
    P.prism_moe_layer_static(*args, got)
    torch.cuda.synchronize()
    return want, got, (free_before, reserved_before)


def _same(cfg, want, got):
    for name in FIELDS:
        assert torch.equal(getattr(got, name), getattr(want, name)), name
    nr = int(want.n_local_remote[1])
    assert torch.equal(got.remote_src[:nr], want.remote_src[:nr])


def test_two_calls_in_a_row_the_second_smaller():
    big = make_config("cfg4_finegrained", T=700, H=128, F=192, bias_group_tokens=128)
    small = make_config("cfg3_mixtral_decode", T=19, H=256, F=448)
    first = True
    for cfg in (big, small):
        inp = make_inputs(cfg)
        want, got, (free_before, reserved_before) = _both(cfg, inp)
        _same(cfg, want, got)
        check_layer(cfg, got, oracle_layer(inp))          # and against the oracle, to the usual bar
        if not first:   # the first call on a device may load the address of the array; later ones change nothing
            assert torch.cuda.mem_get_info()[0] == free_before
            assert torch.cuda.memory_reserved() == reserved_before
        first = False
    # back to the larger batch: whatever the smaller call left in the array does not matter
    inp = make_inputs(big)
    want, got, _ = _both(big, inp)
    _same(big, want, got)


def test_the_decode_benchmark_shape_fits_and_matches():
    cfg = make_config("cfg3_mixtral_decode")
    inp = make_inputs(cfg, weights="local", threads=16)
    want, got, _ = _both(cfg, inp)
    _same(cfg, want, got)


def test_sizes_beyond_the_array_are_refused_before_any_launch():
    lib = P.load_library()
    d = P.make_desc(4096, 14336, 8, 2, 0, "bf16")
    assert P.workspace_bytes(d, 4096) > P.STATIC_SCRATCH_BYTES
    w = P.ExpertWeights()
    one = ctypes.c_void_p(0x1000)      # never dereferenced: the size check comes first
    w.w_gate = w.w_up = w.w_down = 0x1000
    code = lib.prism_moe_layer_static(ctypes.byref(d), one, one, None, ctypes.byref(w), one, 4096, one, one,
                                      one, one, None, one, one, one, one, None)
    assert code == 3 and lib.prism_status_string(code) == b"workspace too small"
    assert lib.prism_moe_layer_static(ctypes.byref(d), None, None, None, None, None, -1, None, None, None,
                                      None, None, None, None, None, None, None) == 1
