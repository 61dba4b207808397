"""The C-ABI library builds, loads and exports every symbol include/*.h declares;
host-side validation returns error codes (no kernel is launched in these tests)."""
import ctypes
import os
import re

import pytest

import paper_2508_12851_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    return sorted(set(re.findall(r"\b(prism_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    from paper_2508_12851_amd.placement import PLACEMENT_SYMBOLS
    lib = P.load_library()
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["prism.h", "prism_placement.h"]
    assert sorted(P.SYMBOLS) == _declared_symbols("prism.h")
    assert sorted(PLACEMENT_SYMBOLS) == _declared_symbols("prism_placement.h")
    for name in _declared_symbols("prism.h") + _declared_symbols("prism_placement.h"):
        assert hasattr(lib, name), name


def test_every_entry_point_has_declared_argument_types():
    """A ctypes call without argtypes would truncate 64-bit device addresses."""
    lib = P.load_library()
    for name in P.SYMBOLS:
        assert getattr(lib, name).argtypes is not None, name


def test_status_strings():
    lib = P.load_library()
    assert lib.prism_status_string(0) == b"ok"
    texts = {lib.prism_status_string(i) for i in range(5)}
    assert len(texts) == 5 and all(texts)


def test_workspace_bytes_grows_with_tokens_and_is_aligned():
    d = P.make_desc(4096, 14336, 8, 2, 0, "bf16")
    small, big = P.workspace_bytes(d, 32), P.workspace_bytes(d, 4096)
    assert 0 < small < big and small % 256 == 0 and big % 256 == 0
    # h and y for T*k rows dominate: (8192*14336 + 8192*4096) * 2 bytes
    assert big >= (8192 * 14336 + 8192 * 4096) * 2
    assert P.workspace_bytes(d, 0) > 0


def test_workspace_for_max_tokens_serves_every_smaller_batch():
    """prism_workspace_bytes never shrinks as T grows (also across the decode-path boundary)."""
    for d in (P.make_desc(4096, 14336, 8, 2, 0, "bf16"), P.make_desc(2048, 1408, 60, 4, 4, "bf16"),
              P.make_desc(64, 96, 4, 2, 1, "f32"), P.make_desc(1024, 256, 256, 8, 2, "bf16")):
        sizes = [P.workspace_bytes(d, t) for t in (*range(0, 700), 1000, 4096)]   # every path boundary
        assert sizes == sorted(sizes), sizes


@pytest.mark.parametrize("kw,status", [
    (dict(top_k=0), 1), (dict(top_k=9, n_experts=8), 1), (dict(n_experts=257), 2),
    (dict(top_k=9, n_experts=16), 2), (dict(hidden=100), 2), (dict(ffn=100), 2),
    (dict(n_shared=17), 2), (dict(dtype_code=7), 1),
])
def test_validation_error_codes(kw, status):
    base = dict(hidden=128, ffn=128, n_experts=8, top_k=2, n_shared=0, dtype_code=1)
    base.update(kw)
    d = P.LayerDesc(base["hidden"], base["ffn"], base["n_experts"], base["top_k"],
                    base["n_shared"], base["dtype_code"], 0)
    n = ctypes.c_size_t(0)
    assert P.load_library().prism_workspace_bytes(ctypes.byref(d), 16, ctypes.byref(n)) == status


def test_unknown_gate_mode_is_rejected():
    d = P.make_desc(128, 128, 8, 2, 0, "bf16")
    d.gate_mode = 7
    n = ctypes.c_size_t(0)
    assert P.load_library().prism_workspace_bytes(ctypes.byref(d), 16, ctypes.byref(n)) == 1
    d.gate_mode = 1
    assert P.load_library().prism_workspace_bytes(ctypes.byref(d), 16, ctypes.byref(n)) == 0


def test_weight_layout_validation():
    lib = P.load_library()
    n = ctypes.c_size_t(0)
    d = P.make_desc(128, 128, 8, 2, 0, "bf16", weight_layout="tiled")
    assert lib.prism_workspace_bytes(ctypes.byref(d), 16, ctypes.byref(n)) == 0
    d.weight_layout = 5
    assert lib.prism_workspace_bytes(ctypes.byref(d), 16, ctypes.byref(n)) == 1
    d = P.make_desc(128, 128, 8, 2, 0, "f32", weight_layout="tiled")       # bf16 layers only
    assert lib.prism_workspace_bytes(ctypes.byref(d), 16, ctypes.byref(n)) == 2
    # prism_pack_weights: NULL, misaligned, rows not in 16s and columns not in 32s are refused before any launch
    assert lib.prism_pack_weights(None, 64, 64, None, None) == 1
    assert lib.prism_pack_weights(ctypes.c_void_p(0x1000), 0, 64, ctypes.c_void_p(0x2000), None) == 1
    assert lib.prism_pack_weights(ctypes.c_void_p(0x1008), 64, 64, ctypes.c_void_p(0x2000), None) == 1
    assert lib.prism_pack_weights(ctypes.c_void_p(0x1000), 72, 64, ctypes.c_void_p(0x2000), None) == 2
    assert lib.prism_pack_weights(ctypes.c_void_p(0x1000), 64, 100, ctypes.c_void_p(0x2000), None) == 2


def test_null_pointers_and_negative_tokens_are_rejected_before_any_launch():
    lib = P.load_library()
    d = P.make_desc(128, 128, 8, 2, 0, "bf16")
    n = ctypes.c_size_t(0)
    assert lib.prism_workspace_bytes(ctypes.byref(d), -1, ctypes.byref(n)) == 1
    assert lib.prism_workspace_bytes(ctypes.byref(d), 16, None) == 1
    assert lib.prism_workspace_bytes(None, 16, ctypes.byref(n)) == 1
    # counts == NULL
    assert lib.prism_route(ctypes.byref(d), None, None, None, 4, None, None, None, None, None, None) == 1
    # required outputs NULL
    assert lib.prism_dispatch(ctypes.byref(d), None, None, 4, None, None, None, None, None, None,
                              None, 0, None) == 1
    w = P.ExpertWeights()
    assert lib.prism_expert_ffn(ctypes.byref(d), None, ctypes.byref(w), None, None, 4, None, None, 0,
                                None) == 1
    assert lib.prism_combine(ctypes.byref(d), None, None, None, None, 4, None, None, 0, None) == 1
    assert lib.prism_moe_layer(ctypes.byref(d), None, None, None, None, None, 4, None, None, None,
                               None, None, None, None, None, None, None, 0, None) == 1
    with pytest.raises(P.PrismError):
        P.workspace_bytes(P.make_desc(100, 128, 8, 2), 4)


def test_a_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    """Without the built library the binding raises: there is no other path that could answer."""
    from paper_2508_12851_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libprism.so"))
    with pytest.raises(P.PrismError, match="not built"):
        binding.load_library(build_if_missing=False)
    # nothing in the package imports the oracle
    pkg = os.path.join(ROOT, "paper_2508_12851_amd")
    for dirpath, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, name)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), name
