"""Thin ctypes binding of libprism's C ABI (include/prism.h).

Argument marshalling only: every step of the layer runs in the HIP kernels of
libprism.so.  PyTorch is used for device memory and streams.  There is no CPU
fallback: if the library is missing, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libprism.so")

PRISM_F32, PRISM_BF16 = 0, 1
SYMBOLS = ("prism_status_string", "prism_workspace_bytes", "prism_route", "prism_dispatch",
           "prism_expert_ffn", "prism_combine", "prism_moe_layer", "prism_moe_layer_traced",
           "prism_ceiling_mfma_bf16", "prism_ceiling_hbm_read", "prism_pack_remote",
           "prism_combine_remote", "prism_debug_check_weights", "prism_pack_weights",
           "prism_layer_permutation", "prism_moe_layer_static", "prism_ceiling_hbm_read_pattern")
STAGES = ("route", "dispatch", "ffn_up", "ffn_down", "combine")
GATE_MODES = {"renormalized": 0, "softmax_all": 1}
WEIGHT_LAYOUTS = {"row_major": 0, "tiled": 1}


class PrismError(RuntimeError):
    pass


class LayerDesc(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int32), ("ffn", ctypes.c_int32), ("n_experts", ctypes.c_int32),
                ("top_k", ctypes.c_int32), ("n_shared", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("bias_group_tokens", ctypes.c_int32), ("gate_mode", ctypes.c_int32),
                ("weight_layout", ctypes.c_int32)]


class ExpertWeights(ctypes.Structure):
    _fields_ = [("w_gate", ctypes.c_void_p), ("w_up", ctypes.c_void_p), ("w_down", ctypes.c_void_p),
                ("shared_w_gate", ctypes.c_void_p), ("shared_w_up", ctypes.c_void_p),
                ("shared_w_down", ctypes.c_void_p)]


_lib = None


def load_library(build_if_missing: bool = True) -> ctypes.CDLL:
    """Load libprism.so (building it in-tree first if it does not exist)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise PrismError(f"{LIB_PATH} is not built; run python -m paper_2508_12851_amd.build")
        from . import build as _build
        _build.build_library(verbose=False)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    dp = ctypes.POINTER(LayerDesc)
    wp = ctypes.POINTER(ExpertWeights)
    lib.prism_status_string.restype = ctypes.c_char_p
    lib.prism_status_string.argtypes = [ctypes.c_int]
    lib.prism_workspace_bytes.argtypes = [dp, i32, ctypes.POINTER(sz)]
    lib.prism_route.argtypes = [dp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.prism_dispatch.argtypes = [dp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.prism_expert_ffn.argtypes = [dp, vp, wp, vp, vp, i32, vp, vp, sz, vp]
    lib.prism_combine.argtypes = [dp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
    lib.prism_moe_layer.argtypes = [dp, vp, vp, vp, wp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                    vp, sz, vp]
    lib.prism_moe_layer_traced.argtypes = lib.prism_moe_layer.argtypes + [vp]
    lib.prism_moe_layer_static.argtypes = lib.prism_moe_layer.argtypes[:16] + [vp]
    lib.prism_pack_remote.argtypes = [dp, vp, vp, vp, i32, vp, vp]
    lib.prism_combine_remote.argtypes = [dp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
    lib.prism_pack_weights.argtypes = [vp, i32, i32, vp, vp]
    lib.prism_layer_permutation.argtypes = [dp, i32, vp, sz, vp, vp, vp, vp]
    lib.prism_debug_check_weights.argtypes = [dp, wp, vp, ctypes.POINTER(i32)]
    lib.prism_ceiling_mfma_bf16.argtypes = [vp, vp, i32, i32, ctypes.POINTER(ctypes.c_double), vp]
    lib.prism_ceiling_hbm_read.argtypes = [vp, sz, vp, i32, vp]
    lib.prism_ceiling_hbm_read_pattern.argtypes = [vp, sz, vp, i32, i32, sz, i32, ctypes.POINTER(sz), vp]
    for name in SYMBOLS:
        # without argtypes ctypes would pass a device address as a 32-bit int
        if getattr(lib, name).argtypes is None:
            raise PrismError(f"binding bug: no argument types declared for {name}")
    for name in SYMBOLS[1:]:
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _check(code: int, what: str) -> None:
    if code != 0:
        msg = load_library().prism_status_string(code).decode()
        raise PrismError(f"{what}: {msg} (status {code})")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise PrismError("libprism takes contiguous device tensors")
    return t.data_ptr()


def _stream(stream: Optional[torch.cuda.Stream]) -> Optional[int]:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def make_desc(hidden: int, ffn: int, n_experts: int, top_k: int, n_shared: int = 0,
              dtype: str = "bf16", bias_group_tokens: int = 0,
              gate_mode: str = "renormalized", weight_layout: str = "row_major") -> LayerDesc:
    return LayerDesc(hidden, ffn, n_experts, top_k, n_shared,
                     PRISM_F32 if dtype == "f32" else PRISM_BF16, bias_group_tokens,
                     GATE_MODES[gate_mode], WEIGHT_LAYOUTS[weight_layout])


def torch_dtype(desc: LayerDesc) -> torch.dtype:
    return torch.float32 if desc.dtype == PRISM_F32 else torch.bfloat16


class WeightTable:
    """Device arrays of device pointers to the expert weight matrices.

    experts[e] is (w_gate[F,H], w_up[F,H], w_down[H,F]) or None for an expert
    that is not hosted here; shared is a list of S such triples.  The tensors
    are kept alive by this object.
    """

    def __init__(self, experts: Sequence, shared: Sequence = (), device="cuda"):
        self.keep = (list(experts), list(shared))

        def table(items, i):
            ptrs = [0 if it is None else _ptr(it[i]) for it in items]
            if not ptrs:
                return None
            return torch.tensor(ptrs, dtype=torch.int64, device=device)

        self.tables = [table(experts, i) for i in range(3)] + [table(shared, i) for i in range(3)]
        self.struct = ExpertWeights(*[None if t is None else t.data_ptr() for t in self.tables])


def workspace_bytes(desc: LayerDesc, max_tokens: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().prism_workspace_bytes(ctypes.byref(desc), max_tokens, ctypes.byref(n)),
           "prism_workspace_bytes")
    return n.value


def alloc_workspace(desc: LayerDesc, max_tokens: int, device="cuda") -> torch.Tensor:
    return torch.empty(workspace_bytes(desc, max_tokens), dtype=torch.uint8, device=device)


@dataclass
class RouteOut:
    logits: Optional[torch.Tensor]
    topk_idx: torch.Tensor
    topk_gate: torch.Tensor
    counts: torch.Tensor


def prism_route(desc: LayerDesc, x, w_router, router_bias, want_logits=True, counts_accum=None,
                stream=None) -> RouteOut:
    T, E, k = x.shape[0], desc.n_experts, desc.top_k
    dev = x.device
    logits = torch.empty((T, E), dtype=torch.float32, device=dev) if want_logits else None
    idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    gate = torch.empty((T, k), dtype=torch.float32, device=dev)
    counts = torch.empty((E,), dtype=torch.int32, device=dev)
    _check(load_library().prism_route(ctypes.byref(desc), _ptr(x), _ptr(w_router), _ptr(router_bias),
                                      T, _ptr(logits), _ptr(idx), _ptr(gate), _ptr(counts),
                                      _ptr(counts_accum), _stream(stream)), "prism_route")
    return RouteOut(logits, idx, gate, counts)


@dataclass
class DispatchOut:
    local_src: torch.Tensor
    local_offsets: torch.Tensor
    remote_src: torch.Tensor
    remote_offsets: torch.Tensor
    n_local_remote: torch.Tensor
    remote_bytes: torch.Tensor


def prism_dispatch(desc: LayerDesc, topk_idx, local_mask, workspace, stream=None) -> DispatchOut:
    T, E, k = topk_idx.shape[0], desc.n_experts, desc.top_k
    dev = topk_idx.device
    i32 = dict(dtype=torch.int32, device=dev)
    out = DispatchOut(torch.full((T * k,), -1, **i32), torch.empty((E + 1,), **i32),
                      torch.full((T * k,), -1, **i32), torch.empty((E + 1,), **i32),
                      torch.empty((2,), **i32), torch.empty((2,), dtype=torch.int64, device=dev))
    _check(load_library().prism_dispatch(ctypes.byref(desc), _ptr(topk_idx), _ptr(local_mask), T,
                                         _ptr(out.local_src), _ptr(out.local_offsets),
                                         _ptr(out.remote_src), _ptr(out.remote_offsets),
                                         _ptr(out.n_local_remote), _ptr(out.remote_bytes),
                                         _ptr(workspace), workspace.numel(), _stream(stream)),
           "prism_dispatch")
    return out


def prism_expert_ffn(desc: LayerDesc, x, weights: WeightTable, local_src, local_offsets, workspace,
                     y=None, stream=None) -> torch.Tensor:
    T = x.shape[0]
    rows = T * desc.top_k + desc.n_shared * T
    if y is None:
        y = torch.zeros((rows, desc.hidden), dtype=torch_dtype(desc), device=x.device)
    _check(load_library().prism_expert_ffn(ctypes.byref(desc), _ptr(x), ctypes.byref(weights.struct),
                                           _ptr(local_src), _ptr(local_offsets), T, _ptr(y),
                                           _ptr(workspace), workspace.numel(), _stream(stream)),
           "prism_expert_ffn")
    return y


def prism_combine(desc: LayerDesc, y, local_src, local_offsets, topk_gate, workspace, out=None,
                  stream=None) -> torch.Tensor:
    T = topk_gate.shape[0]
    if out is None:
        out = torch.empty((T, desc.hidden), dtype=torch_dtype(desc), device=y.device)
    _check(load_library().prism_combine(ctypes.byref(desc), _ptr(y), _ptr(local_src),
                                        _ptr(local_offsets), _ptr(topk_gate), T, _ptr(out),
                                        _ptr(workspace), workspace.numel(), _stream(stream)),
           "prism_combine")
    return out


@dataclass
class LayerOut:
    out: torch.Tensor
    topk_idx: torch.Tensor
    topk_gate: torch.Tensor
    counts: torch.Tensor
    remote_src: torch.Tensor
    remote_offsets: torch.Tensor
    n_local_remote: torch.Tensor
    remote_bytes: torch.Tensor


def alloc_layer_out(desc: LayerDesc, T: int, device="cuda") -> LayerOut:
    E, k = desc.n_experts, desc.top_k
    i32 = dict(dtype=torch.int32, device=device)
    return LayerOut(torch.empty((T, desc.hidden), dtype=torch_dtype(desc), device=device),
                    torch.empty((T, k), **i32), torch.empty((T, k), dtype=torch.float32, device=device),
                    torch.empty((E,), **i32), torch.full((T * k,), -1, **i32),
                    torch.empty((E + 1,), **i32), torch.empty((2,), **i32),
                    torch.empty((2,), dtype=torch.int64, device=device))


def prism_moe_layer(desc: LayerDesc, x, w_router, router_bias, weights: WeightTable, local_mask,
                    workspace, outputs: Optional[LayerOut] = None, counts_accum=None,
                    stream=None, stage_events=None) -> LayerOut:
    """stage_events: optional ctypes array of 2*len(STAGES) hipEvent_t handles (see prism.h)."""
    T = x.shape[0]
    o = alloc_layer_out(desc, T, x.device) if outputs is None else outputs
    lib = load_library()
    if stage_events is not None:
        _check(lib.prism_moe_layer_traced(ctypes.byref(desc), _ptr(x), _ptr(w_router),
                                          _ptr(router_bias), ctypes.byref(weights.struct),
                                          _ptr(local_mask), T, _ptr(o.out), _ptr(o.topk_idx),
                                          _ptr(o.topk_gate), _ptr(o.counts), _ptr(counts_accum),
                                          _ptr(o.remote_src), _ptr(o.remote_offsets),
                                          _ptr(o.n_local_remote), _ptr(o.remote_bytes),
                                          _ptr(workspace), workspace.numel(), _stream(stream),
                                          ctypes.cast(stage_events, ctypes.c_void_p)),
               "prism_moe_layer_traced")
        return o
    _check(load_library().prism_moe_layer(ctypes.byref(desc), _ptr(x), _ptr(w_router),
                                          _ptr(router_bias), ctypes.byref(weights.struct),
                                          _ptr(local_mask), T, _ptr(o.out), _ptr(o.topk_idx),
                                          _ptr(o.topk_gate), _ptr(o.counts), _ptr(counts_accum),
                                          _ptr(o.remote_src), _ptr(o.remote_offsets),
                                          _ptr(o.n_local_remote), _ptr(o.remote_bytes),
                                          _ptr(workspace), workspace.numel(), _stream(stream)),
           "prism_moe_layer")
    return o


STATIC_SCRATCH_BYTES = 32 << 20


def prism_moe_layer_static(desc: LayerDesc, x, w_router, router_bias, weights: WeightTable, local_mask,
                           outputs: LayerOut, counts_accum=None, stream=None) -> LayerOut:
    """The layer on the library's fixed scratch array: no workspace, nothing allocated (the caller
    supplies every output buffer)."""
    o = outputs
    _check(load_library().prism_moe_layer_static(ctypes.byref(desc), _ptr(x), _ptr(w_router),
                                                 _ptr(router_bias), ctypes.byref(weights.struct),
                                                 _ptr(local_mask), x.shape[0], _ptr(o.out),
                                                 _ptr(o.topk_idx), _ptr(o.topk_gate), _ptr(o.counts),
                                                 _ptr(counts_accum), _ptr(o.remote_src),
                                                 _ptr(o.remote_offsets), _ptr(o.n_local_remote),
                                                 _ptr(o.remote_bytes), _stream(stream)),
           "prism_moe_layer_static")
    return o


@dataclass
class LayerPermutation:
    local_src: torch.Tensor
    local_offsets: torch.Tensor
    inv: torch.Tensor


def prism_layer_permutation(desc: LayerDesc, T: int, workspace, stream=None) -> LayerPermutation:
    """Copies of the permutation the last whole-layer call left in `workspace` (see prism.h)."""
    i32 = dict(dtype=torch.int32, device=workspace.device)
    A = T * desc.top_k
    p = LayerPermutation(torch.full((A,), -1, **i32), torch.empty((desc.n_experts + 1,), **i32),
                         torch.empty((A,), **i32))
    _check(load_library().prism_layer_permutation(ctypes.byref(desc), T, _ptr(workspace),
                                                  workspace.numel(), _ptr(p.local_src),
                                                  _ptr(p.local_offsets), _ptr(p.inv), _stream(stream)),
           "prism_layer_permutation")
    return p


def prism_ceiling_mfma_bf16(operands, out, n_workgroups: int, iters: int, stream=None) -> float:
    """Enqueues the pure-MFMA loop (see prism.h); returns the flop count of the launch."""
    flop = ctypes.c_double(0.0)
    _check(load_library().prism_ceiling_mfma_bf16(_ptr(operands), _ptr(out), n_workgroups, iters,
                                                  ctypes.byref(flop), _stream(stream)),
           "prism_ceiling_mfma_bf16")
    return flop.value


def prism_ceiling_hbm_read(src, out, n_workgroups: int, stream=None) -> int:
    """Enqueues the streaming read of all of src (see prism.h); returns the bytes read."""
    nbytes = src.numel() * src.element_size()
    _check(load_library().prism_ceiling_hbm_read(_ptr(src), ctypes.c_size_t(nbytes), _ptr(out),
                                                 n_workgroups, _stream(stream)),
           "prism_ceiling_hbm_read")
    return nbytes // 16 * 16


def prism_ceiling_hbm_read_pattern(src, out, n_workgroups: int, loads_in_flight: int, span_bytes: int,
                                   mode: int, stream=None) -> int:
    """Enqueues the streaming read with the given access pattern (see prism.h); returns the bytes read."""
    n = ctypes.c_size_t(0)
    _check(load_library().prism_ceiling_hbm_read_pattern(_ptr(src), ctypes.c_size_t(src.numel() * src.element_size()),
                                                         _ptr(out), n_workgroups, loads_in_flight,
                                                         ctypes.c_size_t(span_bytes), mode, ctypes.byref(n),
                                                         _stream(stream)),
           "prism_ceiling_hbm_read_pattern")
    return n.value


def prism_pack_remote(desc: LayerDesc, x, remote_src, remote_offsets, stream=None) -> torch.Tensor:
    """Activation rows to ship, in remote-list order ([T*k, H]; rows past the remote count are zero)."""
    T = x.shape[0]
    packed = torch.zeros((T * desc.top_k, desc.hidden), dtype=x.dtype, device=x.device)
    _check(load_library().prism_pack_remote(ctypes.byref(desc), _ptr(x), _ptr(remote_src),
                                            _ptr(remote_offsets), T, _ptr(packed), _stream(stream)),
           "prism_pack_remote")
    return packed


def prism_combine_remote(desc: LayerDesc, y_remote, remote_src, remote_offsets, topk_gate, out,
                         workspace, stream=None) -> torch.Tensor:
    """Adds the returned expert outputs (remote-list order) into out, in place."""
    T = topk_gate.shape[0]
    _check(load_library().prism_combine_remote(ctypes.byref(desc), _ptr(y_remote), _ptr(remote_src),
                                               _ptr(remote_offsets), _ptr(topk_gate), T, _ptr(out),
                                               _ptr(workspace), workspace.numel(), _stream(stream)),
           "prism_combine_remote")
    return out


def prism_debug_check_weights(desc: LayerDesc, weights: WeightTable, local_mask) -> None:
    """Blocking check that every hosted and every shared expert has usable weight pointers."""
    bad = ctypes.c_int32(-1)
    code = load_library().prism_debug_check_weights(ctypes.byref(desc), ctypes.byref(weights.struct),
                                                    _ptr(local_mask), ctypes.byref(bad))
    if code != 0:
        what = f"expert {bad.value}" if bad.value >= 0 else "arguments"
        _check(code, f"prism_debug_check_weights ({what})")


def prism_pack_weights(w, stream=None) -> torch.Tensor:
    """Row-major bf16 weight matrix -> the layout of 16 x 32 tiles (a new tensor of the same shape)."""
    rows, cols = w.shape
    packed = torch.empty_like(w)
    _check(load_library().prism_pack_weights(_ptr(w), rows, cols, _ptr(packed), _stream(stream)),
           "prism_pack_weights")
    return packed
