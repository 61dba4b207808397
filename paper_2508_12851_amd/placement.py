"""ctypes binding of the scheduler-side placement entry points (include/prism_placement.h).
Argument marshalling only: numpy host arrays in, numpy host arrays out."""
from __future__ import annotations

import ctypes
from typing import Sequence, Tuple

import numpy as np

from .binding import PrismError, load_library

PLACEMENT_SYMBOLS = ("prism_activation_entropy", "prism_expert_count_allocation",
                     "prism_expert_assignment", "prism_proxy_cost", "prism_migration_cost",
                     "prism_migration_decision", "prism_placement_plan")

_ready = False


def _lib():
    global _ready
    lib = load_library()
    if not _ready:
        vp, i32, i64, f64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
        lib.prism_activation_entropy.argtypes = [vp, i32, i32, i32, vp]
        lib.prism_expert_count_allocation.argtypes = [vp, vp, f64, i32, i32, i32, vp,
                                                      ctypes.POINTER(i32)]
        lib.prism_expert_assignment.argtypes = [vp, vp, i32, i32, i32, vp, ctypes.POINTER(i32)]
        lib.prism_proxy_cost.argtypes = [vp, vp, i32, i32, i32, ctypes.POINTER(i64)]
        lib.prism_migration_cost.argtypes = [vp, vp, i32, i32, i32, f64, vp, ctypes.POINTER(f64),
                                             ctypes.POINTER(i64)]
        lib.prism_migration_decision.argtypes = [i64, i64, f64, f64, ctypes.POINTER(i32)]
        lib.prism_placement_plan.argtypes = [vp, vp, f64, i32, i32, i32, vp, vp, vp,
                                             ctypes.POINTER(i32)]
        for name in PLACEMENT_SYMBOLS:
            getattr(lib, name).restype = ctypes.c_int
        _ready = True
    return lib


def _check(code: int, what: str) -> None:
    if code != 0:
        raise PrismError(f"{what}: {load_library().prism_status_string(code).decode()} (status {code})")


def _arr(a, dtype, shape=None) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    if shape is not None and a.shape != tuple(shape):
        raise PrismError(f"expected an array of shape {tuple(shape)}, got {a.shape}")
    return a


def _p(a: np.ndarray) -> int:
    return a.ctypes.data


def _dims(f: np.ndarray) -> Tuple[int, int, int]:
    if f.ndim != 3:
        raise PrismError("f must be [servers, layers, experts]")
    return f.shape


def activation_entropy(f) -> np.ndarray:
    f = _arr(f, np.int64)
    N, L, E = _dims(f)
    v = np.empty((N, L), np.float64)
    _check(_lib().prism_activation_entropy(_p(f), N, L, E, _p(v)), "prism_activation_entropy")
    return v


def expert_count_allocation(v, server_mem: Sequence[float], expert_mem: float,
                            n_experts: int) -> Tuple[np.ndarray, bool]:
    v = _arr(v, np.float64)
    N, L = v.shape
    mem = _arr(server_mem, np.float64, (N,))
    counts = np.empty((N, L), np.int32)
    feasible = ctypes.c_int32(0)
    _check(_lib().prism_expert_count_allocation(_p(v), _p(mem), float(expert_mem), N, L, n_experts,
                                                _p(counts), ctypes.byref(feasible)),
           "prism_expert_count_allocation")
    return counts, bool(feasible.value)


def expert_assignment(f, counts) -> Tuple[np.ndarray, bool]:
    f = _arr(f, np.int64)
    N, L, E = _dims(f)
    counts = _arr(counts, np.int32, (N, L))
    placement = np.empty((N, L, E), np.uint8)
    covered = ctypes.c_int32(0)
    _check(_lib().prism_expert_assignment(_p(f), _p(counts), N, L, E, _p(placement),
                                          ctypes.byref(covered)), "prism_expert_assignment")
    return placement, bool(covered.value)


def proxy_cost(f, placement) -> int:
    f = _arr(f, np.int64)
    N, L, E = _dims(f)
    placement = _arr(placement, np.uint8, (N, L, E))
    cost = ctypes.c_int64(0)
    _check(_lib().prism_proxy_cost(_p(f), _p(placement), N, L, E, ctypes.byref(cost)),
           "prism_proxy_cost")
    return cost.value


def migration_cost(old, new, expert_mem: float, speed: Sequence[float]) -> Tuple[float, int]:
    old = _arr(old, np.uint8)
    N, L, E = _dims(old)
    new = _arr(new, np.uint8, (N, L, E))
    speed = _arr(speed, np.float64, (N,))
    seconds, flips = ctypes.c_double(0.0), ctypes.c_int64(0)
    _check(_lib().prism_migration_cost(_p(old), _p(new), N, L, E, float(expert_mem), _p(speed),
                                       ctypes.byref(seconds), ctypes.byref(flips)),
           "prism_migration_cost")
    return seconds.value, flips.value


def migration_decision(cost_old: int, cost_new: int, t_mig: float,
                       seconds_per_remote_call: float) -> bool:
    adopt = ctypes.c_int32(0)
    _check(_lib().prism_migration_decision(int(cost_old), int(cost_new), float(t_mig),
                                           float(seconds_per_remote_call), ctypes.byref(adopt)),
           "prism_migration_decision")
    return bool(adopt.value)


def placement_plan(f, server_mem: Sequence[float], expert_mem: float):
    """-> (v [N,L], counts [N,L], placement [N,L,E] uint8, ok)."""
    f = _arr(f, np.int64)
    N, L, E = _dims(f)
    mem = _arr(server_mem, np.float64, (N,))
    v = np.empty((N, L), np.float64)
    counts = np.empty((N, L), np.int32)
    placement = np.empty((N, L, E), np.uint8)
    ok = ctypes.c_int32(0)
    _check(_lib().prism_placement_plan(_p(f), _p(mem), float(expert_mem), N, L, E, _p(v), _p(counts),
                                       _p(placement), ctypes.byref(ok)), "prism_placement_plan")
    return v, counts, placement, bool(ok.value)
