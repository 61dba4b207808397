"""Plain CPU oracle for one edge server's placement-aware MoE layer forward.

THIS IS TEST INFRASTRUCTURE.  Only the test-suite, the smoke check and the
benchmark's reported CPU-baseline leg may import it; the product (the HIP
library and its binding) never does, and shares no code with it.

What it computes (paper: Prism, Sec. III-A "System Architecture" for the data
flow gate -> local / remote experts -> aggregate; Sec. III-B "Problem
Formulation" for the activation frequency f_n^l(e) and the local/remote
indicator 1_remote(n, e)).  The paper fixes the *roles* of the steps but not
their formulas; where it is silent the readings below are used (they are the
standard definitions of the two model families it evaluates, Sec. IV):

  route      logit[t,e] = fl32( sum_h x[t,h] * W_r[e,h] ) + bias[row(t), e]
             (sum in fp64, rounded once to fp32, fp32 bias added in fp32);
             k picks per token by descending logit, lowest index on ties;
             gates = softmax over the k picked logits (sum to 1);
             counts[e] = number of (token, slot) pairs that picked e -- every
             expert, hosted or not: this is the raw f_n^l(e).
  dispatch   an assignment a = t*k + j is local iff mask[idx[a]] != 0, where
             mask[e] = [ sum_g z_{n,g}^e >= 1 ] (1 - 1_remote).  Local ones are
             bucketed by expert, remote ones likewise, each bucket in
             ascending a.  Bytes to ship = one activation row per remote
             assignment each way.
  expert_ffn y = W_down ( silu(W_gate x) * (W_up x) ), silu(z) = z/(1+e^-z),
             no biases, for every local assignment, and for every
             (token, shared expert).
  combine    out[t] = sum_{local slots j} gate[t,j] * y[(t,j)] + sum_s y_sh[s,t]
             (the aggregation step of Sec. III-A); remote slots contribute
             nothing here (their rows arrive later).
  pack_remote / combine_remote
             the two ends of the remote call: the activation rows shipped for the
             remote list, and the returned expert outputs added, gate-weighted, to
             the local partial sum.  The hosting server's part in between is
             expert_ffn on the shipped rows.

All floating point is fp64 except where stated; the only roundings are the
fp32 logit (+ fp32 bias add), the fp32 gates and the final output rounding to
the layer's I/O dtype.  Inputs are float arrays (bf16 inputs are passed
up-converted, which is exact).

Pins (tests/test_oracle_pins.py): brute-force full-sort routing, k=1 / k=E /
zero-router / duplicated-row / huge-bias closed forms, torch-CPU softmax+topk
on tie-free inputs, histogram and partition invariants, the dense reference
MoE written as a T x E gate matrix, mask-complement additivity, linearity in
W_down, the E=1,k=1 case against torch's SwiGLU MLP, token-permutation
equivariance, hand values for the rounding of the remote combine.  Nothing here is "parity unpinned" except absolute output
values at the large configs, which have no source other than this file.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

__all__ = [
    "route", "dispatch", "expert_ffn", "combine", "moe_layer", "swiglu_rows", "pack_remote",
    "combine_remote",
    "round_to_dtype", "RouteResult", "DispatchResult", "LayerResult",
]


# ---------------------------------------------------------------------------
# rounding to the layer's I/O dtype
# ---------------------------------------------------------------------------

def round_to_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values to fp32, or to bf16 (nearest-even) held in fp32."""
    if dtype == "f32":
        return np.asarray(a, dtype=np.float64).astype(np.float32)
    if dtype != "bf16":
        raise ValueError(dtype)
    # fp64 -> bf16 in one rounding: bf16 keeps 8 significant bits.  Work on the
    # fp64 bit pattern: keep sign, 11 exponent bits and the top 7 mantissa bits.
    a = np.ascontiguousarray(a, dtype=np.float64)
    u = a.view(np.uint64)
    drop = np.uint64(52 - 7)
    half = (np.uint64(1) << (drop - np.uint64(1))) - np.uint64(1)
    lsb = (u >> drop) & np.uint64(1)
    r = ((u + half + lsb) >> drop) << drop
    out = r.view(np.float64)
    # values beyond bf16/fp32 range do not occur for finite layer inputs here
    return out.astype(np.float32)


# ---------------------------------------------------------------------------
# a-1 .. a-3: router, top-k gating, activation counts
# ---------------------------------------------------------------------------

@dataclass
class RouteResult:
    logits: np.ndarray      # [T, E] fp32
    topk_idx: np.ndarray    # [T, k] int32
    topk_gate: np.ndarray   # [T, k] fp32
    counts: np.ndarray      # [E] int32


def route(x: np.ndarray, w_router: np.ndarray, bias: Optional[np.ndarray], k: int,
          bias_group_tokens: int = 0, token_pos: Optional[np.ndarray] = None,
          renormalize: bool = True) -> RouteResult:
    """Gating network of Sec. III-A plus the frequency statistic f_n^l(e) of Sec. III-B.

    x [T,H], w_router [E,H], bias [G,E] fp32 or None.  Token t uses bias row
    pos(t) // bias_group_tokens (row 0 when bias_group_tokens == 0), where
    pos(t) = token_pos[t] if given else t.
    renormalize: gates are the softmax over the k picked logits (they sum to 1);
    otherwise the picked entries of the softmax over all E logits (the two model
    families of Sec. IV differ in this; the paper does not say).
    """
    x64 = np.asarray(x, dtype=np.float64)
    w64 = np.asarray(w_router, dtype=np.float64)
    T, H = x64.shape
    E = w64.shape[0]
    if not (1 <= k <= E):
        raise ValueError("need 1 <= k <= E")
    acc = np.zeros((T, E), dtype=np.float64)
    for h in range(H):                                 # fp64 sum in index order h = 0, 1, ...
        acc += x64[:, h:h + 1] * w64[:, h][None, :]
    logits = acc.astype(np.float32)                    # one rounding
    if bias is not None:
        b = np.asarray(bias, dtype=np.float32).reshape(-1, E)
        pos = np.arange(T) if token_pos is None else np.asarray(token_pos)
        rows = pos // bias_group_tokens if bias_group_tokens > 0 else np.zeros(T, dtype=np.int64)
        logits = (logits + b[rows]).astype(np.float32)  # fp32 add
    idx = np.empty((T, k), dtype=np.int32)
    picked = np.zeros((T, E), dtype=bool)
    tt = np.arange(T)
    for j in range(k):
        cand = np.where(picked, -np.inf, logits.astype(np.float64))
        e = np.argmax(cand, axis=1)                    # first maximum = lowest index
        idx[:, j] = e
        picked[tt, e] = True
    sel = logits[tt[:, None], idx].astype(np.float64)  # [T,k], slot 0 is the maximum
    w = np.exp(sel - sel[:, :1])
    if renormalize:
        denom = w.sum(axis=1, keepdims=True)
    else:
        denom = np.exp(logits.astype(np.float64) - sel[:, :1]).sum(axis=1, keepdims=True)
    gate = (w / denom).astype(np.float32)
    counts = np.zeros(E, dtype=np.int32)
    for t in range(T):
        for j in range(k):
            counts[idx[t, j]] += 1
    return RouteResult(logits, idx, gate, counts)


# ---------------------------------------------------------------------------
# a-4: placement split + stable bucket permutation, remote list, bytes
# ---------------------------------------------------------------------------

@dataclass
class DispatchResult:
    local_src: np.ndarray       # [n_local] int32 flat ids t*k+j, bucketed by expert
    local_offsets: np.ndarray   # [E+1] int32
    remote_src: np.ndarray      # [n_remote] int32
    remote_offsets: np.ndarray  # [E+1] int32
    n_local: int
    n_remote: int
    remote_bytes: np.ndarray    # [2] int64: send, recv


def dispatch(topk_idx: np.ndarray, mask: np.ndarray, hidden: int, elem_size: int) -> DispatchResult:
    """Split assignments by the local/remote indicator of Sec. III-B and bucket them."""
    idx = np.asarray(topk_idx)
    E = int(np.asarray(mask).shape[0])
    flat = idx.reshape(-1)
    loc: List[List[int]] = [[] for _ in range(E)]
    rem: List[List[int]] = [[] for _ in range(E)]
    for a in range(flat.shape[0]):
        e = int(flat[a])
        (loc if mask[e] else rem)[e].append(a)
    local_src = np.array([a for b in loc for a in b], dtype=np.int32)
    remote_src = np.array([a for b in rem for a in b], dtype=np.int32)
    lo = np.zeros(E + 1, dtype=np.int32)
    ro = np.zeros(E + 1, dtype=np.int32)
    for e in range(E):
        lo[e + 1] = lo[e] + len(loc[e])
        ro[e + 1] = ro[e] + len(rem[e])
    R = int(ro[E])
    nbytes = np.array([R * hidden * elem_size, R * hidden * elem_size], dtype=np.int64)
    return DispatchResult(local_src, lo, remote_src, ro, int(lo[E]), R, nbytes)


# ---------------------------------------------------------------------------
# a-5: SwiGLU expert FFN
# ---------------------------------------------------------------------------

def swiglu_rows(xr: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray) -> np.ndarray:
    """y[r] = W_down ( silu(W_gate x[r]) * (W_up x[r]) ) for each row, fp64."""
    xr = np.asarray(xr, dtype=np.float64)
    g = xr @ np.asarray(w_gate, dtype=np.float64).T
    u = xr @ np.asarray(w_up, dtype=np.float64).T
    h = (g / (1.0 + np.exp(-g))) * u
    return h @ np.asarray(w_down, dtype=np.float64).T


def expert_ffn(x: np.ndarray, experts, shared, local_src: np.ndarray, local_offsets: np.ndarray,
               k: int) -> np.ndarray:
    """Rows of y in local_src order, then S blocks of T shared-expert rows.  fp64.

    experts(e) returns (w_gate[F,H], w_up[F,H], w_down[H,F]) as float arrays
    and is called only for experts with a non-empty local segment; shared is
    a sequence of S such triples.
    """
    x = np.asarray(x)
    T, H = x.shape
    n_local = int(local_offsets[-1])
    S = len(shared)
    y = np.zeros((n_local + S * T, H), dtype=np.float64)
    E = len(local_offsets) - 1
    for e in range(E):
        b, en = int(local_offsets[e]), int(local_offsets[e + 1])
        if en == b:
            continue
        tok = np.asarray(local_src[b:en]) // k
        wg, wu, wd = experts(e)
        y[b:en] = swiglu_rows(x[tok], wg, wu, wd)
    for s in range(S):
        wg, wu, wd = shared[s]
        y[n_local + s * T: n_local + (s + 1) * T] = swiglu_rows(x, wg, wu, wd)
    return y


# ---------------------------------------------------------------------------
# a-6: gate-weighted combine
# ---------------------------------------------------------------------------

def combine(y: np.ndarray, local_src: np.ndarray, topk_gate: np.ndarray, T: int, n_shared: int,
            dtype: str) -> np.ndarray:
    """out[t] = sum over local slots (ascending j) of gate*y, then shared rows; one rounding."""
    k = topk_gate.shape[1]
    H = y.shape[1]
    n_local = len(local_src)
    row_of = {int(a): r for r, a in enumerate(local_src)}
    out = np.zeros((T, H), dtype=np.float64)
    for t in range(T):
        for j in range(k):
            r = row_of.get(t * k + j)
            if r is not None:
                out[t] += float(topk_gate[t, j]) * y[r]
        for s in range(n_shared):
            out[t] += y[n_local + s * T + t]
    return round_to_dtype(out, dtype)


# ---------------------------------------------------------------------------
# the remote call (Sec. III-A: the requesting server asks the hosting server and
# aggregates what comes back; Sec. III-B: what is shipped is the activation, the
# hosting server executes the expert, results return)
# ---------------------------------------------------------------------------

def pack_remote(x: np.ndarray, remote_src: np.ndarray, k: int) -> np.ndarray:
    """The activation rows shipped to the hosting servers: row r is the token of remote
    assignment remote_src[r] (flat id t*k + j), in remote-list order."""
    return np.stack([x[int(a) // k] for a in remote_src]) if len(remote_src) else \
        np.zeros((0, x.shape[1]), dtype=x.dtype)


def combine_remote(out_local: np.ndarray, y_remote: np.ndarray, remote_src: np.ndarray,
                   topk_gate: np.ndarray, dtype: str) -> np.ndarray:
    """Adds the returned expert outputs to the local partial sum:
    out[t] = out_local[t] + sum over remote slots (ascending j) of gate[t,j] * y_remote[row(t,j)],
    rounded once more to the layer dtype.  y_remote [R, H] is in remote-list order."""
    k = topk_gate.shape[1]
    out = np.array(out_local, dtype=np.float64)
    row_of = {int(a): r for r, a in enumerate(remote_src)}
    for t in range(out.shape[0]):
        for j in range(k):
            r = row_of.get(t * k + j)
            if r is not None:
                out[t] += float(topk_gate[t, j]) * y_remote[r]
    return round_to_dtype(out, dtype)


# ---------------------------------------------------------------------------
# the whole layer
# ---------------------------------------------------------------------------

@dataclass
class LayerResult:
    route: RouteResult
    dispatch: DispatchResult
    out: np.ndarray             # [T, H] fp32 holding values of the I/O dtype


def moe_layer(x: np.ndarray, w_router: np.ndarray, bias: Optional[np.ndarray], experts,
              shared: Sequence, mask: np.ndarray, k: int, dtype: str,
              bias_group_tokens: int = 0, token_pos: Optional[np.ndarray] = None,
              renormalize: bool = True) -> LayerResult:
    """One server's MoE layer forward: route -> dispatch -> local FFN -> combine."""
    x = np.asarray(x)
    T, H = x.shape
    es = 4 if dtype == "f32" else 2
    r = route(x, w_router, bias, k, bias_group_tokens, token_pos, renormalize)
    d = dispatch(r.topk_idx, mask, H, es)
    y = expert_ffn(x, experts, shared, d.local_src, d.local_offsets, k)
    out = combine(y, d.local_src, r.topk_gate, T, len(shared), dtype)
    return LayerResult(r, d, out)
