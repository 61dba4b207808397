"""Seeded input generator for the placement-aware MoE layer workloads.

Recipe (every tensor has its own child stream ``SeedSequence([seed, id])`` so
any tensor can be regenerated alone):

* tokens ``x ~ N(0, 1)``; router and expert weights ``~ N(0, 1/H)``, so raw
  router logits are roughly N(0, 1);
* popularity bias: a seeded permutation gives every expert a rank
  ``r(e) in 1..E`` and ``bias[e] = -s * ln r(e)`` -- added to N(0, 1) logits
  this produces a Zipf(s)-like skew of expert popularity (the skew of
  Fig. 2 of the paper); with ``bias_group_tokens > 0`` every block of that
  many tokens gets its own permutation (per-request locality);
* placement mask (the per-server collapse of ``z_{n,g}^e``, Sec. III-B):
  either given explicitly, or the ``n_local`` most popular experts (what the
  first loop of Alg. 2 would host), or a seeded uniformly random subset;
* values are drawn in fp32; for bf16 configs they are rounded to nearest-even
  bf16 once and stored as ``uint16`` bit patterns.  Every consumer sees the
  rounded values.

Nothing in this file computes any step of the layer.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

# --------------------------------------------------------------------------
# bf16 storage helpers (format conversion only)
# --------------------------------------------------------------------------


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (round-to-nearest-even), return uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact up-conversion of bf16 bit patterns to fp32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# configuration
# --------------------------------------------------------------------------

_ID_X = 0
_ID_ROUTER = 1
_ID_RANKS = 2
_ID_MASK = 3
_ID_EVICT = 4
_ID_EXPERT0 = 1000       # + 3*e + {0: gate, 1: up, 2: down}
_ID_SHARED0 = 100000     # + 3*s + {0,1,2}


@dataclass(frozen=True)
class LayerConfig:
    name: str
    dtype: str                      # "f32" | "bf16"
    T: int                          # tokens in the batch
    H: int                          # hidden size
    E: int                          # routed experts
    F: int                          # expert FFN dim
    k: int                          # top-k
    S: int = 0                      # shared (always-on) experts
    n_local: int = 0                # hosted routed experts ("hosts L of E")
    zipf_s: float = 1.0
    bias_group_tokens: int = 0      # 0: one bias row for all tokens
    seed: int = 0                   # weights (and everything else by default)
    tokens_seed: Optional[int] = None
    mask_kind: str = "top"          # "top" | "random" | "given"
    mask_given: Tuple[int, ...] = ()
    n_phases: int = 1
    n_swapped: int = 0              # experts swapped between phase 0 and 1

    @property
    def es(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def A(self) -> int:
        return self.T * self.k

    @property
    def n_bias_rows(self) -> int:
        if self.bias_group_tokens <= 0:
            return 1
        return (self.T + self.bias_group_tokens - 1) // self.bias_group_tokens


CONFIGS: Dict[str, LayerConfig] = {
    # Tiny fp32 layer; mask {0,2,5,7}.
    "cfg1_tiny_f32": LayerConfig("cfg1_tiny_f32", "f32", T=64, H=256, E=8, F=512, k=2,
                                 n_local=4, zipf_s=1.0, seed=0, mask_kind="given",
                                 mask_given=(0, 2, 5, 7)),
    # Mixtral-8x7B-shaped prefill batch.
    "cfg2_mixtral_prefill": LayerConfig("cfg2_mixtral_prefill", "bf16", T=4096, H=4096, E=8,
                                        F=14336, k=2, n_local=5, zipf_s=1.0, seed=1),
    # Same layer (same weights), decode batch.
    "cfg3_mixtral_decode": LayerConfig("cfg3_mixtral_decode", "bf16", T=32, H=4096, E=8,
                                       F=14336, k=2, n_local=5, zipf_s=1.0, seed=1,
                                       tokens_seed=2),
    # Fine-grained experts + shared experts, per-512-token popularity ranking.
    "cfg4_finegrained": LayerConfig("cfg4_finegrained", "bf16", T=8192, H=2048, E=60, F=1408,
                                    k=4, S=4, n_local=36, zipf_s=1.2, bias_group_tokens=512,
                                    seed=3),
    # DeepSeek-V2-Lite-shaped, two phases with a mask change (migration scenario).
    "cfg5_dsv2lite_migration": LayerConfig("cfg5_dsv2lite_migration", "bf16", T=8192, H=2048,
                                           E=64, F=1408, k=6, S=2, n_local=32, zipf_s=1.0,
                                           seed=4, n_phases=2, n_swapped=16),
}


def make_config(name: str, **overrides) -> LayerConfig:
    """A named config, optionally shrunk/changed (tests use scaled-down shapes)."""
    return dataclasses.replace(CONFIGS[name], **overrides)


# --------------------------------------------------------------------------
# pieces
# --------------------------------------------------------------------------


def _rng(seed: int, tensor_id: int, sub: int = 0) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([int(seed), int(tensor_id), int(sub)]))


def zipf_bias(ranks: np.ndarray, s: float) -> np.ndarray:
    """bias[e] = -s * ln(rank(e)), rank 1 = most popular.  fp32."""
    return (-float(s) * np.log(ranks.astype(np.float64))).astype(np.float32)


def top_popular_mask(ranks_rows: np.ndarray, s: float, n_local: int) -> np.ndarray:
    """uint8[E] mask of the n_local experts with the largest expected popularity.

    Expected popularity of expert e in a bias row is proportional to
    rank(e)^-s; rows are averaged.  Ties go to the lowest index.
    """
    ranks_rows = np.atleast_2d(ranks_rows)
    pop = ranks_rows.astype(np.float64) ** (-float(s))
    pop = pop / pop.sum(axis=1, keepdims=True)
    mean_pop = pop.mean(axis=0)
    E = mean_pop.shape[0]
    order = sorted(range(E), key=lambda e: (-mean_pop[e], e))
    mask = np.zeros(E, dtype=np.uint8)
    mask[order[:n_local]] = 1
    return mask


def random_mask(seed: int, E: int, n_local: int) -> np.ndarray:
    """uint8[E] mask of a seeded uniformly random n_local-subset."""
    mask = np.zeros(E, dtype=np.uint8)
    mask[_rng(seed, _ID_MASK).permutation(E)[:n_local]] = 1
    return mask


def _store(a32: np.ndarray, dtype: str) -> np.ndarray:
    return a32 if dtype == "f32" else f32_to_bf16_bits(a32)


def _normal(seed: int, tid: int, shape, std: float, dtype: str, sub: int = 0) -> np.ndarray:
    a = _rng(seed, tid, sub).standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return _store(a, dtype)


# --------------------------------------------------------------------------
# the bundle
# --------------------------------------------------------------------------


@dataclass
class LayerInputs:
    """All tensors of one call of the layer.

    Storage dtype: float32 for "f32" configs, uint16 bf16 bit patterns for
    "bf16" configs (``f32(arr)`` up-converts exactly).  Expert weights are
    generated on demand and cached: ``expert(e)`` -> (w_gate[F,H], w_up[F,H],
    w_down[H,F]); ``shared(s)`` likewise.
    """
    cfg: LayerConfig
    phase: int
    x: np.ndarray                   # [T, H]
    w_router: np.ndarray            # [E, H]
    ranks: np.ndarray               # [G, E] int64, 1 = most popular
    bias: np.ndarray                # [G, E] fp32
    mask: np.ndarray                # [E] uint8
    _experts: Dict[int, Tuple[np.ndarray, np.ndarray, np.ndarray]] = field(default_factory=dict)
    _shared: Dict[int, Tuple[np.ndarray, np.ndarray, np.ndarray]] = field(default_factory=dict)

    def f32(self, a: np.ndarray) -> np.ndarray:
        return a if a.dtype == np.float32 else bf16_bits_to_f32(a)

    def _triple(self, base_id: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        c = self.cfg
        std = float(c.H) ** -0.5
        wg = _normal(c.seed, base_id + 0, (c.F, c.H), std, c.dtype)
        wu = _normal(c.seed, base_id + 1, (c.F, c.H), std, c.dtype)
        wd = _normal(c.seed, base_id + 2, (c.H, c.F), std, c.dtype)
        return wg, wu, wd

    def expert(self, e: int):
        if e not in self._experts:
            self._experts[e] = self._triple(_ID_EXPERT0 + 3 * e)
        return self._experts[e]

    def shared(self, s: int):
        if s not in self._shared:
            self._shared[s] = self._triple(_ID_SHARED0 + 3 * s)
        return self._shared[s]

    def materialize(self, experts: Optional[List[int]] = None, threads: int = 8) -> None:
        """Generate (in parallel) the listed routed experts and all shared ones."""
        c = self.cfg
        if experts is None:
            experts = list(range(c.E))
        jobs = [("e", e) for e in experts if e not in self._experts]
        jobs += [("s", s) for s in range(c.S) if s not in self._shared]
        if not jobs:
            return

        def run(job):
            kind, i = job
            return job, self._triple((_ID_EXPERT0 if kind == "e" else _ID_SHARED0) + 3 * i)

        with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
            for (kind, i), tri in ex.map(run, jobs):
                (self._experts if kind == "e" else self._shared)[i] = tri

    def drop_weights(self) -> None:
        self._experts.clear()
        self._shared.clear()


def _ranks_for(cfg: LayerConfig, phase: int) -> np.ndarray:
    G = cfg.n_bias_rows
    rows = []
    for g in range(G):
        perm = _rng(cfg.seed, _ID_RANKS, phase * 100003 + g).permutation(cfg.E)
        ranks = np.empty(cfg.E, dtype=np.int64)
        ranks[perm] = np.arange(1, cfg.E + 1)
        rows.append(ranks)
    return np.stack(rows)


def _mask_for(cfg: LayerConfig, phase: int, ranks_by_phase: List[np.ndarray]) -> np.ndarray:
    if cfg.mask_kind == "given":
        m = np.zeros(cfg.E, dtype=np.uint8)
        m[list(cfg.mask_given)] = 1
        return m
    if cfg.mask_kind == "random":
        return random_mask(cfg.seed, cfg.E, cfg.n_local)
    m0 = top_popular_mask(ranks_by_phase[0], cfg.zipf_s, cfg.n_local)
    if phase == 0:
        return m0
    # Phase 1 of the migration scenario: evict n_swapped seeded members of the
    # phase-0 mask and host instead the n_swapped non-members that are most
    # popular under the phase-1 ranking.
    members = np.flatnonzero(m0)
    evict = _rng(cfg.seed, _ID_EVICT).permutation(members)[: cfg.n_swapped]
    non_members = [e for e in range(cfg.E) if not m0[e]]
    r1 = ranks_by_phase[1].astype(np.float64) ** (-float(cfg.zipf_s))
    pop1 = (r1 / r1.sum(axis=1, keepdims=True)).mean(axis=0)
    non_members.sort(key=lambda e: (-pop1[e], e))
    m1 = m0.copy()
    m1[evict] = 0
    m1[non_members[: cfg.n_swapped]] = 1
    return m1


def make_inputs(cfg, phase: int = 0, weights: Optional[str] = None,
                threads: int = 8) -> LayerInputs:
    """Draw one call's inputs.

    cfg      a LayerConfig or the name of one in CONFIGS
    phase    0, or 1 for the second phase of a two-phase (migration) config:
             fresh tokens, fresh popularity ranking, changed mask, same weights
    weights  None: expert weights stay lazy; "local": generate hosted + shared
             experts now; "all": generate every expert now
    """
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    if not (0 <= phase < cfg.n_phases):
        raise ValueError(f"phase {phase} outside 0..{cfg.n_phases - 1}")
    tseed = cfg.seed if cfg.tokens_seed is None else cfg.tokens_seed
    x = _normal(tseed, _ID_X, (cfg.T, cfg.H), 1.0, cfg.dtype, sub=phase)
    w_router = _normal(cfg.seed, _ID_ROUTER, (cfg.E, cfg.H), float(cfg.H) ** -0.5, cfg.dtype)
    ranks_by_phase = [_ranks_for(cfg, p) for p in range(phase + 1)]
    ranks = ranks_by_phase[phase]
    bias = np.stack([zipf_bias(r, cfg.zipf_s) for r in ranks])
    mask = _mask_for(cfg, phase, ranks_by_phase)
    inp = LayerInputs(cfg=cfg, phase=phase, x=x, w_router=w_router, ranks=ranks, bias=bias,
                      mask=mask)
    if weights == "local":
        inp.materialize([int(e) for e in np.flatnonzero(mask)], threads)
    elif weights == "all":
        inp.materialize(None, threads)
    elif weights is not None:
        raise ValueError("weights must be None, 'local' or 'all'")
    return inp
