"""Plain CPU oracle for the scheduler-side placement pipeline that consumes the
activation counts the MoE layer emits.

THIS IS TEST INFRASTRUCTURE.  Only the test-suite may import it; the product
(the native library and its binding) never does, and shares no code with it.

What it computes (paper: Prism, Sec. III-C "Activation-Aware Expert Placement"):

  entropy            v_{n,l} = - sum_e p_e log2 p_e,  p_e = f_n^l(e) / sum_e' f_n^l(e')
                     (the formula printed with Alg. 1; plain Shannon entropy in bits)
  count_allocation   Alg. 1: N_{n,l} = floor( M_n / m_e * v_{n,l} / sum_l v_{n,l} ), then
                     layers whose total over the servers is below E borrow, one
                     expert at a time, from the layer with the largest total, on
                     servers visited in order of descending memory
  assignment         Alg. 2: every server takes its N_{n,l} most frequent experts of
                     layer l; experts nobody holds are then placed on servers that
                     hold duplicates, fewest duplicates first, replacing the
                     server's least used duplicate
  proxy_cost         Eq. 2: sum over servers, layers, experts of f_n^l(e) * 1_remote(n, e)
  migration_cost     Eq. 3: sum over changed placement entries of m_e / speed
  should_migrate     Eq. 4: adopt P' iff C(P') + T_mig(P, P') < C(P)

The algorithms are iterations whose result depends on the order of their steps,
so the functions below take the steps in the paper's order, with plain loops.
Readings where the listings are silent or loose (each also listed in the design
notes of the repository):

  R1  p log2 p = 0 for p = 0.  A (server, layer) without any observation has
      v = 0; a server whose entropies are all 0 splits its memory evenly over the
      layers (the printed ratio would be 0/0).
  R2  N_{n,l} is capped at E (a server cannot hold more than the E distinct experts
      of a layer); the printed formula has no cap.
  R3  Alg. 1, step 2: the donor layer l' is the layer with the largest total AMONG
      layers other than l that are over-provisioned (total > E), lowest index on
      ties; the printed arg max could return l itself or strip a layer below E.
      It is chosen afresh for every server visited, as printed.  A server gives
      only if it has N_{n,l'} > 0 (printed) and N_{n,l} < E (R2).  If a whole pass
      over the servers moves nothing the layer stays short (infeasible input); the
      printed loop would not end.  Servers of equal memory keep index order.
  R4  Preference order: descending f_n^l(e), lower expert index first on ties.
  R5  Alg. 2: a "duplicate" in A_n^l is an expert that at least one other server
      holds too (replacing it cannot uncover anything).  Servers are sorted by
      their number of duplicates once per pass of the while loop (printed), ties
      by index; servers without duplicates are skipped.  The candidate is the
      unassigned expert most frequent ON THAT SERVER (printed), lower index on
      ties; the replaced one is that server's least frequent duplicate, HIGHER
      index on ties (the tail of its preference list).  U_l and the duplicate sets
      are updated after every replacement (the listing updates U_l only after the
      pass, which would let several servers take the same expert in one pass while
      others stay uncovered).  A pass without a replacement ends the loop.
  R6  Eq. 3 is evaluated on the server-level indicator sum_g z_{n,g}^e >= 1 (what
      the layer's mask holds) with one speed per server, and counts every entry
      that differs, removals as well as additions, as printed (the primed symbol
      in the printed indicator is read as the entry of P').
  R7  Eq. 4 compares a count with a time.  Sec. IV-A ("System Parameter
      Settings") says historical communication and computation time of expert
      execution are used as estimation metrics for the cost of a new placement: C
      is multiplied by seconds_per_remote_call before the comparison.

Pins (tests/test_placement_pins.py): entropy closed forms (uniform -> log2 E,
one-hot -> 0, two equal halves -> 1 bit, scale invariance) and the chain rule
against scipy; Alg. 1 on hand-worked examples (visiting order, which layer gives,
ties, a fresh choice per server, layers at exactly E, servers without the donor
layer) and its conservation laws (a
server's total over layers never changes in step 2; totals reach E when the
memory suffices); Alg. 2's top-N property, set sizes, coverage, brute-force
optimality of the unrepaired choice for Eq. 2, and hand-worked repairs; Eq. 2
against a direct count of remote assignments; Eq. 3 on the 16-expert swap of the
migration workload (32 flips); Eq. 4 on both sides of the threshold.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np

__all__ = ["entropy", "count_allocation", "assignment", "proxy_cost", "migration_cost",
           "should_migrate", "placement_plan"]


def entropy(f: np.ndarray) -> np.ndarray:
    """f [N, L, E] activation counts -> v [N, L] in bits (formula printed with Alg. 1; R1)."""
    f = np.asarray(f)
    N, L, E = f.shape
    v = np.zeros((N, L), dtype=np.float64)
    for n in range(N):
        for l in range(L):
            total = float(sum(int(c) for c in f[n, l]))
            if total == 0.0:
                continue
            h = 0.0
            for e in range(E):
                c = int(f[n, l, e])
                if c > 0:
                    p = c / total
                    h -= p * math.log2(p)
            v[n, l] = h
    return v


def count_allocation(v: np.ndarray, server_mem: Sequence[float], expert_mem: float,
                     E: int) -> Tuple[np.ndarray, bool]:
    """Alg. 1.  v [N, L], server_mem M_n, expert_mem m_e -> (N_{n,l} [N, L] int, feasible)."""
    v = np.asarray(v, dtype=np.float64)
    N, L = v.shape
    cnt = np.zeros((N, L), dtype=np.int64)
    # Step 1: initialisation in proportion to the activation diversity
    for n in range(N):
        vsum = float(sum(v[n, l] for l in range(L)))
        for l in range(L):
            share = (v[n, l] / vsum) if vsum > 0.0 else 1.0 / L          # R1
            cnt[n, l] = min(E, int(math.floor(server_mem[n] / expert_mem * share)))   # R2
    # Step 2: adjust to the expert-coverage constraint
    total = [int(sum(cnt[n, l] for n in range(N))) for l in range(L)]
    order = sorted(range(N), key=lambda n: (-server_mem[n], n))
    feasible = True
    for l in range(L):
        while total[l] < E:
            moved = False
            for n in order:
                donors = [lp for lp in range(L) if lp != l and total[lp] > E]        # R3
                if not donors:
                    break
                lp = max(donors, key=lambda j: (total[j], -j))
                if cnt[n, lp] > 0 and cnt[n, l] < E:
                    cnt[n, lp] -= 1
                    cnt[n, l] += 1
                    total[lp] -= 1
                    total[l] += 1
                    moved = True
                    if total[l] == E:
                        break
            if not moved:
                feasible = False
                break
    return cnt, feasible


def _preference(f_nl: np.ndarray) -> List[int]:
    """Experts by descending frequency, lower index first on ties (R4)."""
    return sorted(range(len(f_nl)), key=lambda e: (-int(f_nl[e]), e))


def assignment(f: np.ndarray, cnt: np.ndarray) -> Tuple[np.ndarray, bool]:
    """Alg. 2.  f [N, L, E], N_{n,l} [N, L] -> (placement [N, L, E] uint8, all experts covered)."""
    f = np.asarray(f)
    N, L, E = f.shape
    place = np.zeros((N, L, E), dtype=np.uint8)
    for n in range(N):
        for l in range(L):
            for e in _preference(f[n, l])[: int(cnt[n, l])]:
                place[n, l, e] = 1
    covered = True
    for l in range(L):
        def holders(e):
            return sum(int(place[n, l, e]) for n in range(N))

        unassigned = [e for e in range(E) if holders(e) == 0]
        while unassigned:
            def duplicates(n):                                            # R5
                return [e for e in range(E) if place[n, l, e] and holders(e) >= 2]

            order = sorted(range(N), key=lambda n: (len(duplicates(n)), n))
            replaced = False
            for n in order:
                if not unassigned:
                    break
                dup = duplicates(n)
                if not dup:
                    continue
                e_new = min(unassigned, key=lambda e: (-int(f[n, l, e]), e))
                e_rep = min(dup, key=lambda e: (int(f[n, l, e]), -e))
                place[n, l, e_rep] = 0
                place[n, l, e_new] = 1
                unassigned.remove(e_new)
                replaced = True
            if not replaced:
                covered = False
                break
    return place, covered


def proxy_cost(f: np.ndarray, place: np.ndarray) -> int:
    """Eq. 2: activations of experts the requesting server does not hold."""
    f = np.asarray(f)
    N, L, E = f.shape
    cost = 0
    for n in range(N):
        for l in range(L):
            for e in range(E):
                if not place[n, l, e]:
                    cost += int(f[n, l, e])
    return cost


def migration_cost(old: np.ndarray, new: np.ndarray, expert_mem: float,
                   speed: Sequence[float]) -> Tuple[float, int]:
    """Eq. 3 on server-level placements (R6): (seconds, number of differing entries)."""
    N, L, E = old.shape
    seconds = 0.0
    flips = 0
    for n in range(N):
        for l in range(L):
            for e in range(E):
                if bool(old[n, l, e]) != bool(new[n, l, e]):
                    flips += 1
                    seconds += expert_mem / speed[n]
    return seconds, flips


def should_migrate(cost_old: int, cost_new: int, t_mig: float,
                   seconds_per_remote_call: float) -> bool:
    """Eq. 4 with both sides in seconds (R7)."""
    return cost_new * seconds_per_remote_call + t_mig < cost_old * seconds_per_remote_call


def placement_plan(f: np.ndarray, server_mem: Sequence[float], expert_mem: float):
    """Entropy -> Alg. 1 -> Alg. 2."""
    E = np.asarray(f).shape[2]
    v = entropy(f)
    cnt, feasible = count_allocation(v, server_mem, expert_mem, E)
    place, covered = assignment(f, cnt)
    return v, cnt, place, feasible and covered
