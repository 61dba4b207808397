"""The native placement pipeline (host code behind include/prism_placement.h) against the
placement oracle: integer outputs bit for bit, entropy to 1e-12, on seeded instances with the
shapes of the paper's two model families and on adversarial ones (ties, zeros, no room)."""
import numpy as np
import pytest

import paper_2508_12851_amd as P
from paper_2508_12851_amd import placement as NP
from oracle import placement_oracle as PO


def _zipf_counts(rng, N, L, E, s, total):
    f = np.zeros((N, L, E), np.int64)
    for n in range(N):
        for l in range(L):
            w = 1.0 / (rng.permutation(E) + 1.0) ** s
            f[n, l] = rng.multinomial(total, w / w.sum())
    return f


CASES = {
    # (N servers, L layers, E experts, zipf s, observations per (server, layer), memory in experts)
    "mixtral_like": (4, 32, 8, 1.0, 8192, [80, 80, 80, 80]),
    "dsv2_like": (4, 26, 64, 1.0, 49152, [600, 600, 450, 450]),
    "heterogeneous": (3, 6, 60, 1.2, 4000, [300, 120, 40]),
    "tight": (2, 4, 16, 0.8, 500, [34, 33]),
    "no_room": (2, 3, 16, 1.0, 500, [10, 9]),
    "one_server": (1, 5, 12, 1.0, 300, [70]),
}


@pytest.mark.parametrize("case", list(CASES))
def test_pipeline_matches_oracle(case):
    N, L, E, s, total, mem = CASES[case]
    rng = np.random.default_rng(sum(map(ord, case)))
    f = _zipf_counts(rng, N, L, E, s, total)
    v_ref, cnt_ref, place_ref, ok_ref = PO.placement_plan(f, mem, 1.0)
    v, cnt, place, ok = NP.placement_plan(f, mem, 1.0)
    assert np.max(np.abs(v - v_ref)) <= 1e-12
    assert np.array_equal(cnt, cnt_ref) and np.array_equal(place, place_ref) and ok == ok_ref
    # the steps one by one give the same as the pipeline
    assert np.max(np.abs(NP.activation_entropy(f) - v_ref)) <= 1e-12
    c2, feasible = NP.expert_count_allocation(v_ref, mem, 1.0, E)
    p2, covered = NP.expert_assignment(f, cnt_ref)
    assert np.array_equal(c2, cnt_ref) and np.array_equal(p2, place_ref)
    assert (feasible and covered) == ok_ref
    assert NP.proxy_cost(f, place) == PO.proxy_cost(f, place_ref)
    print(f"{case}: ok={ok}, proxy cost {NP.proxy_cost(f, place)} of {int(f.sum())} activations")


@pytest.mark.parametrize("seed", range(12))
def test_random_small_instances_with_many_ties(seed):
    rng = np.random.default_rng(seed)
    N, L, E = int(rng.integers(1, 5)), int(rng.integers(1, 5)), int(rng.integers(1, 12))
    f = rng.integers(0, 4, size=(N, L, E))                    # few distinct values: ties everywhere
    if seed % 3 == 0:
        f[rng.integers(0, N)] = 0                             # a server without observations
    mem = rng.integers(1, 2 * E * L + 2, size=N).astype(float)
    if seed % 4 == 0:
        mem[:] = mem[0]                                       # equal memories: index order
    m_e = float(rng.choice([1.0, 0.5, 3.0]))
    ref = PO.placement_plan(f, mem, m_e)
    got = NP.placement_plan(f, mem, m_e)
    assert np.max(np.abs(got[0] - ref[0])) <= 1e-12
    assert np.array_equal(got[1], ref[1]) and np.array_equal(got[2], ref[2]) and got[3] == ref[3]
    # assignment alone, with arbitrary counts (not only those Alg. 1 produces)
    cnt = rng.integers(0, E + 1, size=(N, L))
    p_ref, c_ref = PO.assignment(f, cnt)
    p_got, c_got = NP.expert_assignment(f, cnt)
    assert np.array_equal(p_got, p_ref) and c_got == c_ref


HAND_ALLOC = [
    # (v, memory, E, expected N_{n,l}, feasible) -- the hand-worked cases of the oracle's pins
    ([[1.0, 1.0], [1.0, 3.0]], [4.0, 4.0], 4, [[3, 1], [1, 3]], True),
    ([[1.0, 3.0, 4.0], [1.0, 3.0, 4.0]], [8.0, 8.0], 4, [[2, 3, 3], [2, 3, 3]], True),
    ([[2.0, 7.0, 7.0], [2.0, 7.0, 7.0]], [8.0, 8.0], 4, [[2, 2, 3], [2, 3, 2]], True),
    ([[1.0, 2.0, 1.0]], [4.0], 2, [[1, 2, 1]], False),
    ([[0.0, 1.0, 0.0], [1.0, 0.0, 7.0], [0.0, 0.0, 1.0]], [8.0, 8.0, 4.0], 3,
     [[0, 3, 0], [2, 0, 2], [1, 0, 2]], True),
]


@pytest.mark.parametrize("case", range(len(HAND_ALLOC)))
def test_native_count_allocation_on_hand_worked_cases(case):
    v, mem, E, want, feasible = HAND_ALLOC[case]
    cnt, ok = NP.expert_count_allocation(np.array(v), mem, 1.0, E)
    assert cnt.tolist() == want and ok == feasible


def test_native_assignment_on_hand_worked_cases():
    place, _ = NP.expert_assignment(np.array([[[5, 5, 1]]], np.int64), np.array([[1]]))
    assert place[0, 0].tolist() == [1, 0, 0]
    f = np.array([[[9, 8, 1, 0]], [[9, 8, 7, 1]], [[1, 2, 9, 3]]], np.int64)
    place, covered = NP.expert_assignment(f, np.array([[2], [3], [1]]))
    assert covered and place[:, 0].tolist() == [[1, 1, 0, 0], [1, 1, 1, 0], [0, 0, 0, 1]]
    f = np.array([[[10, 8, 1, 0]], [[9, 7, 5, 2]]], np.int64)
    place, covered = NP.expert_assignment(f, np.array([[2], [2]]))
    assert covered and place[:, 0].tolist() == [[1, 0, 1, 0], [0, 1, 0, 1]]


def test_costs_and_migration_rule_match_oracle():
    rng = np.random.default_rng(3)
    N, L, E = 3, 4, 20
    f = rng.integers(0, 1000, size=(N, L, E))
    old = (rng.random((N, L, E)) < 0.5).astype(np.uint8)
    new = (rng.random((N, L, E)) < 0.5).astype(np.uint8)
    speed = [10.0, 25.0, 3.0]
    assert NP.proxy_cost(f, old) == PO.proxy_cost(f, old)
    s_ref, k_ref = PO.migration_cost(old, new, 17.3, speed)
    s_got, k_got = NP.migration_cost(old, new, 17.3, speed)
    assert k_got == k_ref and s_got == pytest.approx(s_ref, rel=1e-12)
    for t_mig in (0.0, 1.0, 1e3, 1e9):
        for spr in (0.0, 1e-3, 0.5):
            a, b = PO.proxy_cost(f, old), PO.proxy_cost(f, new)
            assert NP.migration_decision(a, b, t_mig, spr) == PO.should_migrate(a, b, t_mig, spr)
            assert NP.migration_decision(b, a, t_mig, spr) == PO.should_migrate(b, a, t_mig, spr)


def test_invalid_arguments_are_refused():
    f = np.ones((2, 2, 4), np.int64)
    with pytest.raises(P.PrismError):
        NP.activation_entropy(-f)                                   # negative counts
    with pytest.raises(P.PrismError):
        NP.placement_plan(f, [4.0, 0.0], 1.0)                       # a server without memory
    with pytest.raises(P.PrismError):
        NP.placement_plan(f, [4.0, 4.0], 0.0)                       # expert size 0
    with pytest.raises(P.PrismError):
        NP.expert_assignment(f, np.full((2, 2), 5))                 # more experts than the layer has
    with pytest.raises(P.PrismError):
        NP.migration_cost(np.zeros((1, 1, 2), np.uint8), np.zeros((1, 1, 2), np.uint8), 1.0, [0.0])
    with pytest.raises(P.PrismError):
        NP.migration_decision(-1, 0, 0.0, 1.0)
