"""Pins of the placement oracle (oracle/placement_oracle.py) against what the paper and the
mathematics fix: closed forms of the entropy, hand-worked runs of Alg. 1 and Alg. 2,
conservation laws, brute force on tiny instances, and the link between Eq. 2 and the
layer's own remote count."""
import itertools
import math

import numpy as np
import pytest
from scipy.stats import entropy as scipy_entropy

from oracle import placement_oracle as PO
from oracle import prism_oracle as O
from prism_inputs import CONFIGS, make_config, make_inputs


# ---------------------------------------------------------------------------
# entropy (formula printed with Alg. 1)
# ---------------------------------------------------------------------------

def test_entropy_closed_forms():
    f = np.zeros((1, 5, 8), np.int64)
    f[0, 0] = 7                     # uniform over 8 experts -> log2 8 = 3 bits
    f[0, 1, 3] = 100                # one expert takes everything -> 0
    f[0, 2, :2] = 50                # two equal halves -> 1 bit
    f[0, 3] = [4, 2, 1, 1, 0, 0, 0, 0]   # 1/2, 1/4, 1/8, 1/8 -> 1.75 bits
    # row 4 stays empty -> 0 by the stated reading
    v = PO.entropy(f)
    assert v.shape == (1, 5)
    assert v[0].tolist() == pytest.approx([3.0, 0.0, 1.0, 1.75, 0.0], abs=1e-15)


def test_entropy_scale_invariance_bounds_and_library_value():
    rng = np.random.default_rng(0)
    f = rng.integers(0, 1000, size=(3, 4, 60))
    v = PO.entropy(f)
    assert np.allclose(PO.entropy(7 * f), v, atol=1e-12)
    assert np.all(v >= 0) and np.all(v <= math.log2(60) + 1e-12)
    for n in range(3):
        for l in range(4):
            assert v[n, l] == pytest.approx(scipy_entropy(f[n, l], base=2), abs=1e-12)


def test_entropy_grouping_rule():
    """H(p) = H(group masses) + sum_g mass_g H(p within g): fails for a wrong log base or sign."""
    f = np.array([[[6, 2, 3, 1, 4]]], np.int64)
    whole = PO.entropy(f)[0, 0]
    g = PO.entropy(np.array([[[8, 8]]], np.int64))[0, 0]          # masses {6,2} and {3,1,4}
    a = PO.entropy(np.array([[[6, 2]]], np.int64))[0, 0]
    b = PO.entropy(np.array([[[3, 1, 4]]], np.int64))[0, 0]
    assert whole == pytest.approx(g + 0.5 * a + 0.5 * b, abs=1e-14)


# ---------------------------------------------------------------------------
# Alg. 1
# ---------------------------------------------------------------------------

def test_count_allocation_hand_worked_borrow():
    # E = 4, two servers with room for 4 experts each.  Step 1: server 0 splits 1:1 -> [2, 2];
    # server 1 splits 1:3 -> [1, 3].  Layer totals [3, 5]: layer 0 borrows one expert from
    # layer 1 on the first server visited (server 0): [[3, 1], [1, 3]].
    cnt, ok = PO.count_allocation(np.array([[1.0, 1.0], [1.0, 3.0]]), [4.0, 4.0], 1.0, E=4)
    assert ok and cnt.tolist() == [[3, 1], [1, 3]]


def test_count_allocation_visits_the_larger_server_first():
    # same entropies, but server 1 has more memory and is visited first.  Step 1: server 0 (room
    # for 4) -> [2, 2]; server 1 (room for 8) -> [2, 6] capped to [2, 4] (E = 4).  Totals [4, 6]:
    # nothing short.  With E = 5: cap 5 -> [2, 5], totals [4, 7]; layer 0 takes one from layer 1
    # on server 1.
    v = np.array([[1.0, 1.0], [1.0, 3.0]])
    cnt, ok = PO.count_allocation(v, [4.0, 8.0], 1.0, E=4)
    assert ok and cnt.tolist() == [[2, 2], [2, 4]]
    cnt, ok = PO.count_allocation(v, [4.0, 8.0], 1.0, E=5)
    assert ok and cnt.tolist() == [[2, 2], [3, 4]]


def test_count_allocation_three_layers_hand_worked():
    # shares 1/6, 1/6, 4/6 of room for 6 -> [1, 1, 4] on both servers, totals [2, 2, 8], E = 4.
    # layer 0: server 0 then server 1 each move one from layer 2 -> totals [4, 2, 6];
    # layer 1: the same again -> [[2, 2, 2], [2, 2, 2]].
    v = np.array([[1.0, 1.0, 4.0], [1.0, 1.0, 4.0]])
    cnt, ok = PO.count_allocation(v, [6.0, 6.0], 1.0, E=4)
    assert ok and cnt.tolist() == [[2, 2, 2], [2, 2, 2]]


def test_count_allocation_infeasible_and_degenerate_inputs():
    # room for 8 experts in total, 2 layers x 5 experts needed: no layer is over-provisioned
    cnt, ok = PO.count_allocation(np.ones((2, 2)), [2.0, 6.0], 1.0, E=5)
    assert not ok and cnt.tolist() == [[1, 1], [3, 3]]
    # all-zero entropies: even split (stated reading)
    cnt, ok = PO.count_allocation(np.zeros((1, 4)), [8.0], 1.0, E=2)
    assert ok and cnt.tolist() == [[2, 2, 2, 2]]
    # expert size scales the room: 10 units of memory / 2.5 per expert = 4 experts
    cnt, _ = PO.count_allocation(np.ones((1, 2)), [10.0], 2.5, E=8)
    assert cnt.tolist() == [[2, 2]]


def test_count_allocation_donor_is_the_largest_over_provisioned_layer():
    # two servers with room for 8 and shares 1/8, 3/8, 4/8 -> [1, 3, 4] each, totals [2, 6, 8]; E = 4:
    # layer 0 is short by two and both other layers have spare experts.  Server 0: layer 2 (8 > 6)
    # gives -> totals [3, 6, 7]; server 1: layer 2 again (7 > 6).
    v = np.array([[1.0, 3.0, 4.0], [1.0, 3.0, 4.0]])
    cnt, ok = PO.count_allocation(v, [8.0, 8.0], 1.0, E=4)
    assert ok and cnt.tolist() == [[2, 3, 3], [2, 3, 3]]


def test_count_allocation_donor_is_chosen_afresh_for_every_server():
    # shares 2/16, 7/16, 7/16 of room for 8 -> [1, 3, 3] on both servers, totals [2, 6, 6], E = 4:
    # layer 0 is short by two.  Server 0: equal totals, the lower layer index (1) gives -> totals
    # [3, 5, 6]; server 1: now layer 2 is the largest.
    v = np.array([[2.0, 7.0, 7.0], [2.0, 7.0, 7.0]])
    cnt, ok = PO.count_allocation(v, [8.0, 8.0], 1.0, E=4)
    assert ok and cnt.tolist() == [[2, 2, 3], [2, 3, 2]]


def test_count_allocation_a_layer_with_exactly_E_does_not_give():
    # [1, 2, 1] with E = 2: layers 0 and 2 are short, layer 1 has exactly E and nothing to spare
    cnt, ok = PO.count_allocation(np.array([[1.0, 2.0, 1.0]]), [4.0], 1.0, E=2)
    assert not ok and cnt.tolist() == [[1, 2, 1]]


def test_count_allocation_a_server_without_the_donor_layer_is_passed_over():
    # E = 3.  Step 1: server 0 (room 8) -> [0, 3, 0] (capped), server 1 (room 8, shares 1/8, 0, 7/8)
    # -> [1, 0, 3] (capped), server 2 (room 4) -> [0, 0, 3] (capped).  Totals [1, 3, 6]: layer 0
    # needs two, only layer 2 has spare ones.  Visiting order 0, 1, 2: server 0 holds nothing of
    # layer 2 and is passed over, servers 1 and 2 move one each.
    v = np.array([[0.0, 1.0, 0.0], [1.0, 0.0, 7.0], [0.0, 0.0, 1.0]])
    cnt, ok = PO.count_allocation(v, [8.0, 8.0, 4.0], 1.0, E=3)
    assert ok and cnt.tolist() == [[0, 3, 0], [2, 0, 2], [1, 0, 2]]


@pytest.mark.parametrize("seed", range(6))
def test_count_allocation_conservation_laws(seed):
    rng = np.random.default_rng(seed)
    N, L, E = int(rng.integers(1, 5)), int(rng.integers(1, 7)), int(rng.integers(2, 20))
    v = rng.random((N, L)) * 4
    mem = rng.integers(E, 3 * E * L, size=N).astype(float)
    cnt, ok = PO.count_allocation(v, mem, 1.0, E)
    # step-1 value per server, written out again here from the printed formula
    first = np.array([[min(E, math.floor(mem[n] * v[n, l] / v[n].sum())) for l in range(L)]
                      for n in range(N)])
    assert np.array_equal(cnt.sum(axis=1), first.sum(axis=1))     # step 2 moves inside a server
    assert np.all(cnt >= 0) and np.all(cnt <= E)
    assert np.all(cnt.sum(axis=1) <= mem)                         # memory constraint of Sec. III-B
    if ok:
        assert np.all(cnt.sum(axis=0) >= E)                       # expert-coverage constraint
    if first.sum() >= E * L and N == 1:
        assert ok                                                 # one server with enough room always succeeds


# ---------------------------------------------------------------------------
# Alg. 2
# ---------------------------------------------------------------------------

def test_assignment_hand_worked_repair():
    # both servers prefer experts 0 and 1; 2 and 3 are uncovered.  Equal duplicate counts ->
    # server 0 first: it uses expert 2 more than 3 and gives up its less used duplicate 1;
    # then expert 1 is no longer a duplicate on server 1, which swaps 0 for the last one, 3.
    f = np.array([[[10, 8, 1, 0]], [[9, 7, 5, 2]]], np.int64)
    place, covered = PO.assignment(f, np.array([[2], [2]]))
    assert covered
    assert place[:, 0].tolist() == [[1, 0, 1, 0], [0, 1, 0, 1]]
    assert PO.proxy_cost(f, place) == (8 + 0) + (9 + 5)


def test_assignment_fewest_duplicates_first_and_ties():
    # server 0 holds {0,1,2}, server 1 holds {0}; expert 3 is uncovered.  Duplicates: server 0
    # has one (expert 0), server 1 has one (expert 0): tie -> server 0 goes first and swaps
    # expert 0 (its only duplicate) for 3 although 0 is its favourite.
    f = np.array([[[9, 5, 4, 1]], [[6, 1, 1, 1]]], np.int64)
    place, covered = PO.assignment(f, np.array([[3], [1]]))
    assert covered and place[:, 0].tolist() == [[0, 1, 1, 1], [1, 0, 0, 0]]
    # equal frequencies: preference by lower index; the replaced duplicate is the higher index
    f = np.zeros((2, 1, 4), np.int64)
    place, covered = PO.assignment(f, np.array([[2], [2]]))
    assert covered and place[:, 0].tolist() == [[1, 0, 1, 0], [0, 1, 0, 1]]


def test_assignment_top_n_ties_go_to_the_lower_index():
    place, _ = PO.assignment(np.array([[[5, 5, 1]]], np.int64), np.array([[1]]))
    assert place[0, 0].tolist() == [1, 0, 0]


def test_assignment_repair_starts_with_the_server_with_fewest_duplicates():
    # holdings {0,1}, {0,1,2}, {2}; expert 3 is uncovered.  Duplicates: 2, 3 and 1 -> server 2 goes
    # first and swaps its only expert, 2 (server 1 holds it too), for 3; nothing is left to repair.
    f = np.array([[[9, 8, 1, 0]], [[9, 8, 7, 1]], [[1, 2, 9, 3]]], np.int64)
    place, covered = PO.assignment(f, np.array([[2], [3], [1]]))
    assert covered and place[:, 0].tolist() == [[1, 1, 0, 0], [1, 1, 1, 0], [0, 0, 0, 1]]


def test_assignment_cannot_cover_without_room():
    f = np.array([[[5, 4, 3, 2, 1]]], np.int64)
    place, covered = PO.assignment(f, np.array([[3]]))
    assert not covered and place[0, 0].tolist() == [1, 1, 1, 0, 0]


@pytest.mark.parametrize("seed", range(8))
def test_assignment_invariants(seed):
    rng = np.random.default_rng(100 + seed)
    N, L, E = int(rng.integers(1, 5)), int(rng.integers(1, 4)), int(rng.integers(2, 14))
    f = rng.integers(0, 50, size=(N, L, E))
    cnt = rng.integers(0, E + 1, size=(N, L))
    place, covered = PO.assignment(f, cnt)
    assert np.array_equal(place.sum(axis=2), cnt)                 # set sizes never change
    if np.all(cnt.sum(axis=0) >= E):
        assert covered and np.all(place.sum(axis=0) >= 1)         # every expert somewhere
    if covered:
        assert np.all(place.sum(axis=0) >= 1)
    # before any repair the choice is the top-N: no held expert is less frequent than a
    # dropped one, on servers whose layer needed no repair (all its top-N still held)
    for n in range(N):
        for l in range(L):
            order = sorted(range(E), key=lambda e: (-int(f[n, l, e]), e))
            top = set(order[: cnt[n, l]])
            held = set(np.flatnonzero(place[n, l]))
            if held == top and 0 < cnt[n, l] < E:
                assert min(f[n, l, e] for e in held) >= max(f[n, l, e] for e in set(range(E)) - held)


def test_unrepaired_choice_minimises_eq2_by_brute_force():
    """One server: among all subsets of size N_{n,l} the top-N has the lowest proxy cost."""
    rng = np.random.default_rng(5)
    f = rng.integers(0, 30, size=(1, 1, 7))
    for size in range(8):
        place, _ = PO.assignment(f, np.array([[size]]))
        best = min(int(f[0, 0].sum()) - sum(int(f[0, 0, e]) for e in s)
                   for s in itertools.combinations(range(7), size))
        assert PO.proxy_cost(f, place) == best


# ---------------------------------------------------------------------------
# Eq. 2 - 4
# ---------------------------------------------------------------------------

def test_proxy_cost_is_the_layers_remote_count():
    """Eq. 2 for one server and one layer with raw counts = the remote assignments the layer's
    dispatch step lists (computed by the independent layer oracle)."""
    cfg = make_config("cfg4_finegrained", T=200, H=64, F=64)
    inp = make_inputs(cfg)
    r = O.route(inp.f32(inp.x), inp.f32(inp.w_router), inp.bias, cfg.k, cfg.bias_group_tokens)
    d = O.dispatch(r.topk_idx, inp.mask, cfg.H, cfg.es)
    assert PO.proxy_cost(r.counts.reshape(1, 1, -1), inp.mask.reshape(1, 1, -1)) == d.n_remote
    assert PO.proxy_cost(r.counts.reshape(1, 1, -1), np.ones((1, 1, cfg.E), np.uint8)) == 0
    assert PO.proxy_cost(r.counts.reshape(1, 1, -1), np.zeros((1, 1, cfg.E), np.uint8)) == cfg.A


def test_migration_cost_of_the_16_expert_swap():
    cfg = CONFIGS["cfg5_dsv2lite_migration"]
    m0 = make_inputs(cfg, phase=0).mask.reshape(1, 1, -1)
    m1 = make_inputs(cfg, phase=1).mask.reshape(1, 1, -1)
    m_e = 3 * cfg.H * cfg.F * 2                                   # bytes of one bf16 expert
    seconds, flips = PO.migration_cost(m0, m1, m_e, [25e9])
    assert flips == 32                                            # 16 evicted + 16 admitted
    assert seconds == pytest.approx(32 * m_e / 25e9)
    assert PO.migration_cost(m0, m0, m_e, [25e9]) == (0.0, 0)
    # per-server speeds weigh the flips of their own server
    old = np.zeros((2, 1, 3), np.uint8)
    new = np.array([[[1, 0, 0]], [[1, 1, 0]]], np.uint8)
    seconds, flips = PO.migration_cost(old, new, 6.0, [2.0, 3.0])
    assert flips == 3 and seconds == pytest.approx(1 * 3.0 + 2 * 2.0)


def test_migration_rule_on_both_sides_of_the_threshold():
    assert PO.should_migrate(100, 60, 3.9, 0.1)        # 6.0 + 3.9 < 10.0
    assert not PO.should_migrate(100, 60, 4.1, 0.1)    # 6.0 + 4.1 > 10.0
    assert not PO.should_migrate(100, 100, 0.0, 0.1)   # no gain, strict inequality
    assert not PO.should_migrate(60, 100, 0.0, 0.1)    # worse plan


def test_plan_lowers_eq2_against_random_placement_of_the_same_size():
    """Skewed, server-specific popularity: the plan covers every expert and its proxy cost is
    below that of a random placement with the same number of experts per server and layer
    (the paper's 'Redundance' baseline distributes experts at random up to capacity)."""
    rng = np.random.default_rng(11)
    N, L, E = 2, 3, 16
    f = np.zeros((N, L, E), np.int64)
    for n in range(N):
        for l in range(L):
            ranks = rng.permutation(E) + 1
            f[n, l] = (10000 / ranks ** 1.2).astype(np.int64)
    v, cnt, place, ok = PO.placement_plan(f, [0.75 * L * E, 0.75 * L * E], 1.0)
    assert ok and np.all(place.sum(axis=0) >= 1)
    assert np.all(cnt.sum(axis=1) <= 0.75 * L * E)
    for trial in range(5):
        rand = np.zeros_like(place)
        for n in range(N):
            for l in range(L):
                rand[n, l, rng.choice(E, size=cnt[n, l], replace=False)] = 1
        assert PO.proxy_cost(f, place) < PO.proxy_cost(f, rand)
