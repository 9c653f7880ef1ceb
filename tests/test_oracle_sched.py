"""Pins for the oracle's scheduler: Eq. (8) against hand-worked values and an independent algebraic form,
exhaustive search against its defining properties, Algorithm 2 against Properties 1-3 and the size bound of
its solution set."""
import itertools
import math
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sched_cases.txt")


def _cases():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, bp, comm, sizes, cost = [x.strip() for x in line.split(";")]
        out.append((name, [int(v) for v in bp.split(",")], [int(v) for v in comm.split(",")],
                    [int(v) for v in sizes.split(",")], int(cost)))
    return out


def _cost_excess_form(bp, comm, sizes):
    """H * sum(bp) + sum over non-empty sets of max(0, comm(set) - backward work left after the set's first
    layer): the same objective after cancelling the terms of Eq. (8) that do not depend on the cut."""
    L, H = len(bp), len(sizes)
    total, pos = H * sum(bp), 0
    for s in sizes:
        if s:
            layers = [L - 1 - j for j in range(pos, pos + s)]
            rem = sum(bp[: layers[0]])
            total += max(0, sum(comm[l] for l in layers) - rem)
        pos += s
    return total


def _all_cuts(L, H):
    for bars in itertools.combinations_with_replacement(range(L + 1), H - 1):
        edges = (0,) + bars + (L,)
        yield [edges[i + 1] - edges[i] for i in range(H)]


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c[0])
def test_cost_matches_hand_worked_values(oracle, case):
    _, bp, comm, sizes, cost = case
    assert oracle.sched_cost(bp, comm, sizes) == cost
    assert _cost_excess_form(bp, comm, sizes) == cost


def test_cost_equals_excess_form_on_random_instances(oracle):
    rng = np.random.default_rng(0)
    for _ in range(300):
        L, H = int(rng.integers(1, 9)), int(rng.integers(1, 5))
        bp = rng.integers(0, 20, L).tolist()
        comm = rng.integers(0, 40, L).tolist()
        for sizes in _all_cuts(L, H):
            assert oracle.sched_cost(bp, comm, sizes) == _cost_excess_form(bp, comm, sizes)


def test_brute_force_enumerates_every_cut_and_takes_the_minimum(oracle):
    rng = np.random.default_rng(1)
    for _ in range(200):
        L, H = int(rng.integers(1, 7)), int(rng.integers(1, 4))
        bp = rng.integers(1, 12, L).tolist()
        comm = rng.integers(1, 25, L).tolist()
        sizes, cost, n = oracle.sched_brute(bp, comm, H)
        assert n == math.comb(L + H - 1, H - 1)
        costs = {tuple(c): _cost_excess_form(bp, comm, c) for c in _all_cuts(L, H)}
        assert cost == min(costs.values())
        # tie-break: lexicographically largest size vector among the minimisers
        assert tuple(sizes) == max(c for c, v in costs.items() if v == cost)


def test_hand_worked_optima(oracle):
    assert oracle.sched_brute([3, 5], [4, 2], 2)[:2] == ([2, 0], 19)
    assert oracle.sched_brute([1, 1, 8, 1, 2], [2, 5, 2, 1, 9], 2)[:2] == ([1, 4], 26)


def test_everything_hidden_goes_to_the_first_set(oracle):
    # if the whole model's communication fits under the backward work left after the top layer, set 1 takes all
    bp, comm = [10, 10, 10, 10, 1], [1, 2, 3, 4, 5]
    for H in (1, 2, 3, 5):
        for res in (oracle.sched_brute(bp, comm, H)[:2], oracle.sched_alg2(bp, comm, H)[:2]):
            assert res == ([5] + [0] * (H - 1), H * sum(bp))


def test_hopeless_communication_gives_one_layer_per_set_in_alg2(oracle):
    # every single layer overflows: Property 3 places one layer, Property 2 then pushes the next to a new set
    bp, comm = [1, 2, 3, 4], [100, 100, 100, 100]
    sizes, cost, omega = oracle.sched_alg2(bp, comm, 4)
    assert sizes == [1, 1, 1, 1] and omega == [[1, 1, 1, 1]]
    # excess = comm_l - (backward work below l): 100-6, 100-3, 100-1, 100-0; the optimum cannot do better,
    # because every cut pays sum(comm) minus at most one `rem` per non-empty set, and these are the largest rems
    assert cost == 4 * 10 + (94 + 97 + 99 + 100)
    assert oracle.sched_brute(bp, comm, 4)[1] == cost


def test_alg2_counter_example_and_bounds(oracle):
    sizes, cost, omega = oracle.sched_alg2([1, 1, 8, 1, 2], [2, 5, 2, 1, 9], 2)
    assert (sizes, cost) == ([3, 2], 33) and omega == [[3, 2], [2, 3]]
    rng = np.random.default_rng(2)
    worse = total = 0
    for _ in range(2000):
        L, H = int(rng.integers(1, 7)), int(rng.integers(1, 4))
        bp = rng.integers(1, 12, L).tolist()
        comm = rng.integers(1, 25, L).tolist()
        sizes, cost, omega = oracle.sched_alg2(bp, comm, H)
        opt = oracle.sched_brute(bp, comm, H)[1]
        assert sum(sizes) == L and all(sum(o) == L for o in omega)
        assert cost == min(_cost_excess_form(bp, comm, o) for o in omega) >= opt
        # Sec. 3.3, complexity analysis: a branch needs a non-empty set that is not the last one, and the layer
        # after the assign-branch is always delayed, so there is at most one branch per set and per layer.
        # (The printed O(2^min(L-H, H)) is asymptotic: L = H = 2 already yields two solutions.)
        assert len(omega) <= 2 ** min(L - 1, H - 1)
        total += 1
        worse += cost > opt
    assert worse / total < 0.08                               # "equivalent to brute force in most cases"


def test_alg2_rules_hold_on_every_recorded_solution(oracle):
    # replay each solution: a set is only closed while non-empty (Property 3) and never after a layer that
    # would still have been hidden (Property 1); a set that already overflows takes no further layer (Property 2)
    rng = np.random.default_rng(3)
    for _ in range(500):
        L, H = int(rng.integers(2, 9)), int(rng.integers(2, 5))
        bp = rng.integers(1, 12, L).tolist()
        comm = rng.integers(1, 25, L).tolist()
        for sizes in oracle.sched_alg2(bp, comm, H)[2]:
            pos = 0
            for h, s in enumerate(sizes):
                last = h == H - 1
                if pos < L and not last:
                    assert s >= 1
                if s and not last:
                    h0 = L - 1 - pos
                    rem = sum(bp[:h0])
                    members = [L - 1 - j for j in range(pos, pos + s)]
                    for j in range(1, s):                      # when member j was added the set did not overflow yet
                        assert sum(comm[l] for l in members[:j]) <= rem
                    nxt = L - 1 - (pos + s)
                    if nxt >= 0:                               # the next layer was not hideable here
                        assert sum(comm[l] for l in members) + comm[nxt] > rem
                pos += s


def test_enp_sizes(oracle):
    assert oracle.sched_enp(8, 4) == [2, 2, 2, 2]
    assert oracle.sched_enp(34, 8) == [5, 5, 4, 4, 4, 4, 4, 4]
    assert oracle.sched_enp(3, 5) == [1, 1, 1, 0, 0]
    assert oracle.sets_from_sizes(5, [2, 0, 3]) == [[4, 3], [], [2, 1, 0]]
