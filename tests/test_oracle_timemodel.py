"""Pins for the oracle's wall-clock model (Eq. (7) with the communication timestamps tau) and for bubble filling
(Sec. 3.4, Eq. (12)): hand-worked instances, the printed three-term form against the time-line form, limits."""
import itertools

import numpy as np
import pytest


def _all_cuts(L, H):
    for bars in itertools.combinations_with_replacement(range(L + 1), H - 1):
        edges = (0,) + bars + (L,)
        yield [edges[i + 1] - edges[i] for i in range(H)]


def test_eq7_hand_worked(oracle):
    # layers 0..3, bp = 2 each (sum 8), comm = 1,1,9,1.
    bp, comm = [2, 2, 2, 2], [1, 1, 9, 1]
    # set {2,1}: backward of 3 (2) + of 2 (2) -> tau(2) = 4 on the iteration's clock, comm of 2 ends at 13;
    # backward of 1 is done at 6 < 13, so tau(1) = 13, comm of 1 ends at 14; backward ends at 8 -> 14, 6 exposed.
    assert oracle.eq7_summand(bp, comm, 1, 2) == 14
    assert oracle.iteration_timeline(bp, comm, [2, 1]) == (14, 6)
    # set {3,0}: comm of 3 runs 2..3; layer 0's backward is done at 8, its comm runs 8..9 (waits for BP, not for comm)
    assert oracle.iteration_timeline(bp, comm, [3, 0]) == (9, 1)
    # the plain-sum model of Eq. (8) would say max(6, 1 + 1) -> nothing exposed: the tau recursion sees the wait
    # empty set: one backward pass
    assert oracle.eq7_summand(bp, comm, 2, 0) == 8 and oracle.iteration_timeline(bp, comm, []) == (8, 0)
    it, ex, period = oracle.time_model([1, 1, 1, 1], bp, comm, [[3], [2], [1, 0]])
    # {3}: comm 2..3 hidden -> 8;  {2}: comm 4..13 -> 13;  {1,0}: comm of 1 6..7, of 0 8..9 -> 9; forward 4 each
    assert (it, ex, period) == ([12, 17, 13], [0, 5, 1], 42)


def test_printed_form_equals_time_line_on_contiguous_sets(oracle):
    rng = np.random.default_rng(0)
    for _ in range(300):
        L, H = int(rng.integers(1, 9)), int(rng.integers(1, 5))
        bp = rng.integers(0, 20, L).tolist()
        comm = rng.integers(0, 40, L).tolist()
        for sizes in _all_cuts(L, H):
            pos = 0
            for s in sizes:
                layers = [L - 1 - j for j in range(pos, pos + s)]
                assert oracle.eq7_summand(bp, comm, pos, s) == oracle.iteration_timeline(bp, comm, layers)[0]
                pos += s


def test_eq7_never_below_eq8_and_equal_without_waiting(oracle):
    # the span from first start to last end is at least the plain sum of the set's communication times
    rng = np.random.default_rng(1)
    for _ in range(300):
        L, H = int(rng.integers(1, 9)), int(rng.integers(1, 5))
        bp = rng.integers(0, 20, L).tolist()
        comm = rng.integers(0, 40, L).tolist()
        for sizes in _all_cuts(L, H):
            sets = oracle.sets_from_sizes(L, sizes)
            eq7 = sum(oracle.iteration_timeline(bp, comm, S)[0] for S in sets)
            assert eq7 >= oracle.sched_cost(bp, comm, sizes)
    # each communication at least as long as the next layer's backward: no waiting, the two models agree
    bp, comm = [1, 2, 3, 4], [5, 4, 6, 9]
    for sizes in _all_cuts(4, 3):
        sets = oracle.sets_from_sizes(4, sizes)
        assert sum(oracle.iteration_timeline(bp, comm, S)[0] for S in sets) == oracle.sched_cost(bp, comm, sizes)


def test_time_model_limits(oracle):
    fp, bp = [1, 2, 3], [4, 5, 6]
    # no communication: H iterations of forward + backward (T_LSGD without its t_COMM term, Eq. (4))
    it, ex, period = oracle.time_model(fp, bp, [0, 0, 0], [[2], [1], [0]])
    assert period == 3 * (6 + 15) and ex == [0, 0, 0]
    # everything every iteration, communication far longer than backward: layer 2 starts after its own backward,
    # the rest follow back to back (wait-free backward propagation): 6 + 300
    it, ex, _ = oracle.time_model(fp, bp, [100, 100, 100], [[2, 1, 0]])
    assert it == [6 + 6 + 300] and ex == [6 + 300 - 15]


def test_fill_bubbles_hand_worked(oracle):
    bp, comm = [10, 10, 10, 10], [1, 1, 1, 1]
    # cut {3} | {2} | {1,0}.  Set 1 starts at the top: no disjoint prefix.  Set 2 = {2}: rem = 20, own 1 -> may take
    # layer 3 (prefix limit 1).  Set 3 = {1,0}: rem = 10, own 2 -> takes 3 and 2 (2 + 2 <= 10).
    extra, sets = oracle.fill_bubbles(bp, comm, [1, 1, 2])
    assert extra == [0, 1, 2] and sets == [[3], [3, 2], [3, 2, 1, 0]]
    # an overflowing set takes nothing; a hidden one takes only what still fits
    bp, comm = [2, 2, 2, 2], [1, 1, 9, 3]
    extra, sets = oracle.fill_bubbles(bp, comm, [1, 1, 2])
    # {2}: rem 4 < own 9 -> 0.  {1,0}: rem 2, own 2 -> budget 2, layer 3 (3) does not fit -> 0
    assert extra == [0, 0, 0]
    bp, comm = [5, 5, 5, 5], [1, 1, 1, 4]
    extra, sets = oracle.fill_bubbles(bp, comm, [2, 2])
    # {1,0}: rem 5, own 2: layer 3 (4) -> 6 > 5 no.  An empty set: rem after the top layer = 15: 4,1,1,1 all fit
    assert extra == [0, 0]
    extra, sets = oracle.fill_bubbles(bp, comm, [4, 0])
    assert extra == [0, 4] and sets[1] == [3, 2, 1, 0]


def test_fill_bubbles_properties(oracle):
    rng = np.random.default_rng(2)
    for _ in range(400):
        L, H = int(rng.integers(1, 9)), int(rng.integers(1, 5))
        bp = rng.integers(1, 30, L).tolist()
        comm = rng.integers(1, 30, L).tolist()
        for sizes in list(_all_cuts(L, H))[::3]:
            extra, sets = oracle.fill_bubbles(bp, comm, sizes)
            base = oracle.sets_from_sizes(L, sizes)
            pos = 0
            for h, (e, S, B0) in enumerate(zip(extra, sets, base)):
                assert S == [L - 1 - j for j in range(e)] + B0 and len(set(S)) == len(S)
                h0 = B0[0] if B0 else L - 1
                rem = sum(bp[:h0])
                own = sum(comm[l] for l in B0)
                tot = sum(comm[l] for l in S)
                assert max(rem, tot) == max(rem, own)                   # Eq. (12): the iteration got no longer
                limit = pos if B0 else L
                if e < limit:                                            # and the prefix is maximal
                    assert max(rem, tot + comm[L - 1 - e]) > max(rem, own)
                pos += sizes[h]
            assert sorted(set(l for S in sets for l in S)) == list(range(L))   # still everything at least once
