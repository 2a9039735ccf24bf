"""Pins of the length-balancing oracle (paper section 3.1.1): hand-worked schedules, brute force on
tiny inputs, the list-scheduling bounds, and the degenerate cases."""
import itertools
import random

import pytest

from oracle.length_balance import balance_lengths, makespan


def _check_shape(lens, G, equal, out):
    group_of, order, bounds, totals = out
    n = len(lens)
    assert sorted(order) == list(range(n))
    assert bounds[0] == 0 and bounds[-1] == n and len(bounds) == G + 1
    assert all(bounds[g] <= bounds[g + 1] for g in range(G))
    for g in range(G):
        seg = order[bounds[g]:bounds[g + 1]]
        assert all(group_of[i] == g for i in seg)
        assert totals[g] == sum(lens[i] for i in seg)
        # inside a group: the order of assignment = decreasing length, then increasing index
        assert seg == sorted(seg, key=lambda i: (-lens[i], i))
        if equal:
            assert len(seg) == n // G + (1 if g < n % G else 0)
    assert sum(totals) == sum(lens)


def test_hand_worked_list_schedule():
    # the classic tight case of longest-first list scheduling on three machines: optimum 9, greedy 11
    lens = [5, 5, 4, 4, 3, 3, 3]
    group_of, order, bounds, totals = balance_lengths(lens, 3, equal_count=False)
    assert group_of == [0, 1, 2, 2, 0, 1, 0]
    assert totals == [11, 8, 8]
    assert order == [0, 4, 6, 1, 5, 2, 3] and bounds == [0, 3, 5, 7]
    # unsorted input, same multiset: the visit order comes from the lengths, not from the positions
    lens2 = [3, 4, 5, 3, 5, 3, 4]
    g2, _, _, t2 = balance_lengths(lens2, 3, equal_count=False)
    assert t2 == [11, 8, 8]
    assert g2 == [0, 2, 0, 1, 1, 0, 2]


def test_hand_worked_equal_count():
    lens = [10, 1, 1, 1, 1, 1]
    free = balance_lengths(lens, 2, equal_count=False)
    assert free[0] == [0, 1, 1, 1, 1, 1] and free[3] == [10, 5]
    capped = balance_lengths(lens, 2, equal_count=True)
    assert capped[0] == [0, 1, 1, 1, 0, 0] and capped[3] == [12, 3]
    _check_shape(lens, 2, True, capped)


def _brute_optimum(lens, G, equal):
    n = len(lens)
    best = None
    for assign in itertools.product(range(G), repeat=n):
        if equal:
            cnt = [assign.count(g) for g in range(G)]
            if sorted(cnt) != sorted(n // G + (1 if g < n % G else 0) for g in range(G)):
                continue
        m = makespan(lens, assign, G)
        best = m if best is None else min(best, m)
    return best


@pytest.mark.parametrize("G", [2, 3])
def test_against_brute_force(G):
    rng = random.Random(100 + G)
    for trial in range(60):
        n = rng.randint(1, 8)
        lens = [rng.choice([0, 1, 2, 3, 5, 8, 13, 40, 100]) + rng.randint(0, 3) for _ in range(n)]
        for equal in (False, True):
            out = balance_lengths(lens, G, equal)
            _check_shape(lens, G, equal, out)
            got = makespan(lens, out[0], G)
            assert got == max(out[3])
            opt = _brute_optimum(lens, G, equal)
            assert got >= opt
            if not equal:
                # Graham's bound for longest-first list scheduling
                assert 3 * G * got <= (4 * G - 1) * opt
            else:
                # no group ends more than one longest sample above the optimum
                assert got <= opt + max(lens)


def test_spread_bound_and_invariants_large():
    rng = random.Random(7)
    for G in (1, 4, 8, 13):
        lens = [int(min(32768, max(16, rng.lognormvariate(6.5, 1.0)))) for _ in range(1000)]
        out = balance_lengths(lens, G, False)
        _check_shape(lens, G, False, out)
        # the group that ends largest was the smallest when it got its last sample
        assert max(out[3]) - min(out[3]) <= max(lens)
        out = balance_lengths(lens, G, True)
        _check_shape(lens, G, True, out)
        # far better than dealing the samples out in input order
        naive = [0] * G
        for i, v in enumerate(lens):
            naive[i * G // len(lens)] += v
        assert max(out[3]) <= max(naive)


def test_degenerate_cases():
    assert balance_lengths([], 3, True) == ([], [], [0, 0, 0, 0], [0, 0, 0])
    # one group takes everything, longest first
    g, order, bounds, totals = balance_lengths([2, 9, 4], 1, True)
    assert g == [0, 0, 0] and order == [1, 2, 0] and bounds == [0, 3] and totals == [15]
    # equal lengths: dealt round-robin by sample index
    for equal in (False, True):
        g, _, _, totals = balance_lengths([6] * 10, 4, equal)
        assert g == [i % 4 for i in range(10)]
        assert totals == [18, 18, 12, 12]
    # fewer samples than groups: one each, the longest to group 0
    g, order, bounds, totals = balance_lengths([3, 8], 4, True)
    assert g == [1, 0] and totals == [8, 3, 0, 0] and bounds == [0, 1, 2, 2, 2]
    # all-zero lengths are legal; ties everywhere
    g, _, _, totals = balance_lengths([0, 0, 0], 2, False)
    assert g == [0, 0, 0] and totals == [0, 0]
    g, _, _, _ = balance_lengths([0, 0, 0], 2, True)
    assert g == [0, 0, 1]
    with pytest.raises(ValueError):
        balance_lengths([1, -1], 2, False)
    with pytest.raises(ValueError):
        balance_lengths([1], 0, False)
