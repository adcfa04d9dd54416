"""The Ascending / Descending layer-level schedules (appendix "Implementation Details
of Baselines", layer-level baseline).

The oracle is pinned to things other than itself: examples worked by hand, the
properties the text states (exact budget, non-decreasing, steps of at most one,
bounds), closed forms at the ends of the feasible range, and brute force on small
inputs (where only one sequence with the stated properties and the oracle's K_min /
K_max exists, the oracle must return it).  Then the library's host routine is compared
with the oracle, integer for integer.  No GPU is involved.
"""
import itertools
import os

import pytest

from oracle import schedules
from paper_2604_08133_amd import binding as B

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "schedule_examples.txt")


def golden_cases():
    out = []
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        head, tail = line.split(":")
        _, L, K, budget = head.split()
        out.append((int(L), int(K), int(budget), [int(v) for v in tail.split()]))
    return out


def has_properties(K, K_orig, budget):
    return (sum(K) == budget and all(1 <= v <= K_orig for v in K)
            and all(0 <= b - a <= 1 for a, b in zip(K, K[1:])))


# ---------------------------------------------------------------- oracle pins

def test_oracle_hand_worked_examples():
    cases = golden_cases()
    assert len(cases) >= 10
    for L, K, budget, expect in cases:
        assert schedules.ascending(L, K, budget) == expect, (L, K, budget)
        assert schedules.descending(L, K, budget) == expect[::-1]


def test_oracle_properties_over_the_whole_range():
    for L in range(1, 28):
        for K in (1, 2, 3, 4, 6, 8):
            for budget in range(L, L * K + 1):
                asc = schedules.ascending(L, K, budget)
                assert len(asc) == L and has_properties(asc, K, budget), (L, K, budget, asc)
                assert schedules.descending(L, K, budget) == asc[::-1]


def test_oracle_closed_forms():
    for L, K in ((26, 6), (16, 8), (24, 4), (7, 7)):
        assert schedules.ascending(L, K, L) == [1] * L
        assert schedules.ascending(L, K, L * K) == [K] * L
        # the latest and the earliest ramp from 1 to K are the only sequences with their sums
        late = [1] * (L - K) + list(range(1, K + 1))
        early = list(range(1, K + 1)) + [K] * (L - K)
        assert schedules.ascending(L, K, sum(late)) == late
        assert schedules.ascending(L, K, sum(early)) == early
    # L == K_orig and the budget of the plain ramp: the interpolation itself
    assert schedules.ascending(6, 6, 21) == [1, 2, 3, 4, 5, 6]


def test_oracle_against_brute_force_on_small_inputs():
    # all non-decreasing, step <= 1 sequences from lo to hi (ends fixed: the text adjusts
    # only the layers between the first and the last) with the right sum; where exactly one exists for the
    # widest feasible (lo, hi) the oracle must return it, otherwise one of them
    for L in range(3, 8):
        for K in (2, 3, 4):
            for budget in range(L, L * K + 1):
                got = schedules.ascending(L, K, budget)
                lo, hi = got[0], got[-1]
                pool = [list(s) for s in itertools.product(range(lo, hi + 1), repeat=L)
                        if s[0] == lo and s[-1] == hi and has_properties(list(s), K, budget)]
                assert got in pool, (L, K, budget, got)
                if len(pool) == 1:
                    assert got == pool[0]
                # K_min is raised (K_max lowered) only when the budget does not fit
                if lo > 1:
                    assert not any(has_properties(list(s), K, budget)
                                   for s in itertools.product(range(lo - 1, K + 1), repeat=L)
                                   if s[0] == lo - 1 and s[-1] == K)
                if hi < K:
                    assert not any(has_properties(list(s), K, budget)
                                   for s in itertools.product(range(1, hi + 2), repeat=L)
                                   if s[0] == 1 and s[-1] == hi + 1)


def test_oracle_rejects_infeasible_budgets():
    for args in ((4, 3, 3), (4, 3, 13), (0, 3, 0), (4, 0, 4)):
        with pytest.raises(ValueError):
            schedules.ascending(*args)


# ---------------------------------------------------------- library vs oracle

def test_library_equals_oracle():
    for L in list(range(1, 14)) + [26, 27, 48]:
        for K in (1, 2, 3, 6, 8):
            for budget in range(L, L * K + 1):
                asc = schedules.ascending(L, K, budget)
                assert B.allocmoe_layer_schedule(B.SCHEDULE_ASCENDING, L, K, budget) == asc
                assert B.allocmoe_layer_schedule(B.SCHEDULE_DESCENDING, L, K, budget) == asc[::-1]


def test_library_paper_budgets():
    # DeepSeek-V2-Lite: 26 MoE layers, Top-6, the budget settings of the efficiency study
    for budget in (130, 104, 78, 52):
        asc = B.allocmoe_layer_schedule(B.SCHEDULE_ASCENDING, 26, 6, budget)
        assert has_properties(asc, 6, budget)
        assert asc == schedules.ascending(26, 6, budget)


def test_library_errors():
    with pytest.raises(B.AllocMoEError):
        B.allocmoe_layer_schedule(B.SCHEDULE_ASCENDING, 4, 3, 3)       # below one per layer
    with pytest.raises(B.AllocMoEError):
        B.allocmoe_layer_schedule(B.SCHEDULE_ASCENDING, 4, 3, 13)      # above L * K_orig
    with pytest.raises(B.AllocMoEError):
        B.allocmoe_layer_schedule(7, 4, 3, 8)                          # unknown kind
