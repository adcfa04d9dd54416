"""Alloc-L's layer-wise allocation (Section 3.2, Eqs. (3)-(5)).

First the oracle is pinned to things other than itself: the enumeration of every
allocation (the definition), closed forms, and an independently written greedy
for rows with diminishing returns (where marginal-gain greedy is the textbook
optimum).  Then the library's host routine is compared with the oracle, integer
for integer.  No GPU is involved: the paper runs this step offline on the host.
"""
import itertools
import math
import random

import pytest

from oracle.alloc_l import alloc_l_dp, alloc_l_enumerate
from paper_2604_08133_amd import binding as B


def random_matrix(rng, L, K, kind):
    if kind == "free":          # any values, with repeats so that ties occur
        return [[rng.choice([0.25, 0.5, 1.0, 1.5, rng.random()]) for _ in range(K)] for _ in range(L)]
    if kind == "monotone":      # more experts never hurt (what perplexity profiles look like)
        rows = []
        for _ in range(L):
            steps = sorted((rng.random() for _ in range(K)), reverse=True)
            base = rng.random()
            rows.append([base + s for s in steps])
        return rows
    if kind == "convex":        # decreasing with diminishing returns
        rows = []
        for _ in range(L):
            gains = sorted((rng.random() for _ in range(K - 1)), reverse=True)
            row = [5.0 + rng.random()]
            for g in gains:
                row.append(row[-1] - g)
            rows.append(row)
        return rows
    raise ValueError(kind)


# ---------------------------------------------------------------- oracle pins

@pytest.mark.parametrize("kind", ["free", "monotone", "convex"])
def test_oracle_dp_equals_enumeration(kind):
    rng = random.Random(7)
    for _ in range(150):
        L, K = rng.randint(1, 5), rng.randint(1, 4)
        S = random_matrix(rng, L, K, kind)
        budget = rng.randint(L, L * K + 2)
        assert alloc_l_dp(S, budget) == alloc_l_enumerate(S, budget), (S, budget)


def test_oracle_hand_worked_example():
    # tests/golden/alloc_l_example.txt: 3 layers, K_orig = 3, worked by hand
    rows, cases = [], []
    for line in open(__file__.rsplit("/", 1)[0] + "/golden/alloc_l_example.txt"):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tag, *vals = line.split()
        if tag == "S":
            rows.append([float(v) for v in vals])
        elif tag == "B":
            cases.append((int(vals[0]), [int(v) for v in vals[1:4]], float(vals[4])))
    assert len(rows) == 3 and len(cases) >= 4
    for budget, want_K, want_cost in cases:
        K, cost = alloc_l_dp(rows, budget)
        assert K == want_K and cost == pytest.approx(want_cost, abs=1e-12), (budget, K, cost)
        assert alloc_l_enumerate(rows, budget)[0] == want_K


def test_oracle_closed_forms():
    L, K = 6, 4
    decreasing = [[10.0 - k - 0.1 * i for k in range(K)] for i in range(L)]
    # budget for everything: every layer takes K_orig
    assert alloc_l_dp(decreasing, L * K)[0] == [K] * L
    assert alloc_l_dp(decreasing, L * K + 50)[0] == [K] * L
    # minimum budget: one expert everywhere
    assert alloc_l_dp(decreasing, L)[0] == [1] * L
    # constant rows: nothing to gain, the cheapest allocation (least spend) wins
    assert alloc_l_dp([[3.0] * K for _ in range(L)], 3 * L)[0] == [1] * L
    # identical strictly convex rows, budget a multiple of L: the uniform allocation
    # (the paper's budgets 130/104/78/52 over 26 layers are averages 5/4/3/2)
    row = [20.0, 12.0, 7.0, 4.0, 2.5, 2.0]
    for avg in (5, 4, 3, 2):
        assert alloc_l_dp([row] * 26, 26 * avg)[0] == [avg] * 26
    with pytest.raises(ValueError):
        alloc_l_dp(decreasing, L - 1)


def greedy_convex(S, budget):
    """Textbook optimum for decreasing rows with diminishing returns: start at one
    expert everywhere, repeatedly buy the largest remaining marginal decrease."""
    L, K = len(S), len(S[0])
    alloc = [1] * L
    for _ in range(budget - L):
        gains = [(S[i][alloc[i] - 1] - S[i][alloc[i]], i) for i in range(L) if alloc[i] < K]
        if not gains:
            break
        g, i = max(gains)
        if g <= 0:
            break
        alloc[i] += 1
    return alloc


def test_oracle_matches_marginal_gain_greedy_on_convex_rows():
    rng = random.Random(11)
    for _ in range(100):
        L, K = rng.randint(2, 12), rng.randint(2, 8)
        S = random_matrix(rng, L, K, "convex")
        budget = rng.randint(L, L * K)
        K_dp, cost = alloc_l_dp(S, budget)
        K_gr = greedy_convex(S, budget)
        total = lambda a: sum(S[i][a[i] - 1] for i in range(L))
        assert total(K_dp) == pytest.approx(total(K_gr), rel=1e-12)
        assert sum(K_dp) <= budget


def test_oracle_invariants():
    rng = random.Random(3)
    for _ in range(50):
        L, K = rng.randint(2, 10), rng.randint(2, 6)
        S = random_matrix(rng, L, K, "monotone")
        costs = [alloc_l_dp(S, b)[1] for b in range(L, L * K + 1)]
        assert all(a >= b for a, b in zip(costs, costs[1:]))      # more budget never costs more
        for b in (L, (L * K + L) // 2, L * K):
            alloc, cost = alloc_l_dp(S, b)
            assert all(1 <= k <= K for k in alloc) and sum(alloc) <= b
            assert cost == pytest.approx(sum(S[i][alloc[i] - 1] for i in range(L)))


# ------------------------------------------------ the library against the oracle

@pytest.mark.parametrize("kind", ["free", "monotone", "convex"])
def test_library_equals_oracle(kind):
    rng = random.Random(23)
    for _ in range(120):
        L, K = rng.randint(1, 30), rng.randint(1, 8)
        S = random_matrix(rng, L, K, kind)
        budget = rng.randint(L, L * K + 3)
        want_K, want_cost = alloc_l_dp(S, budget)
        got_K, got_cost = B.allocmoe_alloc_l(S, budget)
        assert got_K == want_K and got_cost == want_cost, (L, K, budget)


def test_library_model_shapes():
    # the paper's three models: (layers, K_orig, budgets) of Section 4.1
    rng = random.Random(5)
    for L, K, budgets in [(26, 6, (130, 104, 78, 52)), (24, 4, (84, 72, 60, 48)),
                          (16, 8, (112, 96, 80, 64))]:
        S = random_matrix(rng, L, K, "monotone")
        for budget in budgets:
            got_K, got_cost = B.allocmoe_alloc_l(S, budget)
            assert (got_K, got_cost) == alloc_l_dp(S, budget)
            assert sum(got_K) <= budget


def test_library_errors():
    S = [[1.0, 0.5], [1.0, 0.5], [1.0, 0.5]]
    with pytest.raises(RuntimeError):
        B.allocmoe_alloc_l(S, 2)                      # below one expert per layer
    with pytest.raises(RuntimeError):
        B.allocmoe_alloc_l([[1.0, math.nan]], 2)
