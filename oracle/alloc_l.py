"""CPU oracle of Alloc-L's layer-wise allocation (Section 3.2, Eqs. (3)-(5)).

TEST INFRASTRUCTURE, NOT THE PRODUCT (see oracle/__init__.py).

Problem: a sensitivity matrix S[i][k-1] (layer i = 0..L-1, k = 1..K_orig experts
per token) and a global budget B; find K = [K_0..K_{L-1}], 1 <= K_i <= K_orig,
sum K_i <= B, minimising sum_i S[i][K_i].

Two routines, both in fp64 with the sum taken in layer order 0, 1, ..., L-1:
  * alloc_l_enumerate: the definition written out -- every allocation is tried
    (small L only);
  * alloc_l_dp: the paper's dynamic programme, DP[i][b] = min_k DP[i-1][b-k] +
    S[i][k] with DP[-1][0] = 0, DP[-1][b>0] = +inf, the answer at the best b <= B,
    recovered by backtracking.

Reading of the paper where it is silent: among allocations of equal total
sensitivity the one that spends less budget wins, then the one with the smaller
K at the deepest layer, then at the layer before it, and so on.
"""
from __future__ import annotations

import itertools
import math
from typing import List, Sequence, Tuple


def _cost(S: Sequence[Sequence[float]], K: Sequence[int]) -> float:
    total = 0.0
    for i, k in enumerate(K):
        total = total + float(S[i][k - 1])
    return total


def _tie_key(K: Sequence[int]):
    return (sum(K),) + tuple(reversed(K))


def alloc_l_enumerate(S: Sequence[Sequence[float]], B: int) -> Tuple[List[int], float]:
    L, K_orig = len(S), len(S[0])
    if B < L:
        raise ValueError("budget below one expert per layer")
    best, best_cost = None, math.inf
    for K in itertools.product(range(1, K_orig + 1), repeat=L):
        if sum(K) > B:
            continue
        c = _cost(S, K)
        if c < best_cost or (c == best_cost and _tie_key(K) < _tie_key(best)):
            best, best_cost = K, c
    return list(best), best_cost


def alloc_l_dp(S: Sequence[Sequence[float]], B: int) -> Tuple[List[int], float]:
    L, K_orig = len(S), len(S[0])
    if B < L:
        raise ValueError("budget below one expert per layer")
    top = min(B, L * K_orig)
    prev = [math.inf] * (top + 1)     # DP[-1][b]
    prev[0] = 0.0
    table = []
    for i in range(L):
        cur = [math.inf] * (top + 1)
        for b in range(top + 1):
            for k in range(1, min(K_orig, b) + 1):
                c = prev[b - k] + float(S[i][k - 1])
                if c < cur[b]:
                    cur[b] = c
        table.append(cur)
        prev = cur
    last = table[L - 1]
    best_b = min(range(top + 1), key=lambda b: (last[b], b))
    K = [0] * L
    b = best_b
    for i in range(L - 1, -1, -1):
        below = table[i - 1] if i > 0 else [0.0] + [math.inf] * top
        for k in range(1, min(K_orig, b) + 1):
            if below[b - k] + float(S[i][k - 1]) == table[i][b]:
                K[i] = k
                break
        b -= K[i]
    return K, last[best_b]
