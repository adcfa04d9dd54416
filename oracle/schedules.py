"""CPU oracle of the heuristic layer-level budget schedules (appendix "Implementation
Details of Baselines", layer-level baseline): Ascending and Descending.

TEST INFRASTRUCTURE, NOT THE PRODUCT (see oracle/__init__.py).

The paper describes the Ascending schedule in words, in four steps, taken here in its
order:
  1. an integer vector by rounded linear interpolation between K_min (first layer) and
     K_max (last layer);
  2. a forward and a backward pass that make it non-decreasing with steps of at most one;
  3. greedy adjustments of the internal layers (not the first, not the last), one unit
     at a time and only where the vector stays non-decreasing, within [K_min, K_max] and
     with steps of at most one, until the allocations sum to the budget B exactly;
  4. K_min = 1 and K_max = K_orig unless B does not fit: then K_min is raised until it
     does.
Descending is the same vector in reverse layer order.

Readings where the text leaves a choice (each also listed in the design notes):
  * "rounded": halves round up, floor(x + 1/2);
  * the greedy adjustment sweeps the internal layers from the shallowest to the deepest,
    changing each layer that may change by one unit, and repeats until the sum is B;
  * a budget BELOW what K_min = 1 can reach (the text only covers the opposite case) is
    met by lowering K_max, symmetrically;
  * a single layer gets K = B.
"""
from __future__ import annotations

import math
from typing import List


def _initial_profile(L: int, lo: int, hi: int) -> List[int]:
    if L == 1:
        return [lo]
    K = [int(math.floor(lo + (hi - lo) * i / (L - 1) + 0.5)) for i in range(L)]
    for i in range(1, L):                       # forward: never below, at most one above
        K[i] = min(max(K[i], K[i - 1]), K[i - 1] + 1)
    for i in range(L - 2, -1, -1):              # backward: never above, at most one below
        K[i] = max(min(K[i], K[i + 1]), K[i + 1] - 1)
    return K


def _may_raise(K: List[int], i: int, hi: int) -> bool:
    v = K[i] + 1
    return v <= hi and v <= K[i + 1] and v - K[i - 1] <= 1


def _may_lower(K: List[int], i: int, lo: int) -> bool:
    v = K[i] - 1
    return v >= lo and v >= K[i - 1] and K[i + 1] - v <= 1


def ascending(L: int, K_orig: int, B: int) -> List[int]:
    if L < 1 or K_orig < 1 or B < L or B > L * K_orig:
        raise ValueError("need L >= 1, K_orig >= 1, L <= B <= L * K_orig")
    if L == 1:
        return [B]
    lo, hi = 1, K_orig
    while lo <= hi:
        K = _initial_profile(L, lo, hi)
        total = sum(K)
        while total != B:
            changed = False
            for i in range(1, L - 1):
                if total < B and _may_raise(K, i, hi):
                    K[i] += 1
                    total += 1
                    changed = True
                elif total > B and _may_lower(K, i, lo):
                    K[i] -= 1
                    total -= 1
                    changed = True
                if total == B:
                    break
            if not changed:
                break
        if total == B:
            return K
        if total < B:
            lo += 1
        else:
            hi -= 1
    raise ValueError("no schedule found")   # not reached for L <= B <= L * K_orig


def descending(L: int, K_orig: int, B: int) -> List[int]:
    return list(reversed(ascending(L, K_orig, B)))
