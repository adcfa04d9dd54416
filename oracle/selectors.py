"""CPU oracle of the alternative token-level selectors (the token-level baselines of
Section 4 / Appendix A.1: Top-P routing as in Dynamic-MoE, and skipping experts whose
score falls below a fraction beta of the token's Top-1 score as in NAEE extended to
Top-K), each *calibrated on the batch to spend exactly the layer budget*, so that they
can be compared with Alloc-T at equal cost.

TEST INFRASTRUCTURE, NOT THE PRODUCT (see oracle/__init__.py).

A selector turns a token's sorted candidate scores s[t,0] >= s[t,1] >= ... into keys
that do not increase along the row; the kept pairs are then, as in Alloc-T (Section
3.3), every token's first K_base candidates plus the B - T*K_base pool entries with
the largest keys (ties: lower token, then lower rank):
  score (Alloc-T)   key = s[t,j]
  top-p             key = -(s[t,0] + ... + s[t,j-1])     kept iff the mass before j is < p
  relative          key = s[t,j] / s[t,0] (0 if s[t,0] <= 0)   kept iff >= beta
The threshold (p or beta) is implied by the budget: it is the key of the last pair kept.
Keys are formed in fp32 (sequential adds, IEEE division), the precision in which the
GPU takes the same decisions.
"""
from __future__ import annotations

import numpy as np
import torch

SCORE, TOP_P, RELATIVE = 0, 1, 2


def selector_keys(topk_s, selector: int) -> np.ndarray:
    s = np.ascontiguousarray(np.asarray(topk_s, dtype=np.float32))
    T, K = s.shape
    if selector == SCORE:
        return s.copy()
    keys = np.empty((T, K), dtype=np.float32)
    if selector == TOP_P:
        mass = np.zeros(T, dtype=np.float32)
        for j in range(K):
            keys[:, j] = -mass
            mass = (mass + s[:, j]).astype(np.float32)
        return keys
    if selector == RELATIVE:
        top = s[:, 0]
        ok = top > 0
        for j in range(K):
            with np.errstate(divide="ignore", invalid="ignore"):
                r = (s[:, j] / top).astype(np.float32)
            keys[:, j] = np.where(ok, r, np.float32(0))
        return keys
    raise ValueError(selector)


def select(topk_s, selector: int, K_base: int, budget: int):
    """(kept [T,K] uint8, keep_count [T] int32) of the calibrated selector."""
    import oracle
    keys = torch.from_numpy(selector_keys(topk_s, selector))
    return oracle.alloc_t(keys, K_base, budget)
