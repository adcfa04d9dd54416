"""Pins for the oracle's integer path (candidates, Alloc-T selection, dispatch).

The oracle is checked against things other than itself: a brute-force
enumeration of the selection problem of Section 3.3, Eqs. (7)-(9); the
reduction to plain Top-K named after Eq. (9); budget conservation; a
hand-worked example (tests/golden); and library routines (torch.topk/sort).
"""
import itertools
import os

import pytest
import torch

import oracle
from paper_2604_08133_amd import synth


# ----------------------------------------------------------------- brute force

def brute_force_optima(s, Kb, B):
    """All optimal solutions of Eqs. (7)-(9) with the budget used in full:
    subsets of the T*K candidates of size B with at least Kb per token that
    maximise the summed score.  Returns (best value, list of index tuples)."""
    T, K = s.shape
    flat = [float(v) for v in s.reshape(-1)]
    best, sets = None, []
    for comb in itertools.combinations(range(T * K), B):
        per_tok = [0] * T
        for i in comb:
            per_tok[i // K] += 1
        if min(per_tok) < Kb:
            continue
        val = sum(flat[i] for i in comb)
        if best is None or val > best + 1e-12:
            best, sets = val, [comb]
        elif abs(val - best) <= 1e-12:
            sets.append(comb)
    return best, sets


def sorted_rows(T, K, seed, levels=None):
    g = torch.Generator().manual_seed(seed)
    if levels is None:
        s = torch.rand((T, K), generator=g, dtype=torch.float32)
    else:  # exact dyadic values with many ties
        s = torch.randint(0, levels, (T, K), generator=g).to(torch.float32) / 8.0
    return torch.sort(s, dim=1, descending=True).values.contiguous()


@pytest.mark.parametrize("T,K", [(2, 3), (3, 3), (3, 4), (4, 3)])
def test_alloc_t_equals_brute_force_distinct(T, K):
    for seed in range(3):
        s = sorted_rows(T, K, 100 * T + 10 * K + seed)
        assert s.reshape(-1).unique().numel() == T * K
        for Kb in range(0, K + 1):
            for B in range(T * Kb, T * K + 1):
                kept, cnt = oracle.alloc_t(s, Kb, B)
                best, sets = brute_force_optima(s, Kb, B)
                assert len(sets) == 1          # distinct scores: unique optimum
                got = tuple(int(i) for i in torch.nonzero(kept.reshape(-1)).reshape(-1))
                assert got == sets[0], (T, K, Kb, B)
                assert int(cnt.sum()) == B


@pytest.mark.parametrize("T,K", [(2, 3), (3, 3), (3, 4)])
def test_alloc_t_ties_optimal_and_lowest_index(T, K):
    for seed in range(4):
        s = sorted_rows(T, K, 7 * T + K + seed, levels=4)
        for Kb in range(0, K + 1):
            for B in range(T * Kb, T * K + 1):
                kept, cnt = oracle.alloc_t(s, Kb, B)
                got = tuple(int(i) for i in torch.nonzero(kept.reshape(-1)).reshape(-1))
                best, sets = brute_force_optima(s, Kb, B)
                val = sum(float(s.reshape(-1)[i]) for i in got)
                assert abs(val - best) <= 1e-12           # an optimum of the ILP
                assert got in sets                          # and feasible
                assert got == min(sets), (s, Kb, B)        # lowest indices among optima


def test_infeasible_budgets_rejected():
    s = sorted_rows(4, 3, 1)
    with pytest.raises(ValueError):
        oracle.alloc_t(s, 2, 7)      # below T*Kb: Eq. (9) cannot hold
    with pytest.raises(ValueError):
        oracle.alloc_t(s, 1, 13)     # above the candidate set T*K
    with pytest.raises(ValueError):
        oracle.alloc_t(s, 4, 12)     # Kb > K


# ------------------------------------------------------ hand-worked golden file

def load_golden(path):
    scores, ids, cases, disp = [], [], [], {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, rest = line.split(None, 1)
            if key == "scores":
                scores.append([float(x) for x in rest.split()])
            elif key == "ids":
                ids.append([int(x) for x in rest.split()])
            elif key == "case":
                lhs, rhs = rest.split(":")
                kb, b = (int(x) for x in lhs.split())
                cases.append((kb, b, [int(x) for x in rhs.split()]))
            elif key == "dispatch_case":
                disp["case"] = tuple(int(x) for x in rest.split())
            else:
                disp.setdefault(key, []).append([int(x) for x in rest.split()])
    return (torch.tensor(scores, dtype=torch.float32), torch.tensor(ids, dtype=torch.int32),
            cases, disp)


def test_hand_worked_example(golden_dir):
    s, ids, cases, disp = load_golden(os.path.join(golden_dir, "alloc_t_worked_example.txt"))
    assert len(cases) >= 15
    for kb, b, expect in cases:
        kept, cnt = oracle.alloc_t(s, kb, b)
        assert cnt.tolist() == expect, (kb, b)
        for t in range(s.shape[0]):   # kept ranks are a prefix of the sorted row
            assert kept[t].tolist() == [1] * expect[t] + [0] * (s.shape[1] - expect[t])
    kb, b = disp["case"]
    kept, _ = oracle.alloc_t(s, kb, b)
    offs, row_token, row_rank, inv_row = oracle.dispatch(ids, kept, 5)
    assert offs.tolist() == disp["expert_offsets"][0]
    assert row_token.tolist() == disp["row_token"][0]
    assert row_rank.tolist() == disp["row_rank"][0]
    assert inv_row.tolist() == disp["inv_row"]


# ------------------------------------------------------- candidates (Eq. (6))

def test_topk_matches_library_on_distinct_scores():
    s = synth.make_scores(257, 64, seed=3)
    ids, vals = oracle.topk(s, 6)
    tv, ti = torch.topk(s, 6, dim=1, largest=True, sorted=True)
    assert torch.equal(vals, tv)
    assert torch.equal(ids.long(), ti)


def test_topk_tie_rule_lower_expert_first():
    s = torch.tensor([[0.25, 0.5, 0.25, 0.5, 0.0, 0.25]], dtype=torch.float32)
    ids, vals = oracle.topk(s, 5)
    assert ids.tolist() == [[1, 3, 0, 2, 5]]
    assert vals.tolist() == [[0.5, 0.5, 0.25, 0.25, 0.25]]


# ------------------------------------ reduction to Top-K, conservation, ranges

@pytest.mark.parametrize("T,E,K", [(64, 8, 2), (200, 64, 6), (333, 60, 4)])
def test_reduces_to_plain_topk(T, E, K):
    s = synth.make_scores(T, E, seed=11)
    ids, vals = oracle.topk(s, K)
    # full budget: every candidate kept == independent per-token Top-K
    kept, cnt = oracle.alloc_t(vals, 1, T * K)
    assert bool(kept.all()) and cnt.tolist() == [K] * T
    # K_base = K_l, B = T*K_l: plain per-token Top-K_l
    for Kl in range(0, K + 1):
        kept, cnt = oracle.alloc_t(vals, Kl, T * Kl)
        expect = torch.zeros((T, K), dtype=torch.uint8)
        expect[:, :Kl] = 1
        assert torch.equal(kept, expect)
        # the kept experts are torch.topk's
        if Kl:
            ti = torch.topk(s, Kl, dim=1).indices
            assert torch.equal(ids[:, :Kl].long(), ti)


@pytest.mark.parametrize("levels", [None, 16])
def test_conservation_ranges_threshold_prefix_nested(levels):
    T, E, K = 150, 16, 5
    s = synth.make_scores(T, E, seed=5, quantize_levels=levels)
    ids, vals = oracle.topk(s, K)
    for Kb in (0, 1, 2):
        prev = None
        for B in range(T * Kb, T * K + 1, 37):
            kept, cnt = oracle.alloc_t(vals, Kb, B)
            assert int(cnt.sum()) == B and int(kept.sum()) == B        # conservation
            assert int(cnt.min()) >= Kb and int(cnt.max()) <= K        # Eq. (9), |C_l|
            # prefix: kept ranks of a token are 0..k_t-1
            ranks = torch.arange(K).expand(T, K)
            assert torch.equal(kept.bool(), ranks < cnt[:, None])
            # threshold: every kept non-base score >= every dropped score
            nb = kept.bool().clone()
            nb[:, :Kb] = False
            dropped = ~kept.bool()
            if nb.any() and dropped.any():
                assert float(vals[nb].min()) >= float(vals[dropped].max())
            # nested in the budget
            if prev is not None:
                assert bool((kept >= prev).all())
            prev = kept
            offs, row_token, row_rank, inv_row = oracle.dispatch(ids, kept, E)
            assert int(offs[-1]) == B


def test_token_permutation_equivariance():
    T, E, K = 97, 32, 4
    s = synth.make_scores(T, E, seed=9)
    _, vals = oracle.topk(s, K)
    assert vals.reshape(-1).unique().numel() == T * K
    g = torch.Generator().manual_seed(4)
    perm = torch.randperm(T, generator=g)
    for B in (T, 2 * T + 13, 3 * T):
        _, cnt = oracle.alloc_t(vals, 1, B)
        _, cnt_p = oracle.alloc_t(vals[perm].contiguous(), 1, B)
        assert torch.equal(cnt[perm], cnt_p)


def test_more_experts_go_to_flatter_tokens():
    """Section 5 (analysis): tokens with less concentrated routing receive more
    activations.  Checked as a positive rank correlation between routing
    entropy and k_t on synthetic scores whose concentration ranges from one
    dominant expert to a handful of comparable ones (a qualitative pin, not
    the paper's value; for near-uniform rows over all N experts every
    candidate is small and the relation reverses)."""
    T, E, K = 2048, 64, 6
    g = torch.Generator().manual_seed(8)
    logits = torch.randn((T, E), generator=g, dtype=torch.float64)
    logits *= torch.rand((T, 1), generator=g, dtype=torch.float64) * 7 + 1.0
    s = oracle.softmax(logits)
    _, vals = oracle.topk(s, K)
    _, cnt = oracle.alloc_t(vals, 1, 3 * T)
    p = s.double()
    ent = -(p * torch.log(p.clamp_min(1e-300))).sum(dim=1)
    ra = torch.argsort(torch.argsort(ent)).double()
    rb = torch.argsort(torch.argsort(cnt.double() + 1e-9 * ra)).double()
    rho = torch.corrcoef(torch.stack([ra, rb]))[0, 1]
    assert float(rho) > 0.3


# ------------------------------------------------------------------- dispatch

def test_dispatch_is_a_sorted_permutation():
    T, E, K = 301, 60, 4
    s = synth.make_scores(T, E, seed=2)
    ids, vals = oracle.topk(s, K)
    kept, cnt = oracle.alloc_t(vals, 1, 2 * T + 55)
    offs, row_token, row_rank, inv_row = oracle.dispatch(ids, kept, E)
    B = int(cnt.sum())
    # library re-derivation: stable sort of the kept pairs by (expert, token)
    tt, jj = torch.nonzero(kept, as_tuple=True)
    ee = ids[tt, jj].long()
    order = torch.argsort(ee * T + tt, stable=True)
    assert torch.equal(row_token.long(), tt[order])
    assert torch.equal(row_rank.long(), jj[order])
    assert torch.equal(offs.long(), torch.cat([torch.zeros(1, dtype=torch.long),
                                               torch.bincount(ee, minlength=E).cumsum(0)]))
    # round trip
    rows = inv_row[row_token.long(), row_rank.long()]
    assert torch.equal(rows.long(), torch.arange(B))
    assert int((inv_row >= 0).sum()) == B
    assert torch.equal(inv_row >= 0, kept.bool())
