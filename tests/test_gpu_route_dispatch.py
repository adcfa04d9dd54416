"""GPU parity of the integer path through the C ABI: candidates, Alloc-T keep
counts and the expert-sorted dispatch must be bit-exact functions of the score
input (compared with the CPU oracle on identical scores)."""
import pytest
import torch

import oracle
from paper_2604_08133_amd import binding as B
from paper_2604_08133_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def gpu_route_dispatch(scores_cpu, K, Kb, budget, select_ws=True):
    """select_ws: hand the selection a workspace, with which it runs on many workgroups
    from 2048 tokens on; without, one workgroup selects whatever the size."""
    T, E = scores_cpu.shape
    desc = B.make_desc(T, 64, E, 64, K, Kb, budget, "f32")
    s = scores_cpu.to(DEV)
    ids = torch.empty((T, K), dtype=torch.int32, device=DEV)
    vals = torch.empty((T, K), dtype=torch.float32, device=DEV)
    cnt = torch.empty((T,), dtype=torch.int32, device=DEV)
    sel_ws = None
    if select_ws:
        sel_ws = torch.empty(B.allocmoe_workspace_layout(desc).scores, dtype=torch.uint8, device=DEV)
    B.allocmoe_route_from_scores(desc, s, ids, vals, cnt, sel_ws)
    offs = torch.empty((E + 1,), dtype=torch.int32, device=DEV)
    row_token = torch.full((max(budget, 1),), -7, dtype=torch.int32, device=DEV)
    row_rank = torch.full((max(budget, 1),), -7, dtype=torch.int32, device=DEV)
    inv_row = torch.empty((T, K), dtype=torch.int32, device=DEV)
    ws = torch.empty(B.allocmoe_workspace_layout(desc).scores, dtype=torch.uint8, device=DEV)
    B.allocmoe_dispatch(desc, ids, cnt, offs, row_token, row_rank, inv_row, ws)
    torch.cuda.synchronize()
    return dict(topk_ids=ids.cpu(), topk_s=vals.cpu(), keep_count=cnt.cpu(),
                expert_offsets=offs.cpu(), row_token=row_token.cpu()[:budget],
                row_rank=row_rank.cpu()[:budget], inv_row=inv_row.cpu())


def oracle_route_dispatch(scores_cpu, K, Kb, budget):
    ids, vals = oracle.topk(scores_cpu, K)
    kept, cnt = oracle.alloc_t(vals, Kb, budget)
    offs, row_token, row_rank, inv_row = oracle.dispatch(ids, kept, scores_cpu.shape[1])
    return dict(topk_ids=ids, topk_s=vals, keep_count=cnt, expert_offsets=offs,
                row_token=row_token, row_rank=row_rank, inv_row=inv_row)


def assert_same(got, want, tag):
    for k in want:
        assert torch.equal(got[k], want[k]), (tag, k)


def budgets_for(T, K, Kb):
    lo, hi = T * Kb, T * K
    mid = (lo + hi) // 2
    return sorted({lo, min(hi, lo + 1), mid, min(hi, mid + 7), max(lo, hi - 1), hi})


@pytest.mark.parametrize("T,E,K", [(64, 8, 2), (32, 64, 6), (1, 64, 6), (63, 17, 5), (333, 60, 4),
                                   (1000, 64, 6), (1025, 64, 8), (4096, 64, 6), (8192, 64, 6),
                                   (8192, 64, 8), (9000, 64, 6),    # these two: the large-size code path
                                   (50, 64, 16), (2100, 64, 16),    # the widest candidate rows allowed
                                   (7, 1, 1), (100, 2, 2), (300, 3, 1)])   # degenerate expert counts
@pytest.mark.parametrize("Kb", [0, 1, 2])
def test_bit_exact_distinct_scores(T, E, K, Kb):
    if Kb > K:
        pytest.skip("K_base > K")
    scores = synth.make_scores(T, E, seed=T + E)
    for budget in budgets_for(T, K, Kb):
        print(f"case T={T} E={E} K={K} Kb={Kb} B={budget}", flush=True)
        assert_same(gpu_route_dispatch(scores, K, Kb, budget),
                    oracle_route_dispatch(scores, K, Kb, budget), (T, E, K, Kb, budget))


@pytest.mark.parametrize("T,E,K,Kb", [(4096, 64, 6, 1), (9000, 64, 6, 0)])
def test_bit_exact_selection_without_workspace(T, E, K, Kb):
    # the single-workgroup selection at sizes where a workspace would spread it
    for levels in (None, 64):
        scores = synth.make_scores(T, E, seed=3 + T, quantize_levels=levels)
        for budget in budgets_for(T, K, Kb):
            assert_same(gpu_route_dispatch(scores, K, Kb, budget, select_ws=False),
                        oracle_route_dispatch(scores, K, Kb, budget), (T, budget, levels))


@pytest.mark.parametrize("levels", [4, 64, 1024])
@pytest.mark.parametrize("T,E,K,Kb", [(200, 16, 4, 1), (3000, 64, 6, 1), (3000, 64, 6, 0),
                                      (2049, 60, 4, 2), (8192, 64, 6, 1), (9500, 64, 6, 1),
                                      # pools small enough for the direct-ranking selection
                                      (40, 16, 4, 1), (32, 64, 6, 1), (64, 8, 2, 0), (60, 16, 4, 0)])
def test_bit_exact_with_ties(levels, T, E, K, Kb):
    scores = synth.make_scores(T, E, seed=levels + T, quantize_levels=levels)
    for budget in budgets_for(T, K, Kb) + [T * Kb + T // 3]:
        print(f"ties T={T} E={E} K={K} Kb={Kb} B={budget} levels={levels}", flush=True)
        assert_same(gpu_route_dispatch(scores, K, Kb, budget),
                    oracle_route_dispatch(scores, K, Kb, budget), (levels, T, budget))


@pytest.mark.parametrize("T", [5000, 2500, 48])   # many workgroups, one workgroup, direct ranking
def test_all_scores_equal(T):
    E, K = 64, 6
    scores = torch.full((T, E), 1.0 / E, dtype=torch.float32)
    for Kb, budget in [(1, T + 1), (1, 3 * T + 11), (0, 17), (2, 5 * T), (1, 6 * T - 1)]:
        print(f"equal T={T} Kb={Kb} B={budget}", flush=True)
        assert_same(gpu_route_dispatch(scores, K, Kb, budget),
                    oracle_route_dispatch(scores, K, Kb, budget), (Kb, budget))


def test_signed_and_zero_scores():
    # route_from_scores orders any finite fp32: negatives, -0.0 == +0.0, tiny values
    g = torch.Generator().manual_seed(12)
    T, E, K = 500, 32, 5
    scores = torch.randn((T, E), generator=g)
    scores[::7, ::3] = 0.0
    scores[::5, 1::4] = -0.0
    scores[3::11] = 1e-41          # subnormals
    for Kb, budget in [(1, 2 * T), (0, T + 3), (2, 4 * T - 5)]:
        got = gpu_route_dispatch(scores, K, Kb, budget)
        want = oracle_route_dispatch(scores, K, Kb, budget)
        assert_same(got, want, (Kb, budget))


def test_conservation_on_device():
    T, E, K = 4096, 64, 6
    scores = synth.make_scores(T, E, seed=77)
    for budget in (T, 12288, 20000, T * K):
        got = gpu_route_dispatch(scores, K, 1, budget)
        assert int(got["keep_count"].sum()) == budget
        assert int(got["expert_offsets"][-1]) == budget
        assert int(got["keep_count"].min()) >= 1 and int(got["keep_count"].max()) <= K


def test_budget_errors_reported_by_status():
    desc = B.make_desc(8, 64, 8, 64, 2, 1, 7, "f32")
    with pytest.raises(B.AllocMoEError) as e:
        t = torch.zeros((8, 8), device=DEV)
        B.allocmoe_route_from_scores(desc, t, t, t, t)
    assert e.value.status == B.EBUDGET


def test_seeded_random_cases():
    # 400 seeded draws of (T, E, K, K_base, budget) and of the kind of score matrix:
    # signed, few distinct levels (many ties), softmax-like, half zeros of both signs, all
    # equal; mostly pools small enough for the direct ranking, one in five large
    import random
    rng = random.Random(5)
    for n in range(400):
        big = rng.random() < 0.2
        T = rng.choice([100, 257, 700, 1500, 4096, 8192, 8200]) if big else rng.randint(1, 80)
        E = rng.choice([1, 2, 3, 7, 16, 33, 64])
        K = rng.randint(1, min(E, 16))
        Kb = rng.randint(0, K)
        budget = rng.randint(T * Kb, T * K)
        kind = rng.choice(["signed", "levels", "softmax", "zeros", "equal"])
        g = torch.Generator().manual_seed(rng.randint(1, 10**6))
        if kind == "signed":
            s = torch.randn((T, E), generator=g)
        elif kind == "levels":
            s = torch.randint(-3, 4, (T, E), generator=g).float() * 0.25
        elif kind == "softmax":
            s = torch.softmax(torch.randn((T, E), generator=g) * 2, dim=1)
        elif kind == "zeros":
            s = torch.randn((T, E), generator=g)
            s[torch.rand((T, E), generator=g) < 0.5] = 0.0
            s[torch.rand((T, E), generator=g) < 0.2] = -0.0
        else:
            s = torch.full((T, E), 0.125)
        print(f"random case {n}: T={T} E={E} K={K} Kb={Kb} B={budget} {kind}", flush=True)
        assert_same(gpu_route_dispatch(s, K, Kb, budget), oracle_route_dispatch(s, K, Kb, budget), n)


@pytest.mark.parametrize("T", [500, 9000])   # the single-workgroup kernel, the large-size kernels
def test_dispatch_with_keep_counts_above_the_budget_stays_inside_it(T):
    # the caller's keep counts sum to more than desc->budget (a contract violation the host
    # cannot see): nothing may leave the kernel that points past the budget's rows
    E, K = 16, 4
    scores = synth.make_scores(T, E, seed=77)
    ids, _ = oracle.topk(scores, K)
    budget = T * 2
    desc = B.make_desc(T, 64, E, 64, K, 1, budget, "f32")
    cnt = torch.full((T,), 3, dtype=torch.int32, device=DEV)          # sums to 3T > 2T
    offs = torch.empty((E + 1,), dtype=torch.int32, device=DEV)
    guard = 64
    row_token = torch.full((budget + guard,), -7, dtype=torch.int32, device=DEV)
    row_rank = torch.full((budget + guard,), -7, dtype=torch.int32, device=DEV)
    inv_row = torch.empty((T, K), dtype=torch.int32, device=DEV)
    ws = torch.empty(B.allocmoe_workspace_layout(desc).scores, dtype=torch.uint8, device=DEV)
    B.allocmoe_dispatch(desc, ids.to(DEV), cnt, offs, row_token, row_rank, inv_row, ws)
    torch.cuda.synchronize()
    assert int(inv_row.max()) < budget and int(inv_row.min()) >= -1
    assert int(offs.max()) <= budget and int(offs[0]) == 0
    assert bool((offs[1:] >= offs[:-1]).all())
    assert bool((row_token[budget:] == -7).all()) and bool((row_rank[budget:] == -7).all())
    placed = inv_row[inv_row >= 0]
    assert placed.numel() == budget and placed.unique().numel() == budget   # every row used once
    # rows that exist are consistent with the pair behind them
    r = inv_row.cpu()
    tt, jj = torch.nonzero(r >= 0, as_tuple=True)
    assert torch.equal(row_token.cpu()[r[tt, jj].long()], tt.int())
    assert torch.equal(row_rank.cpu()[r[tt, jj].long()], jj.int())
