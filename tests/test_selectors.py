"""Calibrated baseline selectors (Top-P and relative-threshold skipping, Appendix A.1),
spending exactly the layer budget.

CPU part pins the oracle (oracle/selectors.py) against an independent statement of the
same rules: find the threshold by sweeping, apply the per-token rule literally.  GPU
part: keep counts and dispatch bit-exact against the oracle, whole layer within
tolerance."""
import numpy as np
import pytest
import torch

import oracle
from oracle import selectors as sel
from paper_2604_08133_amd import synth


def literal_top_p(s, K_base, budget):
    """Per-token rule applied literally: candidate j is kept iff j < K_base or the score
    mass before it (fp32, in order) is below p; p = the smallest threshold that keeps at
    least `budget` pairs; pairs exactly at the boundary are dropped from the end of the
    (token, rank) order until the budget is met."""
    s = np.asarray(s, dtype=np.float32)
    T, K = s.shape
    mass = np.zeros((T, K), dtype=np.float32)
    for j in range(1, K):
        mass[:, j] = (mass[:, j - 1] + s[:, j - 1]).astype(np.float32)
    pool = [(float(mass[t, j]), t, j) for t in range(T) for j in range(K_base, K)]
    want = budget - T * K_base
    kept = np.zeros((T, K), dtype=bool)
    kept[:, :K_base] = True
    if want > 0:
        vals = sorted(v for v, _, _ in pool)
        p_last = vals[want - 1]                       # mass of the last pair kept
        inside = [(t, j) for v, t, j in pool if v < p_last]
        border = sorted((t, j) for v, t, j in pool if v == p_last)
        for t, j in inside + border[:want - len(inside)]:
            kept[t, j] = True
    return kept


def literal_relative(s, K_base, budget):
    s = np.asarray(s, dtype=np.float32)
    T, K = s.shape
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(s[:, :1] > 0, (s / s[:, :1]).astype(np.float32), np.float32(0))
    pool = [(float(ratio[t, j]), t, j) for t in range(T) for j in range(K_base, K)]
    want = budget - T * K_base
    kept = np.zeros((T, K), dtype=bool)
    kept[:, :K_base] = True
    if want > 0:
        vals = sorted((v for v, _, _ in pool), reverse=True)
        beta = vals[want - 1]
        inside = [(t, j) for v, t, j in pool if v > beta]
        border = sorted((t, j) for v, t, j in pool if v == beta)
        for t, j in inside + border[:want - len(inside)]:
            kept[t, j] = True
    return kept


@pytest.mark.parametrize("levels", [None, 16])
@pytest.mark.parametrize("T,E,K,Kb", [(40, 16, 4, 1), (64, 8, 2, 1), (100, 64, 6, 2), (33, 12, 5, 0)])
def test_oracle_selectors_equal_literal_rules(T, E, K, Kb, levels):
    scores = synth.make_scores(T, E, seed=3 * T + K, quantize_levels=levels)
    _, s = oracle.topk(scores, K)
    for budget in sorted({T * Kb, T * Kb + 1, (T * Kb + T * K) // 2, T * K - 1, T * K}):
        for mode, literal in ((sel.TOP_P, literal_top_p), (sel.RELATIVE, literal_relative)):
            kept, cnt = sel.select(s, mode, Kb, budget)
            assert int(cnt.sum()) == budget
            want = literal(s.numpy(), Kb, budget)
            assert np.array_equal(kept.numpy().astype(bool), want), (mode, budget)
            # kept candidates of a token are a prefix of its sorted row
            assert all(kept[t, :int(cnt[t])].all() and not kept[t, int(cnt[t]):].any() for t in range(T))


def test_oracle_selector_special_cases():
    # identical tokens: every pool key ties across tokens, spares go to the lower tokens
    row = torch.tensor([0.4, 0.3, 0.2, 0.1])
    s = row.repeat(6, 1)
    for mode in (sel.TOP_P, sel.RELATIVE):
        _, cnt = sel.select(s, mode, 1, 6 + 4)
        assert cnt.tolist() == [2, 2, 2, 2, 1, 1]
    # relative: a token whose candidates are all equal keeps everything first
    s = torch.tensor([[0.5, 0.5, 0.5], [0.9, 0.3, 0.1]])
    _, cnt = sel.select(s, sel.RELATIVE, 1, 2 + 2)
    assert cnt.tolist() == [3, 1]
    # top-p: the token with the least mass in front keeps more
    _, cnt = sel.select(s, sel.TOP_P, 1, 2 + 1)
    assert cnt.tolist() == [2, 1]
    # keys of the score selector are the scores: same result as Alloc-T
    scores = synth.make_scores(50, 16, seed=9)
    _, s = oracle.topk(scores, 4)
    a = sel.select(s, sel.SCORE, 1, 120)
    b = oracle.alloc_t(s, 1, 120)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


# --------------------------------------------------------------- GPU parity

@pytest.mark.gpu
@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("T,E,K,Kb,levels", [(64, 8, 2, 1, None), (32, 64, 6, 1, None), (333, 60, 4, 1, 16),
                                             (3000, 64, 6, 1, None), (3000, 64, 6, 2, 64),
                                             (9000, 64, 6, 1, None)])
def test_gpu_selectors_bit_exact(mode, T, E, K, Kb, levels):
    from paper_2604_08133_amd import binding as B
    scores = synth.make_scores(T, E, seed=mode + T, quantize_levels=levels)
    dev = torch.device("cuda:0")
    sc = scores.to(dev)
    for budget in sorted({T * Kb, (T * Kb + T * K) // 2, T * Kb + T // 3, T * K}):
        print(f"selector {mode} T={T} E={E} K={K} Kb={Kb} B={budget}", flush=True)
        desc = B.make_desc(T, 128, E, 128, K, Kb, budget, "f32", selector=mode)
        ids = torch.empty((T, K), dtype=torch.int32, device=dev)
        s = torch.empty((T, K), dtype=torch.float32, device=dev)
        cnt = torch.empty((T,), dtype=torch.int32, device=dev)
        ws = torch.empty(B.allocmoe_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        B.allocmoe_route_from_scores(desc, sc, ids, s, cnt, ws)
        torch.cuda.synchronize()
        ref_ids, ref_s = oracle.topk(scores, K)
        assert torch.equal(ids.cpu(), ref_ids) and torch.equal(s.cpu(), ref_s)
        _, ref_cnt = sel.select(ref_s, mode, Kb, budget)
        assert torch.equal(cnt.cpu(), ref_cnt), (mode, budget)


@pytest.mark.gpu
@pytest.mark.parametrize("mode", [1, 2])
def test_gpu_layer_with_selector(mode):
    from paper_2604_08133_amd import binding as B
    from paper_2604_08133_amd.layer import DeviceLayer
    for w, tol in ((synth.tiny(budget=96, K_base=1), 1e-4),
                   (synth.Workload("sel_bf16", T=200, d=256, E=16, I=128, K=4, K_base=1, budget=500,
                                   dtype="bf16", I_shared=128, I_shared_each=128, bias_kind="normal"), 2e-2)):
        layer = synth.make_layer(w)
        dev = DeviceLayer(w, layer)
        desc = B.make_desc(w.T, w.d, w.E, w.I, w.K, w.K_base, w.budget, w.dtype, w.I_shared,
                           w.shared_gate, selector=mode)
        ws = torch.empty(B.allocmoe_workspace_bytes(desc), dtype=torch.uint8, device="cuda:0")
        Y = torch.empty((w.T, w.d), dtype=dev.dtype, device="cuda:0")
        print(f"layer {w.name} selector {mode}", flush=True)
        B.allocmoe_moe_forward(desc, dev.X, dev.weights, Y, ws)
        torch.cuda.synchronize()
        L = B.allocmoe_workspace_layout(desc)
        scores = B.ws_view(ws, L.scores, (w.T, w.E), torch.float32).cpu()
        cnt = B.ws_view(ws, L.keep_count, (w.T,), torch.int32).cpu()
        inv = B.ws_view(ws, L.inv_row, (w.T, w.K), torch.int32).cpu()
        ref = oracle.forward(layer, w.K, w.K_base, w.budget, scores=scores, selector=mode)
        assert torch.equal(cnt, ref["keep_count"]) and torch.equal(inv, ref["inv_row"])
        err = float((Y.cpu().double() - ref["Y"]).abs().max() / ref["Y"].abs().max())
        print(f"  scaled max err {err:.3e}", flush=True)
        assert err <= tol
