"""Pins for the oracle's floating-point path (gate, softmax, experts, Eq. (2)).

Checked against closed forms, special cases that reduce to a textbook MLP, the
dense definition of Eq. (2), and an independent fp64 re-computation with
library routines (torch matmul / softmax / topk) in the plain Top-K case.
"""
import math

import pytest
import torch

import oracle
from paper_2604_08133_amd import synth


def silu(a):
    return a / (1.0 + math.exp(-a))


# -------------------------------------------------------------- Eq. (1) pins

def test_softmax_closed_form_and_invariants():
    logits = torch.tensor([[0.0, math.log(2.0), math.log(5.0)],
                           [math.log(3.0) + 50.0, 50.0, 50.0]], dtype=torch.float64)
    s = oracle.softmax(logits)
    assert torch.allclose(s, torch.tensor([[0.125, 0.25, 0.625], [0.6, 0.2, 0.2]]), atol=1e-7)
    g = torch.Generator().manual_seed(0)
    l = torch.randn((50, 64), generator=g, dtype=torch.float64) * 4
    s = oracle.softmax(l)
    assert torch.allclose(s.double().sum(dim=1), torch.ones(50, dtype=torch.float64), atol=1e-6)
    assert torch.equal(s, oracle.softmax(l + 123.0))          # shift invariance
    assert torch.allclose(s.double(), torch.softmax(l, dim=1), atol=1e-7)
    # huge logits must not overflow (max-subtracted)
    s = oracle.softmax(torch.tensor([[1000.0, 999.0]], dtype=torch.float64))
    assert torch.isfinite(s).all() and abs(float(s[0, 0]) - 1 / (1 + math.exp(-1))) < 1e-7


def test_gate_logits_orientation_and_bias():
    # X [T,d] times Wg [d,E]: one-hot rows pick rows of Wg
    Wg = torch.arange(12, dtype=torch.float32).reshape(3, 4)
    X = torch.eye(3, dtype=torch.float32)
    assert torch.equal(oracle.gate_logits(X, Wg), Wg.double())
    bias = torch.tensor([1.0, -2.0, 0.5, 0.0])
    assert torch.equal(oracle.gate_logits(X, Wg, bias), Wg.double() + bias.double())
    g = torch.Generator().manual_seed(1)
    X = torch.randn((9, 33), generator=g)
    Wg = torch.randn((33, 7), generator=g)
    assert torch.allclose(oracle.gate_logits(X, Wg), X.double() @ Wg.double(), atol=1e-12)


def test_bf16_inputs_are_widened_exactly():
    g = torch.Generator().manual_seed(2)
    X = torch.randn((5, 16), generator=g).to(torch.bfloat16)
    Wg = torch.randn((16, 4), generator=g).to(torch.bfloat16)
    a = oracle.gate_logits(X, Wg)
    b = oracle.gate_logits(X.float(), Wg.float())
    assert torch.equal(a, b)


def test_shared_gate_closed_form():
    X = torch.tensor([[math.log(3.0), 0.0], [0.0, 0.0], [1.0, -1.0]], dtype=torch.float32)
    w = torch.tensor([1.0, 1.0], dtype=torch.float32)
    g = oracle.shared_gate(X, w)
    assert torch.allclose(g, torch.tensor([0.75, 0.5, 0.5], dtype=torch.float64), atol=1e-7)


# ------------------------------------------------------------ expert network

def test_expert_ffn_diagonal_closed_form():
    # W1 = a*I, W3 = b*I, W2 = c*I  =>  E(x)_h = silu(a x_h) * (b x_h) * c
    d = 6
    a, b, c = 1.5, -0.5, 2.0
    x = torch.tensor([0.0, 1.0, -1.0, 2.0, -3.0, 0.25], dtype=torch.float32)
    eye = torch.eye(d, dtype=torch.float32)
    out = oracle.expert_ffn(x, a * eye, b * eye, c * eye)
    expect = [silu(a * float(v)) * (b * float(v)) * c for v in x]
    assert torch.allclose(out, torch.tensor(expect, dtype=torch.float64), atol=1e-12)


def test_expert_ffn_which_branch_is_gated_and_orientation():
    # d = 2, I = 3, non-square: only W1's branch passes through silu, and the
    # matrices multiply on the right of the row vector x.
    x = torch.tensor([1.0, 2.0])
    W1 = torch.tensor([[1.0, 0.0, -1.0], [0.0, 1.0, 0.5]])     # x W1 = [1, 2, 0]
    W3 = torch.tensor([[2.0, 1.0, 0.0], [0.0, 1.0, 1.0]])      # x W3 = [2, 3, 2]
    W2 = torch.tensor([[1.0, 0.0], [0.0, 1.0], [5.0, 5.0]])
    out = oracle.expert_ffn(x, W1, W3, W2)
    h = [silu(1.0) * 2.0, silu(2.0) * 3.0, silu(0.0) * 2.0]
    expect = [h[0] + 5 * h[2], h[1] + 5 * h[2]]
    assert torch.allclose(out, torch.tensor(expect, dtype=torch.float64), atol=1e-12)
    swapped = oracle.expert_ffn(x, W3, W1, W2)
    assert not torch.allclose(out, swapped)


def test_single_expert_layer_is_a_plain_mlp():
    # N = 1, K = 1, B = T: the only score is 1, so y = SwiGLU-MLP(x)
    w = synth.Workload("one", T=7, d=24, E=1, I=40, K=1, K_base=1, budget=7, dtype="f32")
    layer = synth.make_layer(w, seed=3)
    res = oracle.forward(layer, 1, 1, 7)
    assert torch.equal(res["scores"], torch.ones((7, 1)))
    X, W1, W3, W2 = (layer[k].double() for k in ("X", "W1", "W3", "W2"))
    mlp = (torch.nn.functional.silu(X @ W1[0]) * (X @ W3[0])) @ W2[0]
    assert torch.allclose(res["Y"], mlp, atol=1e-12, rtol=1e-12)


# --------------------------------------------------------------- Eq. (2) pins

def lib_topk_moe(layer, K):
    """Independent fp64 computation of the plain Top-K layer with library ops."""
    X = layer["X"].double()
    logits = X @ layer["Wg"].double()
    if layer.get("bias") is not None:
        logits = logits + layer["bias"].double()
    scores = torch.softmax(logits, dim=1).float()       # scores are fp32 by contract
    tv, ti = torch.topk(scores, K, dim=1)
    Y = torch.zeros_like(X)
    W1, W3, W2 = layer["W1"].double(), layer["W3"].double(), layer["W2"].double()
    for e in range(W1.shape[0]):
        out_e = (torch.nn.functional.silu(X @ W1[e]) * (X @ W3[e])) @ W2[e]
        wt = (tv.double() * (ti == e)).sum(dim=1, keepdim=True)
        Y += wt * out_e
    if layer.get("Ws1") is not None:
        sh = (torch.nn.functional.silu(X @ layer["Ws1"].double()) *
              (X @ layer["Ws3"].double())) @ layer["Ws2"].double()
        if layer.get("w_sg") is not None:
            sh = torch.sigmoid(X @ layer["w_sg"].double())[:, None] * sh
        Y += sh
    return scores, Y


@pytest.mark.parametrize("dtype,shared,gate,bias", [("f32", 0, False, "none"),
                                                    ("bf16", 48, False, "normal"),
                                                    ("bf16", 32, True, "zipf")])
def test_full_budget_layer_matches_library_topk_moe(dtype, shared, gate, bias):
    w = synth.Workload("lib", T=23, d=40, E=6, I=24, K=3, K_base=1, budget=69, dtype=dtype,
                       I_shared=shared, I_shared_each=shared, shared_gate=gate,
                       bias_kind=bias)
    layer = synth.make_layer(w, seed=5)
    res = oracle.forward(layer, w.K, w.K_base, w.T * w.K)
    scores, Y = lib_topk_moe(layer, w.K)
    assert torch.allclose(res["scores"], scores, atol=2e-7)
    assert torch.allclose(res["Y"], Y, atol=1e-9, rtol=1e-9)


@pytest.mark.parametrize("Kb,B", [(1, 64), (0, 64), (1, 96), (0, 10), (2, 128), (1, 101)])
def test_dense_eq2_equals_dispatched_path(Kb, B):
    w = synth.tiny(budget=B, K_base=Kb).with_(I=32, d=24, I_shared=16, I_shared_each=16)
    layer = synth.make_layer(w, seed=6)
    res = oracle.forward(layer, w.K, Kb, B)
    dense = oracle.moe_eq2(layer, res["topk_ids"], res["topk_s"], res["kept"], None, dense=True)
    disp = oracle.moe_dispatched(layer, res["topk_s"], res["expert_offsets"],
                                 res["row_token"], res["inv_row"], None)
    assert torch.allclose(dense, res["Y"], atol=1e-12, rtol=1e-12)
    assert torch.allclose(dense, disp, atol=1e-12, rtol=1e-12)


def test_dropped_token_gets_only_the_shared_part():
    # K_base = 0 and a tiny budget: most tokens keep nothing (Section 3.3 allows
    # token dropping when K_base = 0); their output is the shared expert alone.
    w = synth.tiny(budget=3, K_base=0).with_(I=16, d=16, I_shared=8, I_shared_each=8)
    layer = synth.make_layer(w, seed=7)
    res = oracle.forward(layer, w.K, 0, 3)
    dropped = torch.nonzero(res["keep_count"] == 0).reshape(-1)
    assert dropped.numel() >= w.T - 3
    X = layer["X"].double()
    sh = (torch.nn.functional.silu(X @ layer["Ws1"].double()) *
          (X @ layer["Ws3"].double())) @ layer["Ws2"].double()
    assert torch.allclose(res["Y"][dropped], sh[dropped], atol=1e-12)


def test_weights_are_raw_scores_without_renormalisation():
    # One token, two identical experts E(x) = v: y = (sum of kept scores) * v,
    # which is < v unless everything is kept (Eq. (2): retained scores as is).
    d, I, E = 4, 4, 3
    eye = torch.eye(d)
    layer = dict(X=torch.tensor([[1.0, 2.0, -1.0, 0.5]]),
                 Wg=torch.zeros((d, E)),                     # uniform scores 1/3
                 W1=eye.repeat(E, 1, 1).contiguous(), W3=eye.repeat(E, 1, 1).contiguous(),
                 W2=eye.repeat(E, 1, 1).contiguous())
    v = torch.tensor([silu(float(a)) * float(a) for a in layer["X"][0]], dtype=torch.float64)
    for B in (1, 2, 3):
        res = oracle.forward(layer, 3, 0, B)
        assert torch.allclose(res["Y"][0], (B / 3.0) * v, atol=1e-7)


def test_token_subset_matches_full():
    w = synth.tiny(budget=80).with_(I=32, d=32)
    layer = synth.make_layer(w, seed=8)
    full = oracle.forward(layer, w.K, 1, 80)
    sub = oracle.forward(layer, w.K, 1, 80, tokens=[5, 0, 63])
    assert torch.equal(sub["Y"], full["Y"][[5, 0, 63]])
