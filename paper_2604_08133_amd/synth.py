"""Seeded synthetic inputs for the budgeted MoE layer.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests/benchmark.  It draws random tensors and names workload shapes; it
contains none of the method's arithmetic (no gate, softmax, selection, FFN).

The workloads stand in for the paper's evaluated models (Section 4.1, Table 1:
DeepSeek-V2-Lite with 64 routed experts / Top-6, Qwen1.5-MoE-A2.7B with 60
routed experts / Top-4), whose checkpoints and prompts are not available: the
shapes are theirs, the values are Gaussian with variance 1/fan_in.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import torch

BASE_SEED = 20260408

# tensor ids used to derive per-tensor seeds
_TENSOR_IDS = {"X": 0, "Wg": 1, "bias": 2, "W1": 3, "W3": 4, "W2": 5,
               "Ws1": 6, "Ws3": 7, "Ws2": 8, "w_sg": 9, "perm": 10, "budget": 11}


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape of one MoE layer call.  Names follow the paper's notation
    (T tokens, K = K_orig, K_base) with d = H and E = N."""
    name: str
    T: int
    d: int
    E: int
    I: int
    K: int
    K_base: int
    budget: int                 # routed activations for this layer (T*K_l in the paper)
    dtype: str                  # "f32" | "bf16"
    I_shared: int = 0           # fused width of the always-on shared expert(s); 0 = none
    I_shared_each: int = 0      # width of one real shared expert (sets the W2 variance)
    shared_gate: bool = False   # Qwen-style sigmoid gate on the shared expert
    bias_kind: str = "none"     # "none" | "normal" (variance 0.5) | "zipf" (s = 1.1)

    def with_(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


def tiny(budget: int = 64, K_base: int = 1) -> Workload:
    return Workload("tiny_fp32", T=64, d=128, E=8, I=256, K=2, K_base=K_base,
                    budget=budget, dtype="f32")


def deepseek_decode(budget: int = 96) -> Workload:
    return Workload("deepseek_v2_lite_decode", T=32, d=2048, E=64, I=1408, K=6, K_base=1,
                    budget=budget, dtype="bf16", I_shared=2816, I_shared_each=1408)


def deepseek_prefill(budget: int = 12288, T: int = 4096) -> Workload:
    return Workload("deepseek_v2_lite_prefill", T=T, d=2048, E=64, I=1408, K=6, K_base=1,
                    budget=budget, dtype="bf16", I_shared=2816, I_shared_each=1408,
                    bias_kind="normal")


def qwen_moe(budget: int = 4096, T: int = 2048) -> Workload:
    return Workload("qwen15_moe_a27b", T=T, d=2048, E=60, I=1408, K=4, K_base=1,
                    budget=budget, dtype="bf16", I_shared=5632, I_shared_each=5632,
                    shared_gate=True)


def olmoe(budget: int = 8192, T: int = 2048) -> Workload:
    """OLMoE-1B-7B-shaped layer (Table 1: 64 experts, Top-8, no shared expert)."""
    return Workload("olmoe_1b_7b", T=T, d=2048, E=64, I=1024, K=8, K_base=1, budget=budget,
                    dtype="bf16")


def deepseek_stack_layer(budget: int, T: int = 8192) -> Workload:
    return Workload("deepseek_v2_lite_stack_layer", T=T, d=2048, E=64, I=1408, K=6,
                    K_base=1, budget=budget, dtype="bf16", I_shared=2816,
                    I_shared_each=1408, bias_kind="zipf")


def _gen(name: str, seed: int, layer: int, device: str) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000003 + _TENSOR_IDS[name] * 1009 + layer)
    return g


def _normal(shape, var: float, name: str, seed: int, layer: int, dtype: torch.dtype,
            device: str) -> torch.Tensor:
    g = _gen(name, seed, layer, device)
    t = torch.randn(shape, generator=g, dtype=torch.float32, device=device)
    t.mul_(math.sqrt(var))
    return t.to(dtype)


def make_layer(w: Workload, seed: int = BASE_SEED, layer: int = 0,
               device: str = "cpu", only=None) -> dict:
    """Draw the tensors of one layer.  Values depend on (seed, layer, tensor
    name, device kind) and the tensor's shape only, never on which other tensors
    are drawn.  `only` (a collection of names) restricts what is generated; the
    rest is None.  Matrices are row-major: X [T,d]; Wg [d,E]; W1,W3 [E,d,I];
    W2 [E,I,d]; Ws1,Ws3 [d,I_shared]; Ws2 [I_shared,d]; w_sg [d]; bias [E] fp32.
    bf16 workloads hold round-to-nearest-even bf16 values."""
    dt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    names = ("X", "Wg", "W1", "W3", "W2", "bias", "Ws1", "Ws3", "Ws2", "w_sg")
    want = set(names if only is None else only)
    out = {n: None for n in names}

    def draw(name, shape, var, dtype=dt):
        if name in want:
            out[name] = _normal(shape, var, name, seed, layer, dtype, device)

    draw("X", (w.T, w.d), 1.0)
    draw("Wg", (w.d, w.E), 1.0 / w.d)
    draw("W1", (w.E, w.d, w.I), 1.0 / w.d)
    draw("W3", (w.E, w.d, w.I), 1.0 / w.d)
    draw("W2", (w.E, w.I, w.d), 1.0 / w.I)
    if w.bias_kind == "normal":
        draw("bias", (w.E,), 0.5, torch.float32)
    elif w.bias_kind == "zipf" and "bias" in want:
        g = _gen("perm", seed, layer, "cpu")
        perm = torch.randperm(w.E, generator=g)
        out["bias"] = (-1.1 * torch.log(perm.to(torch.float32) + 1.0)).to(device)
    if w.I_shared > 0:
        each = w.I_shared_each or w.I_shared
        draw("Ws1", (w.d, w.I_shared), 1.0 / w.d)
        draw("Ws3", (w.d, w.I_shared), 1.0 / w.d)
        draw("Ws2", (w.I_shared, w.d), 1.0 / each)
        if w.shared_gate:
            draw("w_sg", (w.d,), 1.0 / w.d)
    return out


def make_scores(T: int, E: int, seed: int = BASE_SEED, temperature: float = 1.0,
                quantize_levels: Optional[int] = None) -> torch.Tensor:
    """Routing-score-like rows for the selection/dispatch tests: positive fp32
    rows that sum to about one.  With quantize_levels the values are snapped to
    a coarse grid so that many exact ties occur."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed * 7919 + T * 31 + E)
    u = torch.rand((T, E), generator=g, dtype=torch.float64).clamp_min_(1e-12)
    e = (-torch.log(u)) ** temperature
    s = (e / e.sum(dim=1, keepdim=True)).to(torch.float32)
    if quantize_levels:
        s = torch.round(s * quantize_levels) / quantize_levels
    return s.contiguous()


def stack_budgets(L: int, T: int, K: int, K_base: int, ratio: float,
                  seed: int = BASE_SEED) -> list:
    """Per-layer budgets for the multi-layer stack workload: Dirichlet(2) shares
    of ratio*L*T*K, clipped to [T*max(K_base,1), T*K], the remainder spread so
    that the total is exact.  (In the paper these come from Alloc-L's dynamic
    programme, Section 3.2; here they are a seeded stand-in.)"""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed * 1000003 + _TENSOR_IDS["budget"] * 1009)
    # Gamma(2,1) draws as sums of two exponentials from the seeded generator
    u = torch.rand((L, 2), generator=g, dtype=torch.float64).clamp_min_(1e-12)
    shares = (-torch.log(u)).sum(dim=1)
    shares = shares / shares.sum()
    total = int(round(ratio * L * T * K))
    lo, hi = T * max(K_base, 1), T * K
    b = [min(hi, max(lo, int(round(float(p) * total)))) for p in shares]
    diff = total - sum(b)
    step = 1 if diff > 0 else -1
    i = 0
    while diff != 0:
        room = (hi - b[i]) if step > 0 else (b[i] - lo)
        if room > 0:
            take = min(room, max(1, abs(diff) // L))
            b[i] += step * take
            diff -= step * take
        i = (i + 1) % L
    return b


def sensitivity_matrix(L: int, K: int, seed: int = BASE_SEED) -> list:
    """A seeded stand-in for the sensitivity matrix S [L, K] that Alloc-L profiles on a
    calibration set (Section 3.2, Algorithm 1; neither the models nor the data are
    available here): row i is the loss of layer i with k = 1..K experts per token,
    decreasing in k with diminishing returns, the scale of the drop differing from
    layer to layer (shallow and deep layers are more sensitive in the paper's figures)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed * 1000003 + _TENSOR_IDS["budget"] * 1009 + 77)
    u = torch.rand((L, K), generator=g, dtype=torch.float64)
    rows = []
    for i in range(L):
        depth = abs(2.0 * i / max(L - 1, 1) - 1.0)           # 1 at both ends, 0 in the middle
        scale = 0.5 + 1.5 * depth + float(u[i, 0])
        gains = sorted((float(v) * scale / (j + 1) for j, v in enumerate(u[i, 1:])), reverse=True)
        row = [10.0 + scale * 2.0]
        for gain in gains:
            row.append(row[-1] - gain)
        rows.append(row)
    return rows
