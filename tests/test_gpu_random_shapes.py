"""GPU parity of the layer forward over seeded random shapes: token counts on both
sides of every kernel-choice threshold, expert counts 1 .. 64, any K_base <= K, budgets
anywhere in [T*K_base, T*K], with and without shared expert / gate / popularity bias /
8-bit weights.  Indices on all tokens, outputs on a seeded sample (same protocol and
tolerances as tests/test_gpu_layer.py)."""
import random

import pytest

from paper_2604_08133_amd import synth
from paper_2604_08133_amd.layer import DeviceLayer
from tests.test_gpu_fp8 import quantised_reference
from tests.test_gpu_layer import check_layer, sample_tokens

pytestmark = pytest.mark.gpu

SMALL_T = [1, 2, 7, 16, 17, 33, 64, 65, 100, 129, 200, 300, 513, 700]
LARGE_T = [1000, 2048, 3000, 4097, 8192, 8193, 9000]


def draw_case(rng, token_counts):
    d = rng.choice([128, 256, 512])
    I = rng.choice([64, 128, 192, 256, 384])
    Ish = rng.choice([0, 64, 128, 256])
    E = rng.choice([1, 2, 3, 5, 8, 16, 17, 33, 60, 64])
    K = rng.randint(1, min(E, 8))
    Kb = rng.randint(0, K)
    T = rng.choice(token_counts)
    budget = rng.randint(T * Kb, T * K)
    fp8 = rng.random() < 0.3 and d % 128 == 0 and I % 128 == 0 and Ish % 128 == 0
    gate = Ish > 0 and rng.random() < 0.3
    bias = rng.choice(["none", "normal", "zipf"])
    w = synth.Workload("random_shape", T=T, d=d, E=E, I=I, K=K, K_base=Kb, budget=budget,
                       dtype="bf16", I_shared=Ish, I_shared_each=Ish, shared_gate=gate,
                       bias_kind=bias)
    return w, fp8, rng.randint(1, 10**6)


@pytest.mark.parametrize("stream_seed,token_counts,n_cases", [(11, SMALL_T, 60), (12, LARGE_T, 25)])
def test_random_shapes(stream_seed, token_counts, n_cases):
    rng = random.Random(stream_seed)
    for _ in range(n_cases):
        w, fp8, seed = draw_case(rng, token_counts)
        layer = synth.make_layer(w, seed=seed)
        toks = sample_tokens(w.T, min(w.T, 6), seed)
        tag = f"d={w.d} E={w.E} I={w.I} K={w.K} Ish={w.I_shared} gate={w.shared_gate} " \
              f"bias={w.bias_kind} fp8={fp8} seed={seed}"
        if fp8:
            ref, _ = quantised_reference(layer)
            check_layer(w, layer, dev=DeviceLayer(w, layer, weights_fp8=True), ref_layer=ref,
                        tokens=toks, tag=tag)
        else:
            check_layer(w, layer, tokens=toks, tag=tag)
