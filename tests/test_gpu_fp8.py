"""8-bit (E4M3 + column scale) expert weights on the device: the packed codes and scales
against the oracle's quantiser, byte for byte, and the layer forward against the oracle
run on the values the codes stand for.
"""
import numpy as np
import pytest
import torch

from oracle import quant
from paper_2604_08133_amd import binding as B, synth
from paper_2604_08133_amd.layer import DeviceLayer
from tests.test_gpu_layer import check_layer, sample_tokens, stratified_tokens

pytestmark = pytest.mark.gpu


def align256(n):
    return (n + 255) // 256 * 256


def fragments(codes):
    """codes uint8 [G, Kd, N] -> the packed order [G, N/32, Kd/32 * 1024] documented in
    the header: lane l of fragment (nb, kb) holds k = 32 kb + 16 h + 8 (l/32) + i in byte
    8 h + i, column 32 nb + l%32."""
    G, Kd, N = codes.shape
    kb, l, h, i = np.meshgrid(np.arange(Kd // 32), np.arange(64), np.arange(2), np.arange(8),
                              indexing="ij")
    k = 32 * kb + 16 * h + 8 * (l // 32) + i                     # [KB, 64, 2, 8]
    col = l % 32
    out = np.empty((G, N // 32, Kd // 32, 64, 2, 8), dtype=np.uint8)
    for nb in range(N // 32):
        out[:, nb] = codes[:, k, 32 * nb + col]
    return out.reshape(G, N // 32, -1)


def quantised_reference(layer):
    """(ref_layer for the oracle: fp32 tensors holding the values the codes stand for;
    codes and scales per matrix)."""
    ref = {k: (v.float() if isinstance(v, torch.Tensor) and v.dtype == torch.bfloat16 else v)
           for k, v in layer.items()}
    q = {}
    for name in ("W1", "W3", "W2", "Ws1", "Ws3", "Ws2"):
        if layer.get(name) is None:
            continue
        codes, scale = quant.quantise_columns(layer[name].float().numpy())
        q[name] = (codes, scale)
        ref[name] = torch.from_numpy(quant.dequantise(codes, scale).astype(np.float32))
    return ref, q


def test_packed_codes_and_scales_bit_exact():
    w = synth.Workload("fp8_pack", T=8, d=128, E=3, I=256, K=2, K_base=1, budget=12, dtype="bf16",
                       I_shared=128, I_shared_each=128)
    layer = synth.make_layer(w, seed=71)
    layer["W1"][1, :, 5] = 0            # an all-zero column: scale 1, codes 0
    _, q = quantised_reference(layer)
    dev = DeviceLayer(w, layer, weights_fp8=True)
    packed = dev.packed.cpu().numpy()
    E, d, I, Is = w.E, w.d, w.I, w.I_shared
    off = 0

    def take(n):
        nonlocal off
        at = off
        off = align256(off + n)
        return at

    q13, q2, qs13, qs2 = take(E * 2 * d * I), take(E * I * d), take(2 * d * Is), take(Is * d)
    take(5 * 16 * d * 2)                                  # the bf16 gate (5 blocks of 16 columns)
    sc13, sc2, scs13, scs2 = take(E * 2 * I * 4), take(E * d * 4), take(2 * Is * 4), take(d * 4)
    assert off == packed.size

    def region(at, n):
        return packed[at:at + n]

    want13 = np.concatenate([fragments(q["W1"][0]), fragments(q["W3"][0])], axis=2).reshape(-1)
    assert np.array_equal(region(q13, want13.size), want13)
    want2 = fragments(q["W2"][0]).reshape(-1)
    assert np.array_equal(region(q2, want2.size), want2)
    wants13 = np.concatenate([fragments(q["Ws1"][0][None]), fragments(q["Ws3"][0][None])], axis=2).reshape(-1)
    assert np.array_equal(region(qs13, wants13.size), wants13)
    wants2 = fragments(q["Ws2"][0][None]).reshape(-1)
    assert np.array_equal(region(qs2, wants2.size), wants2)

    def scales(at, shape):
        return region(at, int(np.prod(shape)) * 4).view(np.float32).reshape(shape)

    assert np.array_equal(scales(sc13, (E, 2, I)), np.stack([q["W1"][1], q["W3"][1]], axis=1))
    assert np.array_equal(scales(sc2, (E, d)), q["W2"][1])
    assert np.array_equal(scales(scs13, (2, Is)), np.stack([q["Ws1"][1], q["Ws3"][1]]))
    assert np.array_equal(scales(scs2, (d,)), q["Ws2"][1])
    assert scales(sc13, (E, 2, I))[1, 0, 5] == 1.0


@pytest.mark.parametrize("T,E,K,budget,Kb,I,Ish,gate", [
    (40, 8, 3, 70, 1, 128, 128, False),       # ragged row tiles, several experts per tile size
    (7, 4, 2, 9, 1, 256, 0, False),           # no shared expert
    (300, 16, 4, 700, 0, 128, 256, True),     # routed and shared expert on the tile kernel
    (700, 4, 2, 1000, 1, 256, 256, False),    # several 256-row tiles per expert, partial tiles
    (100, 4, 3, 200, 1, 128, 128, False),     # routed on the tile kernel, shared streaming
    (200, 64, 2, 300, 1, 128, 256, False),    # routed streaming, shared on the tile kernel
    (513, 6, 4, 2052, 0, 384, 0, False),      # full budget, no shared expert
])
def test_layer_with_fp8_weights(T, E, K, budget, Kb, I, Ish, gate):
    w = synth.Workload("fp8_layer", T=T, d=256, E=E, I=I, K=K, K_base=Kb, budget=budget,
                       dtype="bf16", I_shared=Ish, I_shared_each=Ish, shared_gate=gate,
                       bias_kind="normal")
    layer = synth.make_layer(w, seed=72)
    ref, _ = quantised_reference(layer)
    check_layer(w, layer, dev=DeviceLayer(w, layer, weights_fp8=True), ref_layer=ref, tag="fp8")


def test_deepseek_shapes_with_fp8_weights():
    # the decode workload (weight-streaming kernel), then 1024 tokens of the same layer
    # (tile kernel: 48 rows per expert on average, popularity-biased), outputs on a
    # seeded sample of tokens
    w = synth.deepseek_decode()
    layer = synth.make_layer(w)
    ref, _ = quantised_reference(layer)
    tokens = sample_tokens(w.T, 6, seed=9)
    check_layer(w, layer, dev=DeviceLayer(w, layer, weights_fp8=True), ref_layer=ref,
                tokens=tokens, tag="fp8")
    w2 = synth.deepseek_prefill().with_(T=1024, budget=3 * 1024)
    extra = synth.make_layer(w2, only=("X", "bias"))
    layer2, ref2 = dict(layer), dict(ref)
    for k in ("X", "bias"):
        layer2[k] = extra[k]
        ref2[k] = extra[k].float()
    check_layer(w2, layer2, dev=DeviceLayer(w2, layer2, weights_fp8=True), ref_layer=ref2,
                tokens=sample_tokens(w2.T, 6, seed=10), tag="fp8 tile kernel")
    # the prefill workload at full size (T = 4096, I = 1408: the contraction of the second
    # GEMM is 22 steps of 64, which leaves the 8-bit loop's half pass): first and last row
    # of every tile of the tile map
    w3 = synth.deepseek_prefill()
    extra = synth.make_layer(w3, only=("X", "bias"))
    layer3, ref3 = dict(layer), dict(ref)
    for k in ("X", "bias"):
        layer3[k] = extra[k]
        ref3[k] = extra[k].float()
    check_layer(w3, layer3, dev=DeviceLayer(w3, layer3, weights_fp8=True), ref_layer=ref3,
                tokens=lambda offs, rt: stratified_tokens(offs, rt, w3.T, per_tile="ends",
                                                          dense_rows=1024),
                tag="fp8 tile kernel, full size")


def test_fp8_flag_is_checked():
    # 8-bit weights need bf16 and dimensions that are multiples of 128
    with pytest.raises(B.AllocMoEError):
        B.allocmoe_packed_bytes(B.make_desc(8, 192, 4, 128, 2, 1, 8, "bf16", weights_fp8=True))
    with pytest.raises(B.AllocMoEError):
        B.allocmoe_workspace_bytes(B.make_desc(8, 128, 4, 128, 2, 1, 8, "f32", weights_fp8=True))
