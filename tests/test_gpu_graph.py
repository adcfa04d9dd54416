"""allocmoe_moe_forward under HIP graph capture: the call enqueues kernels (and, for
prefill shapes, an event fork/join with the library's side stream) and nothing else, so
a caller may capture it once and replay it.  Every replay is checked against the eager
result, with eager work and synchronisations between the replays and with new input
written into the captured buffers.
"""
import pytest
import torch

from paper_2604_08133_amd import binding as B, synth
from paper_2604_08133_amd.layer import DeviceLayer

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kind", ["decode-shaped", "prefill-shaped"])
def test_forward_replays_from_a_graph(kind):
    if kind == "decode-shaped":      # both groups on the streaming kernel, one stream
        w = synth.Workload("graph_decode", T=24, d=256, E=16, I=128, K=4, K_base=1, budget=48,
                           dtype="bf16", I_shared=128, I_shared_each=128, bias_kind="normal")
    else:                            # tile kernel, shared expert on the library's side stream
        w = synth.Workload("graph_prefill", T=300, d=256, E=8, I=128, K=3, K_base=1, budget=500,
                           dtype="bf16", I_shared=128, I_shared_each=128, bias_kind="normal")
    layer = synth.make_layer(w, seed=81)
    dev = DeviceLayer(w, layer)
    desc = dev.desc()
    ws = dev.workspace(desc)
    X = dev.X.clone()
    Y_graph = torch.empty((w.T, w.d), dtype=dev.dtype, device=dev.device)
    Y_eager = torch.empty_like(Y_graph)
    B.allocmoe_moe_forward(desc, X, dev.weights, Y_eager, ws)     # also creates the side stream
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.allocmoe_moe_forward(desc, X, dev.weights, Y_graph, ws)
    gen = torch.Generator(device="cpu").manual_seed(5)
    for rep in range(4):
        if rep:                                   # new input in the captured buffer
            X.copy_(torch.randn(X.shape, generator=gen).to(X.dtype))
        Y_graph.zero_()
        graph.replay()
        torch.cuda.synchronize()
        B.allocmoe_moe_forward(desc, X, dev.weights, Y_eager, ws)  # eager, same buffers
        torch.cuda.synchronize()
        assert torch.equal(Y_graph, Y_eager), (kind, rep)
        assert torch.isfinite(Y_eager.float()).all() and Y_eager.float().abs().max() > 0
