"""GPU parity of the whole budgeted MoE layer (allocmoe_moe_forward) with the
CPU oracle.  Protocol: the GPU's scores are checked against the oracle's within
a small absolute tolerance, then the oracle's selection/dispatch is run from
the GPU's scores so that indices compare bit-exactly; the layer output is
compared by scaled max error  max|y - y_ref| / max|y_ref|  against 1e-4 (fp32)
or 2e-2 (bf16 inputs, fp32 accumulation)."""
import pytest
import torch

import oracle
from paper_2604_08133_amd import synth
from paper_2604_08133_amd.layer import DeviceLayer

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


def scaled_err(got, want):
    return float((got.double() - want.double()).abs().max() / want.double().abs().max().clamp_min(1e-30))


def elementwise_rel_err(got, want, floor_frac=0.05):
    """max |y - y_ref| / max(|y_ref|, floor), floor = floor_frac * max|y_ref|: the relative
    error element by element, with an absolute floor because outputs cross zero.  Reported
    next to the scaled error; the gate is the scaled error."""
    want = want.double()
    floor = floor_frac * want.abs().max().clamp_min(1e-30)
    return float(((got.double() - want).abs() / want.abs().clamp_min(floor)).max())


def stratified_tokens(expert_offsets, row_token, T, bm=256, dense_rows=256, per_tile="blocks"):
    """Tokens chosen from the oracle's dispatch so that the rows behind them hit every tile
    of the grouped GEMM's tile map (an expert's rows split evenly over ceil(rows / bm)
    tiles), the first and the last row of every tile and, with per_tile="blocks", one row
    of every 32-row block of every tile; plus the first and the last row of every
    dense_rows-row tile of the shared expert (whose rows are the tokens themselves)."""
    rows = set()
    offs = expert_offsets.tolist()
    for e in range(len(offs) - 1):
        n_rows = offs[e + 1] - offs[e]
        if n_rows == 0:
            continue
        n_tiles = (n_rows + bm - 1) // bm
        rt = (n_rows + n_tiles - 1) // n_tiles
        for i in range(n_tiles):
            first = offs[e] + i * rt
            cnt = min(rt, n_rows - i * rt)
            rows.update((first, first + cnt - 1))
            if per_tile == "blocks":
                rows.update(first + b for b in range(0, cnt, 32))
    toks = {int(row_token[r]) for r in rows}
    for t0 in range(0, T, dense_rows):
        toks.update((t0, min(T, t0 + dense_rows) - 1))
    return sorted(toks)


def check_layer(w, layer, budget=None, K_base=None, tokens=None, dev=None, tag="", ref_layer=None):
    """ref_layer: the tensors the oracle computes with where they differ from what the
    device layer was built from (quantised weights: the values the codes stand for).
    tokens: None (all), a list, or a function (expert_offsets, row_token) -> list that
    picks the checked tokens from the oracle's dispatch."""
    budget = w.budget if budget is None else budget
    K_base = w.K_base if K_base is None else K_base
    dev = dev or DeviceLayer(w, layer)
    layer = ref_layer or layer
    print(f"forward {w.name} T={w.T} B={budget} Kb={K_base} {tag}", flush=True)
    Y = dev.forward(budget=budget, K_base=K_base)
    torch.cuda.synchronize()
    mid = {k: v.cpu() for k, v in dev.intermediates(budget, K_base).items()}
    Y = Y.cpu()

    ref_scores = oracle.softmax(oracle.gate_logits(layer["X"], layer["Wg"], layer.get("bias")))
    assert torch.allclose(mid["scores"], ref_scores, atol=2e-6, rtol=1e-5), "scores"
    if callable(tokens):
        ids, s = oracle.topk(mid["scores"], w.K)
        kept, _ = oracle.alloc_t(s, K_base, budget)
        offs, row_token, _, _ = oracle.dispatch(ids, kept, w.E)
        tokens = tokens(offs, row_token)
        print(f"  outputs checked on {len(tokens)} tokens chosen from the dispatch", flush=True)
    ref = oracle.forward(layer, w.K, K_base, budget, scores=mid["scores"], tokens=tokens)
    for k in ("topk_ids", "topk_s", "keep_count", "expert_offsets", "row_token", "row_rank",
              "inv_row"):
        assert torch.equal(mid[k], ref[k]), k
    assert int(mid["keep_count"].sum()) == budget
    if w.shared_gate:
        assert torch.allclose(mid["shared_gate"].double(), ref["sgate"], atol=1e-5)
    got = Y if tokens is None else Y[list(tokens)]
    err = scaled_err(got, ref["Y"])
    print(f"  scaled max err {err:.3e}; element-wise relative err (floor 5 % of max|y|) "
          f"{elementwise_rel_err(got, ref['Y']):.3e}", flush=True)
    assert err <= TOL[w.dtype], err
    assert torch.isfinite(Y.float()).all()
    return dev


# ------------------------------------------------------------------ fp32, tiny

@pytest.mark.parametrize("Kb,B", [(1, 64), (0, 64), (1, 96), (1, 128), (0, 5), (0, 0), (2, 128)])
def test_tiny_fp32(Kb, B):
    w = synth.tiny(budget=B, K_base=Kb)
    check_layer(w, synth.make_layer(w))


def test_fp32_odd_shapes_with_gated_shared_expert():
    w = synth.Workload("odd_f32", T=37, d=100, E=5, I=72, K=3, K_base=1, budget=61, dtype="f32",
                       I_shared=40, I_shared_each=40, shared_gate=True, bias_kind="normal")
    check_layer(w, synth.make_layer(w, seed=21))


# ------------------------------------------------------------ bf16, small sizes

@pytest.mark.parametrize("T,budget,Kb", [(200, 400, 1), (200, 800, 1), (200, 333, 0), (7, 9, 1),
                                         (129, 129, 1)])
def test_bf16_ragged_tiles(T, budget, Kb):
    w = synth.Workload("ragged_bf16", T=T, d=256, E=16, I=192, K=4, K_base=Kb, budget=budget,
                       dtype="bf16", I_shared=128, I_shared_each=128, bias_kind="normal")
    check_layer(w, synth.make_layer(w, seed=31))


def test_bf16_skewed_experts_and_gate():
    w = synth.Workload("skew_bf16", T=300, d=128, E=60, I=64, K=4, K_base=1, budget=700,
                       dtype="bf16", I_shared=256, I_shared_each=256, shared_gate=True,
                       bias_kind="zipf")
    check_layer(w, synth.make_layer(w, seed=32))


def test_bf16_no_shared_expert():
    w = synth.Workload("olmoe_like", T=96, d=128, E=64, I=128, K=8, K_base=1, budget=400,
                       dtype="bf16")
    check_layer(w, synth.make_layer(w, seed=33))


@pytest.mark.parametrize("T,E,K,budget,Kb,I,Ish,bias", [
    (300, 8, 3, 500, 1, 128, 128, "normal"),    # routed + shared on the tiled kernel, partial tiles
    (700, 4, 2, 1000, 1, 256, 256, "zipf"),     # several 128-row tiles per expert, skewed
    (100, 4, 3, 200, 1, 128, 128, "none"),      # routed tiled, shared on the streaming kernel
    (200, 64, 2, 300, 1, 128, 256, "normal"),   # routed streaming, shared tiled
    (513, 6, 4, 2052, 0, 384, 0, "zipf"),       # full budget, no shared expert, K_base = 0
])
def test_bf16_tiled_kernel_paths(T, E, K, budget, Kb, I, Ish, bias):
    w = synth.Workload("tiled_bf16", T=T, d=256, E=E, I=I, K=K, K_base=Kb, budget=budget,
                       dtype="bf16", I_shared=Ish, I_shared_each=Ish, bias_kind=bias)
    check_layer(w, synth.make_layer(w, seed=51))


def test_bf16_more_tokens_than_the_single_workgroup_plan_takes():
    # T = 9000: selection and dispatch on the large-size kernels, tile map with many
    # tiles per expert; indices on all tokens, outputs on a seeded sample
    w = synth.Workload("big_T_bf16", T=9000, d=256, E=16, I=128, K=4, K_base=1, budget=20000,
                       dtype="bf16", I_shared=128, I_shared_each=128, bias_kind="zipf")
    check_layer(w, synth.make_layer(w, seed=52), tokens=sample_tokens(w.T, 16, 5))


# ------------------------------------------------- the paper-shaped workloads

def test_deepseek_decode_full():
    w = synth.deepseek_decode()
    layer = synth.make_layer(w)
    dev = check_layer(w, layer)                       # 0.5x budget: B = 96
    check_layer(w, layer, budget=192, dev=dev)        # original Top-6
    del dev
    for T, budget in ((1, 3), (5, 17)):               # a single token; a few tokens, ragged budget
        wt = w.with_(T=T, budget=budget)
        lt = dict(layer)
        lt["X"] = layer["X"][:T].contiguous()
        check_layer(wt, lt, tag=f"(T={T})")


def test_qwen_shape_reduced_tokens():
    w = synth.qwen_moe(budget=96, T=48)
    layer = synth.make_layer(w)
    check_layer(w, layer)


def test_olmoe_shape_no_shared_expert():
    # Top-8 of 64 experts, no shared expert: reduced token count, tile-kernel path
    w = synth.olmoe(budget=4 * 256, T=256)
    layer = synth.make_layer(w)
    tokens = sample_tokens(w.T, 24, seed=8)           # outputs checked on a sample, indices on all
    dev = check_layer(w, layer, tokens=tokens)                        # 16 rows per expert: tile kernel
    check_layer(w, layer, budget=8 * 256, tokens=tokens, dev=dev)     # original Top-8, tile kernel
    check_layer(w, layer, budget=256, K_base=1, tokens=tokens, dev=dev)   # Top-1 only: streaming kernel


@pytest.fixture(scope="module")
def deepseek_big():
    """DeepSeek-V2-Lite-shaped weights shared by the full-size tests."""
    w = synth.deepseek_stack_layer(budget=24576, T=8192)
    layer = synth.make_layer(w, seed=synth.BASE_SEED, layer=1)
    dev = DeviceLayer(w, layer)
    return w, layer, dev


def sample_tokens(T, n, seed):
    g = torch.Generator().manual_seed(seed)
    return sorted(torch.randperm(T, generator=g)[:n].tolist())


def test_deepseek_prefill_full_size_sampled(deepseek_big):
    # T = 4096, B = 12288 (0.5x), normal popularity bias; indices checked on all tokens,
    # outputs on the tokens of stratified_tokens: every tile of the tile map, every 32-row
    # block of every tile, each tile's first and last row, and the first and last row of
    # every 256-row tile of the shared expert (a few hundred tokens).
    w8, layer8, _ = deepseek_big
    w = synth.deepseek_prefill()
    layer = dict(layer8)
    layer["X"] = layer8["X"][:w.T].contiguous()
    layer["bias"] = synth.make_layer(w, only=("bias",))["bias"]
    dev = DeviceLayer(w, layer)
    pick = lambda offs, rt: stratified_tokens(offs, rt, w.T)
    check_layer(w, layer, tokens=pick, dev=dev)
    # full budget: first and last row of every tile
    pick_ends = lambda offs, rt: stratified_tokens(offs, rt, w.T, per_tile="ends", dense_rows=w.T)
    check_layer(w, layer, budget=24576, tokens=pick_ends, dev=dev, tag="(1.0x)")
    # 640 tokens of the same layer: both groups on the tile kernel with partly filled
    # tiles, the shared expert in tiles of fewer than 256 rows
    del dev
    w6 = w.with_(T=640, budget=3 * 640)
    layer6 = dict(layer)
    layer6["X"] = layer["X"][:640].contiguous()
    check_layer(w6, layer6, tokens=sample_tokens(640, 6, 4), tag="(T=640)")


def test_deepseek_stack_layer_full_size_sampled(deepseek_big):
    # T = 8192 with Zipf popularity skew; a mid budget (outputs on stratified_tokens: every
    # tile, every 32-row block of every tile, first and last rows, the shared expert's row
    # tiles), the smallest budget (B = T) and a ragged one (first and last row of every tile)
    w, layer, dev = deepseek_big
    check_layer(w, layer, budget=24576, tokens=lambda offs, rt: stratified_tokens(offs, rt, w.T),
                dev=dev)
    pick_ends = lambda offs, rt: stratified_tokens(offs, rt, w.T, per_tile="ends", dense_rows=w.T)
    check_layer(w, layer, budget=8192, tokens=pick_ends, dev=dev, tag="(B=T)")
    check_layer(w, layer, budget=31337, tokens=pick_ends, dev=dev, tag="(ragged)")


def test_qwen_full_size_sampled():
    # the Qwen1.5-MoE-A2.7B-shaped layer at the size bench.py times: T = 2048, 60 experts, Top-4, gated shared
    # expert of width 5632; the swept budgets 0.5x / 0.75x / 1.0x; indices on all tokens,
    # outputs on stratified_tokens (0.5x: every tile, every 32-row block, first and last
    # rows, the shared expert's row tiles; the other budgets: first and last row of every
    # tile).  Weights made on the CPU once.
    w = synth.qwen_moe()
    layer = synth.make_layer(w)
    dev = DeviceLayer(w, layer)
    check_layer(w, layer, tokens=lambda offs, rt: stratified_tokens(offs, rt, w.T), dev=dev)   # 0.5x
    pick_ends = lambda offs, rt: stratified_tokens(offs, rt, w.T, per_tile="ends", dense_rows=w.T)
    check_layer(w, layer, budget=6144, tokens=pick_ends, dev=dev, tag="(0.75x)")
    check_layer(w, layer, budget=8192, tokens=pick_ends, dev=dev, tag="(1.0x)")


def test_forward_is_bitwise_reproducible():
    w = synth.Workload("repro", T=500, d=256, E=32, I=128, K=4, K_base=1, budget=1100,
                       dtype="bf16", I_shared=128, I_shared_each=128)
    dev = DeviceLayer(w, synth.make_layer(w, seed=41))
    a = dev.forward().clone()
    ia = {k: v.clone() for k, v in dev.intermediates().items()}
    for _ in range(5):
        b = dev.forward()
        torch.cuda.synchronize()
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
        for k, v in dev.intermediates().items():
            assert torch.equal(ia[k].view(torch.uint8), v.view(torch.uint8)), k


# ------------------------------------------------------------- argument checks

def test_bf16_forward_rejects_misaligned_rows():
    from paper_2604_08133_amd import binding as B
    w = synth.Workload("align_bf16", T=8, d=128, E=4, I=64, K=2, K_base=1, budget=12, dtype="bf16")
    dev = DeviceLayer(w, synth.make_layer(w, seed=41))
    desc = dev.desc()
    ws = dev.workspace(desc)
    flat = torch.empty(w.T * w.d + 8, dtype=torch.bfloat16, device=dev.device)
    Y_ok = flat[:w.T * w.d].view(w.T, w.d)
    Y_odd = flat[1:w.T * w.d + 1].view(w.T, w.d)          # 2 bytes off a 16-byte boundary
    B.allocmoe_moe_forward(desc, dev.X, dev.weights, Y_ok, ws)
    with pytest.raises(B.AllocMoEError) as e:
        B.allocmoe_moe_forward(desc, dev.X, dev.weights, Y_odd, ws)
    assert e.value.status == B.EINVAL
    torch.cuda.synchronize()
