#!/usr/bin/env python3
"""Benchmark of the budget-constrained MoE layer forward on one MI355X.

A step is one pass of the whole hot path (route -> Alloc-T selection ->
dispatch -> SwiGLU expert networks over the selected pairs + shared expert ->
combine) over one batch of seeded synthetic input that is already resident in
HBM.  Prints ONE JSON line: the metric, the roofline of the dominant kernel and the
CPU oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload decode|prefill|qwen|olmoe|stack]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published


def parse_args():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=200)
    p.add_argument("--warmup", type=int, default=20)
    p.add_argument("--workload", default="decode",
                   choices=["decode", "prefill", "qwen", "olmoe", "stack"])
    p.add_argument("--budget-ratio", type=float, default=0.5,
                   help="layer budget as a fraction of T*K (the metric is quoted at 0.5)")
    p.add_argument("--tokens", type=int, default=0,
                   help="override the workload's token count T (budget = ratio*T*K): the step "
                        "time against batch size")
    p.add_argument("--layers", type=int, default=26, help="layers of the stack workload")
    p.add_argument("--budgets", default="dirichlet",
                   choices=["dirichlet", "alloc-l", "ascending", "descending"],
                   help="stack workload: per-layer budgets from the seeded Dirichlet(2) draw "
                        "(the configuration the metric names) or from Alloc-L's dynamic "
                        "programme on a seeded synthetic sensitivity matrix, or from the "
                        "Ascending / Descending schedule (budget = T*K_l)")
    p.add_argument("--weights", default="bf16", choices=["bf16", "fp8"],
                   help="expert-weight format: bf16 (what the metric names) or the 8-bit variant "
                        "(E4M3 codes + one fp32 scale per output column)")
    p.add_argument("--selector", default="score", choices=["score", "top-p", "relative"],
                   help="token-level selector: Alloc-T (the metric's) or one of the calibrated "
                        "baselines of Appendix A.1, at the same budget")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--copy-probe", action="store_true",
                   help="only run a plain device copy of 1 GiB (calibrates the rocprofv3 "
                        "FETCH_SIZE / WRITE_SIZE counters)")
    p.add_argument("--cpu-seconds", type=float, default=20.0,
                   help="rough bound on the oracle's CPU time")
    return p.parse_args()


def workload_for(name: str, ratio: float, tokens: int = 0):
    from paper_2604_08133_amd import synth
    if name == "decode":
        w = synth.deepseek_decode()
    elif name == "prefill":
        w = synth.deepseek_prefill()
    elif name == "qwen":
        w = synth.qwen_moe()
    elif name == "olmoe":
        w = synth.olmoe()
    else:
        w = synth.deepseek_stack_layer(budget=0)
    if tokens > 0:
        w = w.with_(T=tokens)
    return w.with_(budget=int(round(ratio * w.T * w.K)))


def traffic_from_profiles(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` measured with rocprofv3 --pmc, read from
    the committed summary profiles/pmc_<workload>.txt (line
    'traffic_bytes_per_launch <kernel> <bytes>'); None if not recorded."""
    path = os.path.join(ROOT, "profiles", f"pmc_{workload}.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == kernel:
                    return float(parts[2])
    except OSError:
        pass
    return None


def cpu_baseline(w, layer, seconds: float):
    """The oracle as it stands, single-threaded, on a bounded sample of the
    same workload: Eq. (1) + candidates + Alloc-T + dispatch for all T tokens,
    Eq. (2) outputs for the first n tokens; tokens/s extrapolated per token for
    the output part."""
    import oracle
    t0 = time.perf_counter()
    scores = oracle.softmax(oracle.gate_logits(layer["X"], layer["Wg"], layer.get("bias")))
    ids, s = oracle.topk(scores, w.K)
    kept, cnt = oracle.alloc_t(s, w.K_base, w.budget)
    oracle.dispatch(ids, kept, w.E)
    sg = oracle.shared_gate(layer["X"], layer["w_sg"]) if layer.get("w_sg") is not None else None
    t_route = time.perf_counter() - t0
    # output rows: time one token, then as many as fit the bound
    done, t_out = 0, 0.0
    n = 1
    while done < w.T:
        toks = list(range(done, min(w.T, done + n)))
        t1 = time.perf_counter()
        oracle.moe_eq2(layer, ids, s, kept, sg, dense=False, tokens=toks)
        t_out += time.perf_counter() - t1
        done += len(toks)
        per_tok = t_out / done
        left = seconds - t_route - t_out
        if left < per_tok:
            break
        n = max(1, min(w.T - done, int(left / per_tok / 2) or 1))
    total = t_route + (t_out / done) * w.T
    return {
        "value": w.T / total, "unit": "tokens/s", "cores": 1, "kind": "oracle",
        "sample": (f"routing+selection+dispatch for all {w.T} tokens ({t_route:.2f} s) + Eq.(2) "
                   f"outputs of the first {done} tokens ({t_out:.2f} s), output time scaled to "
                   f"{w.T} tokens"),
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives are part "
              "of it); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2604_08133_amd import binding as B
    from paper_2604_08133_amd import synth
    from paper_2604_08133_amd.layer import DeviceLayer

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.load()   # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)
    if args.copy_probe:
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes": n, "launches": 5}))
        return

    w = workload_for(args.workload, args.budget_ratio, args.tokens)
    on_cpu = args.workload == "decode"
    # Inputs: generated on the CPU for the small workload (the oracle baseline
    # needs the same bytes), on the GPU for the big ones.  The stack workload is
    # `--layers` independent layers (own weights, own input, own budget: layers of
    # a model interact only through the budgets Alloc-L gives them).
    layer_cpu = synth.make_layer(w, device="cpu") if on_cpu else None
    fp8 = args.weights == "fp8"
    wb = 1 if fp8 else 2          # bytes per stored expert-weight element
    if args.workload == "stack":
        if args.budgets == "alloc-l":
            S = synth.sensitivity_matrix(args.layers, w.K)
            K_l, _ = B.allocmoe_alloc_l(S, int(round(args.budget_ratio * args.layers * w.K)))
            budgets = [w.T * k for k in K_l]
        elif args.budgets in ("ascending", "descending"):
            kind = B.SCHEDULE_ASCENDING if args.budgets == "ascending" else B.SCHEDULE_DESCENDING
            K_l = B.allocmoe_layer_schedule(kind, args.layers, w.K,
                                            int(round(args.budget_ratio * args.layers * w.K)))
            budgets = [w.T * k for k in K_l]
        else:
            budgets = synth.stack_budgets(args.layers, w.T, w.K, w.K_base, args.budget_ratio)
        works = [w.with_(budget=b) for b in budgets]
        devs = [DeviceLayer(wl, synth.make_layer(wl, layer=i, device="cuda"), weights_fp8=fp8)
                for i, wl in enumerate(works)]
    else:
        works = [w]
        devs = [DeviceLayer(w, layer_cpu if on_cpu else synth.make_layer(w, device="cuda"),
                            weights_fp8=fp8)]
    selector = {"score": B.SELECT_SCORE, "top-p": B.SELECT_TOP_P, "relative": B.SELECT_RELATIVE}[args.selector]
    descs = [dv.desc(selector=selector) for dv in devs]
    ws = torch.empty(max(B.allocmoe_workspace_bytes(dc) for dc in descs), dtype=torch.uint8,
                     device="cuda")
    Y = torch.empty((w.T, w.d), dtype=devs[0].dtype, device="cuda")

    def step():
        for dv, dc in zip(devs, descs):
            B.allocmoe_moe_forward(dc, dv.X, dv.weights, Y, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps

    # per-kernel durations: the same steps again through the event-instrumented
    # entry point (HIP events recorded by the library on the launch stream);
    # along the way, read back how many experts each layer activated
    stage_ms = [0.0] * len(B.STAGES)
    n_active_sum, pairs_sum = 0, 0
    for it in range(args.steps):
        for dv, dc, wl in zip(devs, descs, works):
            ms = B.allocmoe_moe_forward_timed(dc, dv.X, dv.weights, Y, ws)
            stage_ms = [a + b for a, b in zip(stage_ms, ms)]
            if it == 0:
                L = B.allocmoe_workspace_layout(dc)
                offs = B.ws_view(ws, L.expert_offsets, (wl.E + 1,), torch.int32).cpu()
                n_active_sum += int(((offs[1:] - offs[:-1]) > 0).sum())
                assert int(offs[-1]) == wl.budget, "selected pairs != layer budget"
                pairs_sum += int(offs[-1])
    stage_ms = [v / args.steps for v in stage_ms]
    stages = dict(zip(B.STAGES, stage_ms))
    nL = len(devs)

    # ---- roofline of the dominant kernel (summed over the layers of a step)
    d, I, Is, T = w.d, w.I, w.I_shared, w.T
    # ffn1 launch = routed rows + shared expert: W1,W3 once per active expert and
    # once for the shared expert; x rows in, H rows out
    ffn1_bytes = (n_active_sum * 2 * d * I * wb + pairs_sum * (d * 2 + I * 2)
                  + nL * (2 * d * Is * wb + T * (d * 2 + Is * 2) if Is else 0))
    if fp8:   # the column scales
        ffn1_bytes += n_active_sum * 2 * I * 4 + (nL * 2 * Is * 4 if Is else 0)
    ffn1_flops = pairs_sum * 2 * d * (2 * I) + nL * T * 2 * d * (2 * Is)
    dom = "ffn1"
    dom_ms = stages[dom]
    targs = "<true, true>" if fp8 else "<true, false>"   # <SwiGLU half, 8-bit weights>
    # (the library moves the routed group to the tile kernel from 8 rows per expert on)
    streaming = args.workload == "decode" if args.tokens <= 0 else pairs_sum < 8 * w.E * nL
    # with --tokens the side of the roofline follows the arithmetic intensity of the launch
    hbm_side = streaming or (args.tokens > 0 and
                             ffn1_flops / ffn1_bytes * HBM_PEAK_GBS / 1e3 < MFMA_BF16_PEAK_TFLOPS)
    kernel_name = ("ffn_bf16_stream_kernel" if streaming else "ffn_bf16_t256_kernel") + targs
    if hbm_side:
        roof = {"bound": "hbm", "achieved": ffn1_bytes / (dom_ms * 1e-3) / 1e9,
                "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    else:
        roof = {"bound": "mfma", "achieved": ffn1_flops / (dom_ms * 1e-3) / 1e12,
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s"}
        # what the roofline allows at this arithmetic intensity: min(peak, flop/byte x HBM)
        roof["attainable"] = min(MFMA_BF16_PEAK_TFLOPS, ffn1_flops / ffn1_bytes * HBM_PEAK_GBS / 1e3)
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = None if fp8 or args.tokens > 0 else traffic_from_profiles(args.workload, dom)
    roof["kernel"] = kernel_name
    roof["kernel_ms"] = dom_ms / nL
    roof["launches_per_step"] = nL
    roof["algorithmic_bytes"] = ffn1_bytes / nL
    roof["algorithmic_flops"] = ffn1_flops / nL

    # whole-step algorithmic traffic and work (context for the step time)
    step_bytes = (n_active_sum * 3 * d * I * wb + nL * 3 * d * Is * wb   # expert + shared weights
                  + nL * (T * d * 2 * 2 + d * w.E * 2)                 # X (gate), Y, Wg
                  + pairs_sum * (d * 2 + 2 * I * 2 + 2 * d * 2)        # x gather, H w+r, O w+r
                  + (nL * T * (d * 2 + 2 * Is * 2 + 2 * d * 2) if Is else 0))
    step_flops = pairs_sum * 6 * d * I + nL * (T * 6 * d * Is + T * 2 * d * w.E)
    step_info = {
        "algorithmic_bytes": step_bytes, "algorithmic_flops": step_flops,
        "hbm_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "mfma_frac": step_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "active_experts": n_active_sum, "layers": nL,
        "stage_ms": {k: round(v, 5) for k, v in stages.items()},
    }

    out = {
        "metric": "budgeted MoE-layer tokens/s at 0.5x budget",
        "value": w.T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name + (f"_x{nL}_layers" if nL > 1 else ""), "T": w.T, "d": w.d,
                   "E": w.E, "I": w.I, "K": w.K, "K_base": w.K_base,
                   "budget": [wl.budget for wl in works] if nL > 1 else w.budget,
                   "budget_ratio": args.budget_ratio, "I_shared": w.I_shared, "selector": args.selector,
                   "weights": ("bf16" if not fp8 else "e4m3 codes + fp32 column scales (bf16 matrix "
                               "cores after widening in registers)")
                   + ", re-tiled once by allocmoe_pack_weights, outside the timed region"},
        "roofline": roof,
        "step": step_info,
    }
    if not args.no_cpu_baseline:
        if layer_cpu is None:
            # bounded sample for the big workloads: the same shapes at T = 32 tokens
            ws_small = w.with_(T=32, budget=int(round(args.budget_ratio * 32 * w.K)))
            cb = cpu_baseline(ws_small, synth.make_layer(ws_small, device="cpu"), args.cpu_seconds)
            cb["sample"] = f"same layer shapes at T=32 tokens: " + cb["sample"]
        else:
            cb = cpu_baseline(w, layer_cpu, args.cpu_seconds)
        out["cpu_baseline"] = cb
    print(json.dumps(out))


if __name__ == "__main__":
    main()
