#!/usr/bin/env python3
"""Benchmark of the budget-constrained MoE layer forward on one MI355X.

A step is one pass of the whole hot path (route -> Alloc-T selection ->
dispatch -> SwiGLU expert networks over the selected pairs + shared expert ->
combine) over one batch of seeded synthetic input that is already resident in
HBM; for the default workload, the 26-layer stack, a step is that pass through all
26 layers.  Prints ONE JSON line: the metric, the roofline of the dominant kernel,
the other workloads at half and full budget, and the CPU oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload stack|decode|prefill|qwen|olmoe]
    python bench.py --ceilings      # the device's measured ceilings only
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
METRIC = "budgeted MoE-layer tokens/s at 0.5x budget"


def parse_args():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=20)
    p.add_argument("--warmup", type=int, default=5)
    p.add_argument("--workload", default="stack",
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
    p.add_argument("--no-sub-workloads", action="store_true",
                   help="skip the decode / prefill / Qwen / OLMoE sub-records and the full-budget run")
    p.add_argument("--copy-probe", action="store_true",
                   help="only run a plain device copy of 1 GiB (calibrates the rocprofv3 "
                        "FETCH_SIZE / WRITE_SIZE counters)")
    p.add_argument("--ceilings", action="store_true",
                   help="only measure the device's ceilings: matrix-core issue loop on zero and on "
                        "N(0,1) operands (with the shader clock), streaming read of 8 GiB, and "
                        "the vendor library's GEMM on the tile kernel's dense shapes")
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


def traffic_from_profiles(workload: str, key: str):
    """HBM bytes per launch (or per layer's expert region) measured with rocprofv3 --pmc,
    read from the committed summary profiles/pmc_<workload>.txt (line
    'traffic_bytes_per_launch <key> <bytes>'); None if not recorded."""
    path = os.path.join(ROOT, "profiles", f"pmc_{workload}.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == key:
                    return float(parts[2])
    except OSError:
        pass
    return None


def host_cpu():
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count()
    return {"nproc": os.cpu_count(), "usable_cores": usable, "cpu_model": model}


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
    out = {
        "value": w.T / total, "unit": "tokens/s", "cores": 1, "kind": "oracle",
        "sample": (f"routing+selection+dispatch for all {w.T} tokens ({t_route:.2f} s) + Eq.(2) "
                   f"outputs of the first {done} tokens ({t_out:.2f} s), output time scaled to "
                   f"{w.T} tokens"),
    }
    out.update(host_cpu())
    return out


def measure_ceilings(with_vendor_gemm: bool = True):
    """The device's own ceilings (include/allocmoe.h, allocmoe_probe_*)."""
    import torch
    from paper_2604_08133_amd import binding as B
    lib = B.load()
    nb = lib.allocmoe_probe_mfma_operand_bytes()
    sink = torch.zeros(lib.allocmoe_probe_sink_bytes(), dtype=torch.uint8, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(20260408)
    ops_rand = torch.randn(nb // 2, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    ops_zero = torch.zeros(nb // 2, device="cuda", dtype=torch.bfloat16)
    out = {"mfma_bf16": {}, "hbm_read": {}}
    for name, ops in (("zeros", ops_zero), ("normal", ops_rand)):
        for waves in (1, 2):
            best = (0.0, 0.0)
            for _ in range(3):   # ~10 ms each
                tf, mhz = B.allocmoe_probe_mfma(ops, waves, 40000 // waves, sink)
                if tf > best[0]:
                    best = (tf, mhz)
            out["mfma_bf16"][f"{name}_{waves}_waves_per_simd"] = {
                "tflops": round(best[0], 1), "shader_mhz": round(best[1])}
    buf = torch.empty(8 << 30, dtype=torch.uint8, device="cuda")
    buf.fill_(1)
    torch.cuda.synchronize()
    for nt in (True, False):
        out["hbm_read"]["non_temporal" if nt else "default"] = {
            "gbs": round(B.allocmoe_probe_hbm_read(buf, nt, 5, sink), 1), "bytes": buf.numel()}
    del buf
    if with_vendor_gemm:
        # context: what the vendor library's GEMM (torch.matmul) sustains on the dense shapes
        # the tile kernel sees (the shared expert of T tokens: K = d, N = 2*I_shared and
        # K = I_shared, N = d)
        out["vendor_gemm_bf16"] = {}
        for (M, K, N) in ((16384, 2048, 5632), (8192, 2048, 5632), (8192, 2816, 2048)):
            a = torch.randn(M, K, device="cuda", dtype=torch.bfloat16)
            b = torch.randn(K, N, device="cuda", dtype=torch.bfloat16) / K ** 0.5
            for _ in range(5):
                c = a @ b
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                c = a @ b
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 20
            out["vendor_gemm_bf16"][f"{M}x{K}x{N}"] = {"us": round(ms * 1e3, 1),
                                                       "tflops": round(2 * M * K * N / ms / 1e9, 1)}
            del a, b, c
    return out


class Bench:
    """One workload resident on the GPU: builds the layers, times steps."""

    def __init__(self, name, ratio, args, tokens=0, layers=1, layer_cpu=None):
        import torch
        from paper_2604_08133_amd import binding as B
        from paper_2604_08133_amd import synth
        from paper_2604_08133_amd.layer import DeviceLayer
        self.B, self.torch = B, torch
        self.name = name
        self.fp8 = args.weights == "fp8"
        w = workload_for(name, ratio, tokens)
        self.w = w
        if name == "stack":
            if args.budgets == "alloc-l":
                S = synth.sensitivity_matrix(layers, w.K)
                K_l, _ = B.allocmoe_alloc_l(S, int(round(ratio * layers * w.K)))
                budgets = [w.T * k for k in K_l]
            elif args.budgets in ("ascending", "descending"):
                kind = B.SCHEDULE_ASCENDING if args.budgets == "ascending" else B.SCHEDULE_DESCENDING
                K_l = B.allocmoe_layer_schedule(kind, layers, w.K, int(round(ratio * layers * w.K)))
                budgets = [w.T * k for k in K_l]
            elif ratio >= 1.0:
                budgets = [w.T * w.K] * layers
            else:
                budgets = synth.stack_budgets(layers, w.T, w.K, w.K_base, ratio)
            self.works = [w.with_(budget=b) for b in budgets]
            self.devs = [DeviceLayer(wl, synth.make_layer(wl, layer=i, device="cuda"),
                                     weights_fp8=self.fp8) for i, wl in enumerate(self.works)]
        else:
            self.works = [w]
            tensors = layer_cpu if layer_cpu is not None else synth.make_layer(w, device="cuda")
            self.devs = [DeviceLayer(w, tensors, weights_fp8=self.fp8)]
        sel = {"score": B.SELECT_SCORE, "top-p": B.SELECT_TOP_P, "relative": B.SELECT_RELATIVE}[args.selector]
        self.selector = sel
        self.Y = torch.empty((w.T, w.d), dtype=self.devs[0].dtype, device="cuda")
        self.set_budgets([wl.budget for wl in self.works])

    def set_budgets(self, budgets):
        B, torch = self.B, self.torch
        self.works = [wl.with_(budget=b) for wl, b in zip(self.works, budgets)]
        self.descs = [dv.desc(budget=b, selector=self.selector) for dv, b in zip(self.devs, budgets)]
        need = max(B.allocmoe_workspace_bytes(dc) for dc in self.descs)
        if getattr(self, "ws", None) is None or self.ws.numel() < need:
            self.ws = torch.empty(need, dtype=torch.uint8, device="cuda")

    def step(self):
        for dv, dc in zip(self.devs, self.descs):
            self.B.allocmoe_moe_forward(dc, dv.X, dv.weights, self.Y, self.ws)

    def time_steps(self, steps, warmup):
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t0) / steps

    def time_stages(self, steps):
        """The same steps through the event-instrumented entry point (same launch structure;
        HIP events recorded by the library on the streams the kernels run on).  Returns the
        per-step sums over the layers of every interval, the number of active experts and
        of selected pairs summed over the layers."""
        B, torch = self.B, self.torch
        sums = [0.0] * len(B.STAGES)
        n_active, pairs = 0, 0
        for it in range(steps):
            for dv, dc, wl in zip(self.devs, self.descs, self.works):
                ms = B.allocmoe_moe_forward_timed(dc, dv.X, dv.weights, self.Y, self.ws)
                sums = [a + b for a, b in zip(sums, ms)]
                if it == 0:
                    L = B.allocmoe_workspace_layout(dc)
                    offs = B.ws_view(self.ws, L.expert_offsets, (wl.E + 1,), torch.int32).cpu()
                    n_active += int(((offs[1:] - offs[:-1]) > 0).sum())
                    assert int(offs[-1]) == wl.budget, "selected pairs != layer budget"
                    pairs += int(offs[-1])
        return dict(zip(B.STAGES, [v / steps for v in sums])), n_active, pairs

    def analyse(self, ms_per_step, stages, n_active, pairs, measured):
        """Roofline of the dominant kernel and whole-step context."""
        w, nL = self.w, len(self.devs)
        d, I, Is, T = w.d, w.I, w.I_shared, w.T
        wb = 1 if self.fp8 else 2
        fp8 = self.fp8
        tiled_routed = pairs >= 8 * w.E * nL and d % 256 == 0 and I % 128 == 0
        tiled_shared = Is > 0 and T >= 128
        targs = "<true, true>" if fp8 else "<true, false>"
        if not tiled_routed and not tiled_shared:
            # decode shapes: one launch per half holds the routed rows and the shared expert;
            # the dominant kernel is the first half (W1, W3: two thirds of the weight bytes)
            nbytes = (n_active * 2 * d * I * wb + pairs * (d * 2 + I * 2)
                      + nL * (2 * d * Is * wb + T * (d * 2 + Is * 2) if Is else 0))
            if fp8:
                nbytes += n_active * 2 * I * 4 + (nL * 2 * Is * 4 if Is else 0)
            ms = stages["ffn1"]
            roof = {"bound": "hbm", "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "kernel": "ffn_bf16_stream_kernel" + targs,
                    "kernel_ms": ms / nL, "launches_per_step": nL,
                    "algorithmic_bytes": nbytes / nL,
                    "traffic": None if fp8 else traffic_from_profiles(self.name, "ffn1")}
            if measured:
                roof["measured_peak"] = measured["hbm_read"]["non_temporal"]["gbs"]
        else:
            # prefill shapes: the tile kernel runs the routed rows on the caller's stream and
            # the shared expert on the library's stream beside them (two launches each).  The
            # figure is the summed work of those launches over the wall-clock region in which
            # they run: from the start of the plan stage (the shared expert's first GEMM starts
            # there) to the start of the combine.
            flops = pairs * 6 * d * I + nL * T * 6 * d * Is
            nbytes = (n_active * 3 * d * I * wb + pairs * (d * 2 + 2 * I * 2 + d * 2)
                      + nL * (3 * d * Is * wb + T * (d * 2 + 2 * Is * 2 + d * 2) if Is else 0))
            ms = stages["expert_span"]
            attainable = min(MFMA_BF16_PEAK_TFLOPS, flops / nbytes * HBM_PEAK_GBS / 1e3)
            launches = (2 if pairs else 0) + (2 if Is else 0)
            if attainable < MFMA_BF16_PEAK_TFLOPS * 0.6:
                # weight-bound: below the ridge the HBM side of the roofline is the binding one
                roof = {"bound": "hbm", "achieved": nbytes / (ms * 1e-3) / 1e9,
                        "peak": HBM_PEAK_GBS, "unit": "GB/s"}
                if measured:
                    roof["measured_peak"] = measured["hbm_read"]["non_temporal"]["gbs"]
                roof["mfma_tflops"] = flops / (ms * 1e-3) / 1e12
            else:
                roof = {"bound": "mfma", "achieved": flops / (ms * 1e-3) / 1e12,
                        "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "attainable": attainable}
                if measured:
                    roof["measured_peak"] = measured["mfma_bf16"]["normal_1_waves_per_simd"]["tflops"]
            roof.update({
                "kernel": "ffn_bf16_t256_kernel" + targs + " and " + targs.replace("true,", "false,", 1)
                          + f": the {launches} launches of a layer (selected rows on the caller's "
                          "stream, shared expert on the library's stream), timed as one region "
                          "from the start of the plan stage to the start of the combine",
                "kernel_ms": ms / nL, "launches_per_step": nL * launches,
                "algorithmic_flops": flops / nL, "algorithmic_bytes": nbytes / nL,
                "per_launch_ms": {k: round(stages[k] / nL, 5)
                                  for k in ("ffn1", "ffn2", "shared_ffn1", "shared_ffn2")},
                "traffic": None if fp8 else traffic_from_profiles(self.name, "expert_span")})
        roof["frac"] = roof["achieved"] / roof["peak"]
        if "measured_peak" in roof:
            roof["frac_of_measured_peak"] = roof["achieved"] / roof["measured_peak"]

        step_bytes = (n_active * 3 * d * I * wb + nL * 3 * d * Is * wb
                      + nL * (T * d * 2 * 2 + d * w.E * 2)
                      + pairs * (d * 2 + 2 * I * 2 + 2 * d * 2)
                      + (nL * T * (d * 2 + 2 * Is * 2 + 2 * d * 2) if Is else 0))
        step_flops = pairs * 6 * d * I + nL * (T * 6 * d * Is + T * 2 * d * w.E)
        step_info = {
            "algorithmic_bytes": step_bytes, "algorithmic_flops": step_flops,
            "hbm_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "mfma_frac": step_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "active_experts": n_active, "layers": nL,
            "stage_ms": {k: round(v, 5) for k, v in stages.items()},
        }
        return roof, step_info


def sub_record(name, args, measured, layer_cpu=None):
    """ms/step at half and at full budget, the dominant kernel and its roofline fraction."""
    import torch
    b = Bench(name, 0.5, args, layer_cpu=layer_cpu)
    steps = 100 if name == "decode" else 40
    ms_half = b.time_steps(steps, 10)
    stages, n_active, pairs = b.time_stages(steps)
    roof, _ = b.analyse(ms_half, stages, n_active, pairs, measured)
    b.set_budgets([b.w.T * b.w.K])
    ms_full = b.time_steps(steps, 10)
    rec = {
        "workload": b.w.name, "T": b.w.T, "budget_half": b.w.budget,
        "ms_per_step_half_budget": round(ms_half, 5), "ms_per_step_full_budget": round(ms_full, 5),
        "tokens_per_s_half_budget": b.w.T / (ms_half * 1e-3),
        "speedup_half_vs_full": round(ms_full / ms_half, 4),
        "dominant_kernel": roof["kernel"].split(":")[0], "bound": roof["bound"],
        "achieved": round(roof["achieved"], 1), "unit": roof["unit"], "frac": round(roof["frac"], 4),
        "stage_ms": {k: round(v, 5) for k, v in stages.items()},
    }
    if "frac_of_measured_peak" in roof:
        rec["frac_of_measured_peak"] = round(roof["frac_of_measured_peak"], 4)
    del b
    torch.cuda.empty_cache()
    return rec


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives are part "
              "of it); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2604_08133_amd import binding as B
    from paper_2604_08133_amd import synth

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
    if args.ceilings:
        print(json.dumps({"ceilings": measure_ceilings()}))
        return

    full_record = (args.workload == "stack" and not args.no_sub_workloads and args.tokens <= 0
                   and args.weights == "bf16" and args.selector == "score"
                   and args.budgets == "dirichlet" and abs(args.budget_ratio - 0.5) < 1e-9)
    measured = measure_ceilings(with_vendor_gemm=False)

    # decode inputs are generated on the CPU: the oracle baseline runs on the same bytes
    decode_w = workload_for("decode", 0.5)
    decode_cpu = synth.make_layer(decode_w, device="cpu") if (
        full_record or args.workload == "decode") and args.tokens <= 0 else None

    workloads = {}
    if full_record:
        for name in ("decode", "prefill", "qwen", "olmoe"):
            workloads[name] = sub_record(name, args, measured,
                                         layer_cpu=decode_cpu if name == "decode" else None)

    bench = Bench(args.workload, args.budget_ratio, args, tokens=args.tokens, layers=args.layers,
                  layer_cpu=decode_cpu if args.workload == "decode" else None)
    ms_per_step = bench.time_steps(args.steps, args.warmup)
    stages, n_active, pairs = bench.time_stages(args.steps)
    roof, step_info = bench.analyse(ms_per_step, stages, n_active, pairs, measured)
    w, nL = bench.w, len(bench.devs)
    budgets = [wl.budget for wl in bench.works]

    out = {
        "metric": METRIC,
        "value": w.T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name + (f"_x{nL}_layers" if nL > 1 else ""), "T": w.T, "d": w.d,
                   "E": w.E, "I": w.I, "K": w.K, "K_base": w.K_base,
                   "budget": budgets if nL > 1 else w.budget,
                   "budget_ratio": args.budget_ratio, "I_shared": w.I_shared, "selector": args.selector,
                   "weights": ("bf16" if not bench.fp8 else "e4m3 codes + fp32 column scales (bf16 "
                               "matrix cores after widening in registers)")
                   + ", re-tiled once by allocmoe_pack_weights, outside the timed region"},
        "roofline": roof,
        "step": step_info,
        "measured_ceilings": measured,
    }
    if nL > 1:
        out["layer_tokens_per_s"] = w.T * nL / (ms_per_step * 1e-3)
    if full_record:
        # the same stack with every layer at the full budget T*K (the original Top-K routing):
        # the layer-level counterpart of the paper's whole-model speed-up figures
        bench.set_budgets([w.T * w.K] * nL)
        ms_full = bench.time_steps(max(5, args.steps // 2), 2)
        out["ms_per_step_full_budget"] = ms_full
        out["speedup_half_vs_full"] = ms_full / ms_per_step
        out["workloads"] = workloads
    del bench
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        if args.workload == "decode" and decode_cpu is not None:
            cb = cpu_baseline(w, decode_cpu, args.cpu_seconds)
        else:
            # bounded sample for the big workloads: the same layer shapes (one layer) at T = 1024
            # tokens, of which as many get their outputs computed as fit the time bound
            Ts = min(w.T, 1024)
            ws_small = w.with_(T=Ts, budget=int(round(args.budget_ratio * Ts * w.K)))
            cb = cpu_baseline(ws_small, synth.make_layer(ws_small, device="cpu"), args.cpu_seconds)
            cb["sample"] = f"one layer of the same shapes at T={Ts} tokens: " + cb["sample"]
            if nL > 1:
                # a step of the stack is nL such layers: per-layer tokens/s divided by nL
                cb["value_per_layer"] = cb["value"]
                cb["value"] = cb["value"] / nL
                cb["sample"] += f"; a step is {nL} layers: value = per-layer tokens/s / {nL}"
        out["cpu_baseline"] = cb
    print(json.dumps(out))


if __name__ == "__main__":
    main()
