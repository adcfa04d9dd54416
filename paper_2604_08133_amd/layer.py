"""Device-side holder of one MoE layer's tensors for tests and the benchmark.

Only plumbing: moves the seeded tensors to the GPU, packs the bf16 expert
weights once, owns the workspace, and calls the C entry points.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B
from .synth import Workload


class DeviceLayer:
    def __init__(self, w: Workload, tensors: dict, device: str = "cuda:0",
                 keep_canonical: bool = False, weights_fp8: bool = False):
        self.w = w
        self.weights_fp8 = weights_fp8   # expert weights packed as E4M3 codes + column scales
        self.device = torch.device(device)
        self.dtype = torch.float32 if w.dtype == "f32" else torch.bfloat16
        t = {k: (v.to(self.device) if v is not None else None) for k, v in tensors.items()}
        self.X = t["X"]
        self.Wg, self.bias, self.w_sg = t["Wg"], t.get("bias"), t.get("w_sg")
        self.packed: Optional[torch.Tensor] = None
        canonical = B.make_weights(Wg=self.Wg, gate_bias=self.bias, W1=t["W1"], W3=t["W3"],
                                   W2=t["W2"], Ws1=t.get("Ws1"), Ws3=t.get("Ws3"),
                                   Ws2=t.get("Ws2"), w_sg=self.w_sg)
        self._canon_tensors = t          # keeps the device tensors alive
        if w.dtype == "bf16":
            desc = self.desc()
            self.packed = torch.empty(B.allocmoe_packed_bytes(desc), dtype=torch.uint8,
                                      device=self.device)
            B.allocmoe_pack_weights(desc, canonical, self.packed)
            torch.cuda.synchronize(self.device)
            if not keep_canonical:
                for k in ("W1", "W3", "W2", "Ws1", "Ws3", "Ws2"):
                    t[k] = None
                canonical = B.make_weights(Wg=self.Wg, gate_bias=self.bias, w_sg=self.w_sg)
            canonical.packed = self.packed.data_ptr()
        self.weights = canonical
        self._ws: Optional[torch.Tensor] = None
        self._ws_budget = None

    def desc(self, budget: Optional[int] = None, K_base: Optional[int] = None,
             selector: int = B.SELECT_SCORE) -> B.LayerDesc:
        w = self.w
        return B.make_desc(w.T, w.d, w.E, w.I, w.K, w.K_base if K_base is None else K_base,
                           w.budget if budget is None else budget, w.dtype, w.I_shared,
                           w.shared_gate, selector=selector, weights_fp8=self.weights_fp8)

    def workspace(self, desc: B.LayerDesc) -> torch.Tensor:
        need = B.allocmoe_workspace_bytes(desc)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def forward(self, budget: Optional[int] = None, K_base: Optional[int] = None,
                Y: Optional[torch.Tensor] = None, X: Optional[torch.Tensor] = None):
        desc = self.desc(budget, K_base)
        ws = self.workspace(desc)
        X = self.X if X is None else X
        if Y is None:
            Y = torch.empty((self.w.T, self.w.d), dtype=self.dtype, device=self.device)
        B.allocmoe_moe_forward(desc, X, self.weights, Y, ws)
        return Y

    def intermediates(self, budget: Optional[int] = None, K_base: Optional[int] = None) -> dict:
        """Views of what the last forward with this descriptor left in the workspace."""
        desc = self.desc(budget, K_base)
        L = B.allocmoe_workspace_layout(desc)
        ws = self.workspace(desc)
        w, Bn = self.w, int(desc.budget)
        i32, f32 = torch.int32, torch.float32
        out = dict(
            scores=B.ws_view(ws, L.scores, (w.T, w.E), f32),
            topk_ids=B.ws_view(ws, L.topk_ids, (w.T, w.K), i32),
            topk_s=B.ws_view(ws, L.topk_s, (w.T, w.K), f32),
            keep_count=B.ws_view(ws, L.keep_count, (w.T,), i32),
            expert_offsets=B.ws_view(ws, L.expert_offsets, (w.E + 1,), i32),
            row_token=B.ws_view(ws, L.row_token, (Bn,), i32),
            row_rank=B.ws_view(ws, L.row_rank, (Bn,), i32),
            inv_row=B.ws_view(ws, L.inv_row, (w.T, w.K), i32),
            H=B.ws_view(ws, L.H, (Bn, w.I), self.dtype),
            O=B.ws_view(ws, L.O, (Bn, w.d), self.dtype),
        )
        if w.shared_gate:
            out["shared_gate"] = B.ws_view(ws, L.shared_gate, (w.T,), f32)
        return out
