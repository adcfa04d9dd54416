"""Thin ctypes binding of liballocmoe.so (see include/allocmoe.h).

Argument marshalling only: every step of the layer runs in the library's HIP
kernels.  PyTorch supplies device memory (`tensor.data_ptr()`) and the stream.
There is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liballocmoe.so")

OK, EINVAL, EBUDGET, ESHAPE, EWORKSPACE, EHIP = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1

EXPORTS = [
    "allocmoe_workspace_bytes", "allocmoe_workspace_layout", "allocmoe_packed_bytes",
    "allocmoe_pack_weights", "allocmoe_route", "allocmoe_route_from_scores",
    "allocmoe_dispatch", "allocmoe_dispatch_static", "allocmoe_moe_forward", "allocmoe_moe_forward_timed",
    "allocmoe_alloc_l", "allocmoe_layer_schedule", "allocmoe_routing_stats",
    "allocmoe_probe_mfma_operand_bytes", "allocmoe_probe_sink_bytes", "allocmoe_probe_mfma",
    "allocmoe_probe_hbm_read",
    "allocmoe_status_string",
]
# intervals of allocmoe_moe_forward_timed (include/allocmoe.h, allocmoe_stage)
STAGES = ["route", "plan", "ffn1", "ffn2", "combine", "shared_ffn1", "shared_ffn2", "expert_span",
          "total"]
_SIZE_T_EXPORTS = ("allocmoe_probe_mfma_operand_bytes", "allocmoe_probe_sink_bytes")


class LayerDesc(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("d", ctypes.c_int32), ("E", ctypes.c_int32),
                ("I", ctypes.c_int32), ("K", ctypes.c_int32), ("K_base", ctypes.c_int32),
                ("budget", ctypes.c_int64), ("I_shared", ctypes.c_int32),
                ("shared_gate", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("flags", ctypes.c_int32)]


class Weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("Wg", "gate_bias", "W1", "W3", "W2", "Ws1", "Ws3", "Ws2", "w_sg", "packed")]


class WsLayout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in
                ("scores", "topk_ids", "topk_s", "keep_count", "shared_gate", "expert_offsets",
                 "row_token", "row_rank", "inv_row", "H", "Hs", "O", "Os", "scratch", "sel_keys",
                 "total")]


class AllocMoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def load() -> ctypes.CDLL:
    """Load the HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2604_08133_amd.build); "
                "there is no CPU fallback")
        lib = ctypes.CDLL(LIB_PATH)
        lib.allocmoe_status_string.restype = ctypes.c_char_p
        lib.allocmoe_status_string.argtypes = [ctypes.c_int]
        for name in EXPORTS:
            if name in _SIZE_T_EXPORTS:
                getattr(lib, name).restype = ctypes.c_size_t
            elif name != "allocmoe_status_string":
                getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().allocmoe_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != OK:
        raise AllocMoEError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_contiguous():
        raise ValueError("tensors passed to allocmoe must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


SELECT_SCORE, SELECT_TOP_P, SELECT_RELATIVE = 0, 1, 2


WEIGHTS_FP8 = 0x100


def make_desc(T, d, E, I, K, K_base, budget, dtype, I_shared=0, shared_gate=False,
              selector=SELECT_SCORE, weights_fp8=False) -> LayerDesc:
    code = {"f32": F32, "bf16": BF16, torch.float32: F32, torch.bfloat16: BF16}.get(dtype, dtype)
    return LayerDesc(T, d, E, I, K, K_base, budget, I_shared, 1 if shared_gate else 0, code,
                     int(selector) | (WEIGHTS_FP8 if weights_fp8 else 0))


def make_weights(Wg=None, gate_bias=None, W1=None, W3=None, W2=None, Ws1=None, Ws3=None,
                 Ws2=None, w_sg=None, packed=None) -> Weights:
    w = Weights()
    for name, t in (("Wg", Wg), ("gate_bias", gate_bias), ("W1", W1), ("W3", W3), ("W2", W2),
                    ("Ws1", Ws1), ("Ws3", Ws3), ("Ws2", Ws2), ("w_sg", w_sg), ("packed", packed)):
        setattr(w, name, _ptr(t).value)
    return w


# --------------------------------------------------------- the C entry points

def allocmoe_workspace_bytes(desc: LayerDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(load().allocmoe_workspace_bytes(ctypes.byref(desc), ctypes.byref(n)),
           "allocmoe_workspace_bytes")
    return n.value


def allocmoe_workspace_layout(desc: LayerDesc) -> WsLayout:
    L = WsLayout()
    _check(load().allocmoe_workspace_layout(ctypes.byref(desc), ctypes.byref(L)),
           "allocmoe_workspace_layout")
    return L


def allocmoe_packed_bytes(desc: LayerDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(load().allocmoe_packed_bytes(ctypes.byref(desc), ctypes.byref(n)),
           "allocmoe_packed_bytes")
    return n.value


def allocmoe_pack_weights(desc: LayerDesc, canonical: Weights, packed: torch.Tensor,
                          stream=None) -> None:
    _check(load().allocmoe_pack_weights(ctypes.byref(desc), ctypes.byref(canonical), _ptr(packed),
                                        ctypes.c_size_t(packed.numel() * packed.element_size()),
                                        _stream(stream)), "allocmoe_pack_weights")


def allocmoe_route(desc: LayerDesc, X, w: Weights, scores, topk_ids, topk_s, keep_count,
                   ws: Optional[torch.Tensor] = None, stream=None) -> None:
    nbytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(load().allocmoe_route(ctypes.byref(desc), _ptr(X), ctypes.byref(w), _ptr(scores),
                                 _ptr(topk_ids), _ptr(topk_s), _ptr(keep_count), _ptr(ws),
                                 ctypes.c_size_t(nbytes), _stream(stream)), "allocmoe_route")


def allocmoe_route_from_scores(desc: LayerDesc, scores, topk_ids, topk_s, keep_count,
                               ws: Optional[torch.Tensor] = None, stream=None) -> None:
    nbytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(load().allocmoe_route_from_scores(ctypes.byref(desc), _ptr(scores), _ptr(topk_ids),
                                             _ptr(topk_s), _ptr(keep_count), _ptr(ws),
                                             ctypes.c_size_t(nbytes), _stream(stream)),
           "allocmoe_route_from_scores")


def allocmoe_dispatch(desc: LayerDesc, topk_ids, keep_count, expert_offsets, row_token, row_rank,
                      inv_row, ws: torch.Tensor, stream=None) -> None:
    _check(load().allocmoe_dispatch(ctypes.byref(desc), _ptr(topk_ids), _ptr(keep_count),
                                    _ptr(expert_offsets), _ptr(row_token), _ptr(row_rank),
                                    _ptr(inv_row), _ptr(ws),
                                    ctypes.c_size_t(ws.numel() * ws.element_size()),
                                    _stream(stream)), "allocmoe_dispatch")


STATIC_MAX_TOKENS = 65536


def allocmoe_dispatch_static(desc: LayerDesc, topk_ids, keep_count, expert_offsets, row_token,
                             row_rank, inv_row, stream=None) -> None:
    """allocmoe_dispatch with the library's own static scratch: no workspace argument."""
    _check(load().allocmoe_dispatch_static(ctypes.byref(desc), _ptr(topk_ids), _ptr(keep_count),
                                           _ptr(expert_offsets), _ptr(row_token), _ptr(row_rank),
                                           _ptr(inv_row), _stream(stream)),
           "allocmoe_dispatch_static")


def allocmoe_moe_forward(desc: LayerDesc, X, w: Weights, Y, ws: torch.Tensor, stream=None) -> None:
    _check(load().allocmoe_moe_forward(ctypes.byref(desc), _ptr(X), ctypes.byref(w), _ptr(Y),
                                       _ptr(ws), ctypes.c_size_t(ws.numel() * ws.element_size()),
                                       _stream(stream)), "allocmoe_moe_forward")


def allocmoe_moe_forward_timed(desc: LayerDesc, X, w: Weights, Y, ws: torch.Tensor,
                               stream=None) -> list:
    """Returns the per-stage durations in ms (order: STAGES); synchronises."""
    ms = (ctypes.c_float * len(STAGES))()
    _check(load().allocmoe_moe_forward_timed(ctypes.byref(desc), _ptr(X), ctypes.byref(w),
                                             _ptr(Y), _ptr(ws),
                                             ctypes.c_size_t(ws.numel() * ws.element_size()),
                                             _stream(stream), ms), "allocmoe_moe_forward_timed")
    return list(ms)


def allocmoe_probe_mfma(operands: torch.Tensor, waves_per_simd: int, iters: int,
                        sink: torch.Tensor, stream=None):
    """Returns (TFLOP/s, shader clock in MHz) of the matrix-core issue loop; synchronises."""
    tf, mhz = ctypes.c_float(0), ctypes.c_float(0)
    _check(load().allocmoe_probe_mfma(_ptr(operands),
                                      ctypes.c_size_t(operands.numel() * operands.element_size()),
                                      ctypes.c_int(waves_per_simd), ctypes.c_int(iters), _ptr(sink),
                                      ctypes.c_size_t(sink.numel() * sink.element_size()),
                                      ctypes.byref(tf), ctypes.byref(mhz), _stream(stream)),
           "allocmoe_probe_mfma")
    return tf.value, mhz.value


def allocmoe_probe_hbm_read(buf: torch.Tensor, nontemporal: bool, repeats: int,
                            sink: torch.Tensor, stream=None) -> float:
    """Returns the achieved GB/s of the streaming read; synchronises."""
    gbs = ctypes.c_float(0)
    _check(load().allocmoe_probe_hbm_read(_ptr(buf), ctypes.c_size_t(buf.numel() * buf.element_size()),
                                          ctypes.c_int(1 if nontemporal else 0),
                                          ctypes.c_int(repeats), _ptr(sink),
                                          ctypes.c_size_t(sink.numel() * sink.element_size()),
                                          ctypes.byref(gbs), _stream(stream)),
           "allocmoe_probe_hbm_read")
    return gbs.value


METRICS = ["spearman_load", "entropy_orig", "entropy_kept", "js_divergence", "spearman_tokens"]


def allocmoe_routing_stats(desc: LayerDesc, scores, topk_ids, topk_s, keep_count, stream=None) -> dict:
    """Allocates the outputs (torch, on the inputs' device) and returns them by name;
    'metrics' is a float tensor of len(METRICS)."""
    dev = scores.device
    E, T = int(desc.E), int(desc.T)
    out = dict(load_orig=torch.empty(E, dtype=torch.int32, device=dev),
               load_kept=torch.empty(E, dtype=torch.int32, device=dev),
               wload_orig=torch.empty(E, dtype=torch.float32, device=dev),
               wload_kept=torch.empty(E, dtype=torch.float32, device=dev),
               token_entropy=torch.empty(T, dtype=torch.float32, device=dev),
               metrics=torch.empty(len(METRICS), dtype=torch.float32, device=dev))
    ws = torch.empty(max(256, 4 * T), dtype=torch.uint8, device=dev)
    _check(load().allocmoe_routing_stats(
        ctypes.byref(desc), _ptr(scores), _ptr(topk_ids), _ptr(topk_s), _ptr(keep_count),
        _ptr(out["load_orig"]), _ptr(out["load_kept"]), _ptr(out["wload_orig"]),
        _ptr(out["wload_kept"]), _ptr(out["token_entropy"]), _ptr(out["metrics"]), _ptr(ws),
        ctypes.c_size_t(ws.numel()), _stream(stream)), "allocmoe_routing_stats")
    return out


def allocmoe_alloc_l(S, B: int):
    """S: [L, K_orig] rows of float (any nested sequence or tensor, host).  Returns
    (K, cost): the allocation as a list of L ints and its total sensitivity."""
    rows = [[float(v) for v in row] for row in S]
    L, K_orig = len(rows), len(rows[0])
    flat = (ctypes.c_double * (L * K_orig))(*[v for row in rows for v in row])
    out = (ctypes.c_int32 * L)()
    cost = ctypes.c_double(0.0)
    _check(load().allocmoe_alloc_l(flat, ctypes.c_int32(L), ctypes.c_int32(K_orig),
                                   ctypes.c_int64(int(B)), out, ctypes.byref(cost)),
           "allocmoe_alloc_l")
    return list(out), cost.value


SCHEDULE_ASCENDING, SCHEDULE_DESCENDING = 0, 1


def allocmoe_layer_schedule(kind: int, L: int, K_orig: int, B: int):
    """The Ascending (kind 0) or Descending (kind 1) per-layer allocation: L ints."""
    out = (ctypes.c_int32 * L)()
    _check(load().allocmoe_layer_schedule(ctypes.c_int(kind), ctypes.c_int32(L),
                                          ctypes.c_int32(K_orig), ctypes.c_int64(int(B)), out),
           "allocmoe_layer_schedule")
    return list(out)


# ------------------------------------------------ conveniences for tests/bench

def ws_view(ws: torch.Tensor, offset: int, shape, dtype: torch.dtype) -> torch.Tensor:
    """A typed view of a region of the (uint8) workspace tensor."""
    n = 1
    for s in shape:
        n *= int(s)
    nbytes = n * torch.empty((), dtype=dtype).element_size()
    return ws[offset:offset + nbytes].view(dtype).reshape(tuple(int(s) for s in shape))
