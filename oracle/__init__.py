"""ctypes binding of the CPU oracle (oracle/allocmoe_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests/, the smoke check and the
benchmark's cpu_baseline leg may import this package.  It imports nothing from
the HIP package and the HIP package imports nothing from here.

All functions take and return CPU torch tensors; bf16 tensors are handed to the
C code as raw 16-bit patterns and widened there.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "allocmoe_oracle.c")
_LIB = os.path.join(_HERE, "liballocmoe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, single-threaded)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-shared",
                               "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_alloc_t.restype = ctypes.c_int
        _lib.oracle_dispatch.restype = ctypes.c_int64
    return _lib


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return 0
    if t.dtype == torch.bfloat16:
        return 1
    raise TypeError(f"oracle supports fp32 and bf16 inputs, got {t.dtype}")


def _p(t: Optional[torch.Tensor]):
    if t is None:
        return ctypes.c_void_p(0)
    assert t.device.type == "cpu" and t.is_contiguous()
    return ctypes.c_void_p(t.data_ptr())


def gate_logits(X, Wg, bias=None) -> torch.Tensor:
    T, d = X.shape
    E = Wg.shape[1]
    assert Wg.shape[0] == d and _dt(X) == _dt(Wg)
    out = torch.empty((T, E), dtype=torch.float64)
    if bias is not None:
        assert bias.dtype == torch.float32 and bias.numel() == E
    _load().oracle_gate_logits(_p(X), _p(Wg), _p(bias), T, d, E, _dt(X), _p(out))
    return out


def softmax(logits: torch.Tensor) -> torch.Tensor:
    assert logits.dtype == torch.float64
    T, E = logits.shape
    out = torch.empty((T, E), dtype=torch.float32)
    _load().oracle_softmax(_p(logits), T, E, _p(out))
    return out


def shared_gate(X, w_sg) -> torch.Tensor:
    T, d = X.shape
    out = torch.empty((T,), dtype=torch.float64)
    _load().oracle_shared_gate(_p(X), _p(w_sg), T, d, _dt(X), _p(out))
    return out


def topk(scores: torch.Tensor, K: int):
    assert scores.dtype == torch.float32
    T, E = scores.shape
    assert 0 < K <= E
    ids = torch.empty((T, K), dtype=torch.int32)
    s = torch.empty((T, K), dtype=torch.float32)
    _load().oracle_topk(_p(scores), T, E, K, _p(ids), _p(s))
    return ids, s


def alloc_t(topk_s: torch.Tensor, K_base: int, budget: int):
    """Returns (kept[T,K] uint8, keep_count[T] int32); raises on infeasible budget."""
    assert topk_s.dtype == torch.float32
    T, K = topk_s.shape
    kept = torch.empty((T, K), dtype=torch.uint8)
    cnt = torch.empty((T,), dtype=torch.int32)
    rc = _load().oracle_alloc_t(_p(topk_s), T, K, K_base, ctypes.c_int64(budget),
                                _p(kept), _p(cnt))
    if rc != 0:
        raise ValueError("infeasible budget")
    return kept, cnt


def dispatch(topk_ids: torch.Tensor, kept: torch.Tensor, E: int):
    T, K = topk_ids.shape
    n = int(kept.sum())
    offs = torch.empty((E + 1,), dtype=torch.int32)
    row_token = torch.empty((n,), dtype=torch.int32)
    row_rank = torch.empty((n,), dtype=torch.int32)
    inv_row = torch.empty((T, K), dtype=torch.int32)
    r = _load().oracle_dispatch(_p(topk_ids), _p(kept), T, K, E, _p(offs), _p(row_token),
                                _p(row_rank), _p(inv_row))
    assert r == n
    return offs, row_token, row_rank, inv_row


def expert_ffn(x, W1, W3, W2) -> torch.Tensor:
    d, I = W1.shape
    out = torch.empty((d,), dtype=torch.float64)
    _load().oracle_expert_ffn(_p(x), _p(W1), _p(W3), _p(W2), d, I, _dt(W1), _p(out))
    return out


def moe_eq2(layer: dict, topk_ids, topk_s, kept, sgate=None, dense: bool = False,
            tokens: Optional[Sequence[int]] = None) -> torch.Tensor:
    """Eq. (2) output rows for `tokens` (default: all), fp64 [len(tokens), d]."""
    X, W1, W3, W2 = layer["X"], layer["W1"], layer["W3"], layer["W2"]
    T, d = X.shape
    E, _, I = W1.shape
    K = topk_ids.shape[1]
    Ws1, Ws3, Ws2 = layer.get("Ws1"), layer.get("Ws3"), layer.get("Ws2")
    I_sh = 0 if Ws1 is None else Ws1.shape[1]
    tok = torch.arange(T, dtype=torch.int32) if tokens is None else \
        torch.tensor(list(tokens), dtype=torch.int32)
    Y = torch.empty((tok.numel(), d), dtype=torch.float64)
    _load().oracle_moe_eq2(_p(X), _p(W1), _p(W3), _p(W2), _p(Ws1), _p(Ws3), _p(Ws2),
                           _p(sgate), _p(topk_ids), _p(topk_s), _p(kept), T, d, E, I, K,
                           I_sh, _dt(X), 1 if dense else 0, _p(tok), tok.numel(), _p(Y))
    return Y


def moe_dispatched(layer: dict, topk_s, expert_offsets, row_token, inv_row,
                   sgate=None) -> torch.Tensor:
    X, W1, W3, W2 = layer["X"], layer["W1"], layer["W3"], layer["W2"]
    T, d = X.shape
    E, _, I = W1.shape
    K = topk_s.shape[1]
    Ws1, Ws3, Ws2 = layer.get("Ws1"), layer.get("Ws3"), layer.get("Ws2")
    I_sh = 0 if Ws1 is None else Ws1.shape[1]
    Y = torch.empty((T, d), dtype=torch.float64)
    _load().oracle_moe_dispatched(_p(X), _p(W1), _p(W3), _p(W2), _p(Ws1), _p(Ws3), _p(Ws2),
                                  _p(sgate), _p(topk_s), _p(expert_offsets), _p(row_token),
                                  _p(inv_row), T, d, E, I, K, I_sh, _dt(X), _p(Y))
    return Y


def route(layer: dict, K: int):
    """Eq. (1) then the candidate set: (scores fp32 [T,E], ids, s, sgate or None)."""
    scores = softmax(gate_logits(layer["X"], layer["Wg"], layer.get("bias")))
    ids, s = topk(scores, K)
    sg = None
    if layer.get("w_sg") is not None:
        sg = shared_gate(layer["X"], layer["w_sg"])
    return scores, ids, s, sg


def forward(layer: dict, K: int, K_base: int, budget: int, scores=None,
            tokens: Optional[Sequence[int]] = None, selector: int = 0) -> dict:
    """Whole layer by the paper's definitions.  If `scores` is given the
    selection starts from it (the split point for bit-exact index parity).
    selector: 0 = Alloc-T, otherwise a calibrated baseline of oracle/selectors.py."""
    sg = shared_gate(layer["X"], layer["w_sg"]) if layer.get("w_sg") is not None else None
    if scores is None:
        scores = softmax(gate_logits(layer["X"], layer["Wg"], layer.get("bias")))
    ids, s = topk(scores, K)
    if selector == 0:
        kept, cnt = alloc_t(s, K_base, budget)
    else:
        from . import selectors
        kept, cnt = selectors.select(s, selector, K_base, budget)
    offs, row_token, row_rank, inv_row = dispatch(ids, kept, layer["W1"].shape[0])
    Y = moe_eq2(layer, ids, s, kept, sg, dense=False, tokens=tokens)
    return dict(scores=scores, topk_ids=ids, topk_s=s, kept=kept, keep_count=cnt,
                expert_offsets=offs, row_token=row_token, row_rank=row_rank,
                inv_row=inv_row, sgate=sg, Y=Y)
