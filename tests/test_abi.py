"""CPU-side checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments on the host before launching
anything (no GPU is touched by these calls)."""
import ctypes
import os
import re

import pytest

from paper_2604_08133_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "allocmoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(allocmoe_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    syms = declared_symbols()
    assert len(syms) >= 9
    for s in syms:
        assert hasattr(lib, s), s
    assert sorted(B.EXPORTS) == syms


def test_status_strings():
    for code in (B.OK, B.EINVAL, B.EBUDGET, B.ESHAPE, B.EWORKSPACE, B.EHIP):
        assert B.status_string(code)


def good(**kw):
    base = dict(T=64, d=128, E=8, I=256, K=2, K_base=1, budget=64, dtype="f32")
    base.update(kw)
    return B.make_desc(**base)


@pytest.mark.parametrize("kw,status", [
    (dict(budget=63), B.EBUDGET),             # below T*K_base: Eq. (9) infeasible
    (dict(budget=129), B.EBUDGET),            # above the T*K candidates
    (dict(K_base=3), B.EINVAL),               # K_base > K
    (dict(K=9, budget=64), B.EINVAL),         # K > E
    (dict(E=65, budget=64), B.ESHAPE),        # more experts than lanes
    (dict(T=0), B.EINVAL),
    (dict(dtype=7), B.EINVAL),
    (dict(dtype="bf16", d=100), B.ESHAPE),    # bf16 path needs multiples of 64
    (dict(shared_gate=True), B.EINVAL),       # gate without a shared expert
])
def test_descriptor_validation(kw, status):
    n = ctypes.c_size_t(0)
    rc = B.load().allocmoe_workspace_bytes(ctypes.byref(good(**kw)), ctypes.byref(n))
    assert rc == status


def test_workspace_layout_is_ordered_and_aligned():
    L = B.allocmoe_workspace_layout(good(I_shared=64))
    offs = [L.scratch, L.scores, L.topk_ids, L.topk_s, L.keep_count, L.shared_gate,
            L.expert_offsets, L.row_token, L.row_rank, L.inv_row, L.H, L.Hs, L.O, L.Os, L.total]
    assert offs[0] == 0 and offs == sorted(offs)
    assert all(o % 256 == 0 for o in offs)
    assert L.total == B.allocmoe_workspace_bytes(good(I_shared=64))


def test_null_and_workspace_errors_without_launch():
    lib = B.load()
    desc = good()
    w = B.make_weights()
    # null X / weights
    assert lib.allocmoe_moe_forward(ctypes.byref(desc), None, ctypes.byref(w), None, None,
                                    ctypes.c_size_t(0), None) == B.EINVAL
    assert lib.allocmoe_route_from_scores(ctypes.byref(desc), None, None, None, None, None,
                                          ctypes.c_size_t(0), None) == B.EINVAL
    # dispatch with a missing workspace
    fake = ctypes.c_void_p(256)
    assert lib.allocmoe_dispatch(ctypes.byref(desc), fake, fake, fake, fake, fake, fake, None,
                                 ctypes.c_size_t(0), None) == B.EWORKSPACE
    # packing is bf16-only
    n = ctypes.c_size_t(0)
    assert lib.allocmoe_packed_bytes(ctypes.byref(desc), ctypes.byref(n)) == B.EINVAL
    assert B.allocmoe_packed_bytes(good(dtype="bf16", d=128, I=256)) == \
        256 * (((8 * 3 * 128 * 256 + 5 * 16 * 128) * 2 + 255) // 256)


def test_bench_refuses_more_than_one_gpu():
    # the build is for one GPU: bench.py --gpus N > 1 exits with a message, before any GPU work
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "--gpus 1" in r.stderr
