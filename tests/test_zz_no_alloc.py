"""allocmoe_dispatch_static (the entry point for callers that cannot allocate: its scratch
is part of the library's device image) against allocmoe_dispatch on the same inputs, and
both against the CPU oracle: bit-exact.  Two calls in a row share the device's scratch
buffer, the second with a smaller input; the sizes take the code path that really uses
the scratch (more tokens than the single-workgroup kernel holds in LDS)."""
import pytest
import torch

import oracle
from paper_2604_08133_amd import binding as B
from paper_2604_08133_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dispatch_both(scores_cpu, K, Kb, budget):
    T, E = scores_cpu.shape
    desc = B.make_desc(T, 64, E, 64, K, Kb, budget, "f32")
    ids_c, vals_c = oracle.topk(scores_cpu, K)
    kept, cnt_c = oracle.alloc_t(vals_c, Kb, budget)
    want = oracle.dispatch(ids_c, kept, E)
    ids, cnt = ids_c.to(DEV), cnt_c.to(DEV)

    def outputs():
        return (torch.full((E + 1,), -7, dtype=torch.int32, device=DEV),
                torch.full((max(budget, 1),), -7, dtype=torch.int32, device=DEV),
                torch.full((max(budget, 1),), -7, dtype=torch.int32, device=DEV),
                torch.full((T, K), -7, dtype=torch.int32, device=DEV))

    a = outputs()
    ws = torch.empty(B.allocmoe_workspace_layout(desc).scores, dtype=torch.uint8, device=DEV)
    B.allocmoe_dispatch(desc, ids, cnt, *a, ws)
    b = outputs()
    B.allocmoe_dispatch_static(desc, ids, cnt, *b)      # no workspace argument
    torch.cuda.synchronize()
    for name, x, y, w in zip(("expert_offsets", "row_token", "row_rank", "inv_row"), a, b, want):
        n = budget if name in ("row_token", "row_rank") else None
        assert torch.equal(x.cpu()[:n], y.cpu()[:n]), (name, "static vs workspace")
        assert torch.equal(y.cpu()[:n], w), (name, "static vs oracle")


def test_static_scratch_dispatch_two_calls_second_smaller():
    for T, E, K, Kb, ratio in ((12000, 64, 6, 1, 0.5), (9000, 60, 4, 1, 0.75), (300, 16, 4, 0, 0.5)):
        print(f"static dispatch T={T} E={E} K={K}", flush=True)
        scores = synth.make_scores(T, E, seed=5 + T)
        dispatch_both(scores, K, Kb, int(ratio * T * K))


def test_static_scratch_rejects_sizes_beyond_its_maximum():
    T = B.STATIC_MAX_TOKENS + 64
    desc = B.make_desc(T, 64, 8, 64, 2, 1, T, "f32")
    t = torch.zeros(8, dtype=torch.int32, device=DEV)
    with pytest.raises(B.AllocMoEError) as e:
        B.allocmoe_dispatch_static(desc, t, t, t, t, t, t)
    assert e.value.status == B.ESHAPE
