"""The entry point for callers that cannot allocate (tess_linear_bwd_dw_noalloc): same
results as tess_linear_bwd_dw, bit for bit, with the library's static device scratch in
place of a caller's workspace.  Two calls in a row, the second on a smaller problem that
finds the first one's partial sums in the scratch; then the depth sum (accumulate), and a
plan that needs more scratch than there is."""
import pytest
import torch

import tess_workloads as wl
import paper_2105_14500_amd as tess
from paper_2105_14500_amd import binding as B

pytestmark = pytest.mark.gpu


def _pair(q, d, m, kb, n, seed, accumulate):
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=seed, w_std=0.1)
    desc = B.make_desc(q, d, 0, 0, 0, m * q * d, kb * q, n * q, B.BF16, B.BF16)
    nbytes = tess.workspace_bytes(desc, B.OP_BWD_DW)
    assert 0 < nbytes <= B.noalloc_scratch_bytes(), "the shape must take the K-split path and fit the scratch"
    xd, dyd = inp["x"].to("cuda:0"), inp["dy"].to("cuda:0")
    odt = torch.float32 if accumulate else torch.bfloat16
    base = torch.randn((kb, n), device="cuda:0").to(odt) if accumulate else None
    outs = []
    for which in ("workspace", "noalloc"):
        dw = base.clone() if accumulate else torch.full((kb, n), float("nan"), dtype=odt, device="cuda:0")
        if which == "workspace":
            ws = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda:0")
            tess.linear_bwd_dw(desc, list(xd), list(dyd), dw, accumulate=accumulate, workspace=ws)
        else:
            B.linear_bwd_dw_noalloc(desc, list(xd), list(dyd), dw, accumulate=accumulate)
        torch.cuda.synchronize()
        outs.append(dw.cpu())
    assert torch.isfinite(outs[0].float()).all()
    assert torch.equal(outs[0], outs[1])


def test_noalloc_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    _pair(2, 2, 2048, 512, 2048, seed=31, accumulate=False)     # 16 MiB of partial sums
    _pair(2, 2, 1024, 256, 512, seed=32, accumulate=False)      # smaller: 2 MiB, over the first call's leftovers
    _pair(4, 2, 4096, 1024, 4096, seed=33, accumulate=True)     # 256 x 256 tiles, 64 MiB, added to a buffer


def test_noalloc_rejects_a_plan_that_does_not_fit():
    q, d, m, kb, n = 8, 2, 2048, 1536, 6144                     # 108 MiB of partial sums
    desc = B.make_desc(q, d, 0, 0, 0, m * q * d, kb * q, n * q, B.BF16, B.BF16)
    assert tess.workspace_bytes(desc, B.OP_BWD_DW) > B.noalloc_scratch_bytes()
    x = [torch.zeros((m, kb), dtype=torch.bfloat16, device="cuda:0") for _ in range(q)]
    dy = [torch.zeros((m, n), dtype=torch.bfloat16, device="cuda:0") for _ in range(q)]
    dw = torch.full((kb, n), 7.0, dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(tess.TessError) as ei:
        B.linear_bwd_dw_noalloc(desc, x, dy, dw)
    assert ei.value.status == 6
    torch.cuda.synchronize()
    assert torch.all(dw == 7.0)
