"""GPU parity of the two-level schedule (main workgroups in step on the first part of every
tile's K range, tail workgroups sharing the rest, shared tiles completed through the
workspace by the last contributor) against the CPU fp64 oracle, through the C ABI.  The
schedule needs between 128 and 248 tiles of 256 x 256 and at least 48 K stages, so the
shapes are large; it is forced with the diagnostic override where the cost model would
not pick it."""
import numpy as np
import pytest
import torch

import tess_workloads as wl
import paper_2105_14500_amd as tess
from paper_2105_14500_amd import binding as B
from oracle import tess_oracle as orc
from gpu_util import TOL, f64, dev, run_share, oracle_share, rel_err, share_desc, workspace

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _force_streamk():
    B.set_plan_override(tile=256, k_splits=0, stream_k=1)      # two-level wherever the shape allows it
    yield
    B.set_plan_override(0, 0, -1)


# (q, d, m, kb, n): per call M x N x K is fwd m x n x q*kb, dX m x kb x q*n, dW kb x n x q*m
SHAPES = [
    (1, 1, 3072, 3072, 3136),   # 156 / 144 / 156 tiles, ragged N edge; tails split between two workgroups
    (2, 1, 4096, 1536, 2048),   # fwd 128 tiles (the fewest), 3072 deep; dX and dW below the range: plain plans
    (1, 1, 3584, 3072, 4352),   # fwd 14 x 17 = 238 tiles (two tail workgroups per XCD), dW 12 x 17 = 204
]


def _plans(q, d, m, kb, n):
    desc = share_desc(q, d, m, kb, n, "bf16", "bf16")
    return {op: B.plan(desc, op) for op in (B.OP_FWD, B.OP_BWD_DX, B.OP_BWD_DW)}


@pytest.mark.parametrize("q,d,m,kb,n", SHAPES)
def test_streamk_small_integers_are_bit_exact(q, d, m, kb, n):
    plans = _plans(q, d, m, kb, n)
    assert any(p[2] == 0 for p in plans.values()), plans        # k_splits 0 = stream-K
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=4242, integers=True)
    got = run_share(q, d, inp["x"], inp["w"], inp["bias"], inp["dy"], "bf16", "f32", act="none")
    want = oracle_share(inp["x"], inp["w"], inp["bias"], inp["dy"], act="none")
    for key in ("y", "dx", "dw"):
        assert np.array_equal(f64(got[key]), want[key]), key


@pytest.mark.parametrize("q,d,m,kb,n", SHAPES[:1])
def test_streamk_matches_oracle(q, d, m, kb, n):
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=77 + m, w_std=0.05)
    got = run_share(q, d, inp["x"], inp["w"], inp["bias"], inp["dy"], "bf16", "bf16",
                    act="gelu_erf", want_preact=True)
    want = oracle_share(inp["x"], inp["w"], inp["bias"], inp["dy"], act="gelu_erf")
    for key in ("y", "preact", "dx", "dw"):
        assert rel_err(got[key], want[key]) <= TOL["bf16"], key


def test_streamk_is_deterministic_and_leaves_its_workspace_reusable():
    """Same call twice on one workspace (the second finds the first one's control words),
    then on a workspace full of ones: bit-identical results each time; the depth sum
    (accumulate) and the bias gradient go through the same fix-up."""
    q, d, m, kb, n = 1, 1, 3072, 3072, 3136
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=5, w_std=0.1)
    desc = B.make_desc(q, d, 0, 0, 0, m * q * d, kb * q, n * q, B.BF16, B.BF16)
    xd, wd, dyd, bd = dev(inp["x"]), dev(inp["w"]), dev(inp["dy"]), dev(inp["bias"])
    nbytes = max(tess.workspace_bytes(desc, op) for op in (0, 1, 2))
    assert nbytes > 0
    outs = []
    for fill in (None, None, 1.0, float("nan")):
        ws = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda:0") if not outs else ws
        if fill is not None:
            ws.fill_(fill)
        y = torch.empty((m, n), dtype=torch.bfloat16, device="cuda:0")
        dx = torch.empty((m, kb), dtype=torch.bfloat16, device="cuda:0")
        dw = torch.zeros((kb, n), dtype=torch.float32, device="cuda:0")
        db = torch.zeros((n,), dtype=torch.float32, device="cuda:0")
        tess.linear_fwd(desc, list(xd), list(wd), bd, B.ACT_GELU_ERF, y, workspace=ws)
        tess.linear_bwd_dx(desc, list(dyd), list(wd), dx, workspace=ws)
        for _ in range(2):      # two depth layers into one buffer
            tess.linear_bwd_dw_bias(desc, list(xd), list(dyd), dw, db, accumulate=True, workspace=ws)
        torch.cuda.synchronize()
        outs.append((y.cpu(), dx.cpu(), dw.cpu(), db.cpu()))
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            assert torch.equal(a, b)
    xs, dys = [f64(inp["x"][t]) for t in range(q)], [f64(inp["dy"][t]) for t in range(q)]
    want_dw = 2.0 * orc.bwd_dw_panels(xs, dys)
    want_db = 2.0 * orc.bias_grad_panels(dys)
    assert rel_err(outs[0][2], want_dw) <= 1e-4
    assert rel_err(outs[0][3], want_db) <= 1e-5
    assert all(tess.plan(desc, op)[2] == 0 for op in (0, 1, 2))


def test_streamk_calls_replay_from_a_hip_graph():
    """A replayed graph passes the same token again: the control words must have been put
    back by the call itself.  Replays alternate with eager work and synchronisations."""
    q, d, m, kb, n = 1, 1, 3072, 3072, 3136
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=9, w_std=0.1)
    desc = B.make_desc(q, d, 0, 0, 0, m * q * d, kb * q, n * q, B.BF16, B.BF16)
    xd, wd, dyd = dev(inp["x"]), dev(inp["w"]), dev(inp["dy"])
    ws = workspace(desc, B.OP_FWD)
    ws2 = workspace(desc, B.OP_BWD_DX)
    y = torch.empty((m, n), dtype=torch.bfloat16, device="cuda:0")
    dx = torch.empty((m, kb), dtype=torch.bfloat16, device="cuda:0")
    tess.linear_fwd(desc, list(xd), list(wd), None, B.ACT_NONE, y, workspace=ws)
    tess.linear_bwd_dx(desc, list(dyd), list(wd), dx, workspace=ws2)
    torch.cuda.synchronize()
    y0, dx0 = y.clone(), dx.clone()
    s = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(graph, stream=s):
            tess.linear_fwd(desc, list(xd), list(wd), None, B.ACT_NONE, y, workspace=ws, stream=s)
            tess.linear_bwd_dx(desc, list(dyd), list(wd), dx, workspace=ws2, stream=s)
    for rep in range(4):
        y.zero_(); dx.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y0) and torch.equal(dx, dx0), rep
        (xd[0] @ wd[0]).sum().item()        # eager work between the replays
