"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration that bench.py times (packed panels, same workspace, dW accumulated
into fp32).  The oracle cannot produce whole outputs at these sizes in seconds,
so it computes sampled outputs one by one: a set of output rows restricted to a
window of columns, on the same seeded inputs."""
import itertools

import numpy as np
import pytest
import torch

import tess_workloads as wl
import paper_2105_14500_amd as tess
from paper_2105_14500_amd import binding as B, partition as P
from oracle import tess_oracle as orc
from gpu_util import TOL, f64, dev, rel_err, workspace, code, tdtype

pytestmark = pytest.mark.gpu

ACT = {"none": (B.ACT_NONE, orc.ACT_NONE), "gelu_erf": (B.ACT_GELU_ERF, orc.ACT_GELU_ERF)}
CASES = [(w.name, L.name) for w in wl.WORKLOADS if w.mode == "one_share" for L in w.layers]
# block shapes of the paper's own experiment grids (Tables 1 and 2): three strong-scaling
# grids with all four layers, the single-processor grid (q = 1: one panel per operand) and
# one weak-scaling grid
_PAPER = {"strong_q2d2_b12_h3072": ("qkv", "out", "up", "down"),
          "strong_q4d4_b16_h3072": ("qkv", "out", "up", "down"),
          "strong_q8d1_b12_h3072": ("qkv", "out", "up", "down"),
          "weak_q1d1_b48_h1024": ("out", "up"),
          "weak_q4d2_b384_h4096": ("qkv",)}
CASES += [(name, lname) for name, lnames in _PAPER.items() for lname in lnames]


def _sample(n, count, seed):
    r = np.random.default_rng(seed)
    idx = np.unique(np.concatenate([[0, n - 1], r.integers(0, n, size=count)]))
    return idx.astype(np.int64)


@pytest.mark.parametrize("wname,lname", CASES)
def test_one_share_full_size(wname, lname):
    w = wl.workload_by_name(wname)
    L = next(l for l in w.layers if l.name == lname)
    q, m, kb, n = w.q, L.m, L.kb, L.n
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=4321, bias_std=L.bias_std)
    desc = B.make_desc(q, w.d, 0, 0, 0, L.a, L.b, L.c, B.BF16, B.BF16)
    assert tess.block_shape(desc) == (m, kb, n)
    x, wt, bias, dy = (dev(inp[k]) for k in ("x", "w", "bias", "dy"))
    nbytes = max(tess.workspace_bytes(desc, op) for op in (0, 1, 2))
    ws = torch.empty(max(nbytes, 4) // 4, dtype=torch.float32, device="cuda:0")
    y = torch.full((m, n), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    dx = torch.full((m, kb), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    dw = torch.zeros((kb, n), dtype=torch.float32, device="cuda:0")
    gact, oact = ACT[L.act]
    tess.linear_fwd(desc, list(x), list(wt), bias, gact, y, workspace=ws)
    tess.linear_bwd_dx(desc, list(dy), list(wt), dx, workspace=ws)
    tess.linear_bwd_dw(desc, list(x), list(dy), dw, accumulate=True, workspace=ws)
    torch.cuda.synchronize()
    # nothing left unwritten anywhere
    assert not torch.isnan(y).any() and not torch.isnan(dx).any()

    rows = _sample(m, 24, 1)
    c0 = (n // 2 // 8) * 8 - 64 if n >= 512 else 0          # window straddling a tile edge
    cw = min(n - c0, 320)
    # forward: Y[rows, c0:c0+cw]
    xs = [f64(inp["x"][t][rows]) for t in range(q)]
    wcols = [f64(inp["w"][t][:, c0:c0 + cw]) for t in range(q)]
    want = orc.fwd_panels(xs, wcols, bias=f64(inp["bias"][c0:c0 + cw]), act=oact)
    errs = {}
    e = errs["y"] = rel_err(y[rows][:, c0:c0 + cw], want)
    assert e <= TOL["bf16"], ("y", e)
    # dX[rows, u0:u0+uw]
    u0 = (kb // 2 // 8) * 8 - 64 if kb >= 512 else 0
    uw = min(kb - u0, 320)
    dys = [f64(inp["dy"][t][rows]) for t in range(q)]
    wrows = [f64(inp["w"][t][u0:u0 + uw]) for t in range(q)]
    want = orc.bwd_dx_panels(dys, wrows)
    e = errs["dx"] = rel_err(dx[rows][:, u0:u0 + uw], want)
    assert e <= TOL["bf16"], ("dx", e)
    # dW[urows, c0:c0+cw2]
    urows = _sample(kb, 12, 2)
    cw2 = min(n - c0, 160)
    xcols = [np.ascontiguousarray(f64(inp["x"][t][:, urows])) for t in range(q)]
    dyw = [f64(inp["dy"][t][:, c0:c0 + cw2]) for t in range(q)]
    want = orc.bwd_dw_panels(xcols, dyw)
    e = errs["dw"] = rel_err(dw[urows][:, c0:c0 + cw2], want)
    assert e <= 1e-3, ("dw", e)            # fp32 output: accumulation order only

    # the backward epilogues next to the path, same buffers and workspace:
    # weight gradient with the bias gradient from the dY panels it streams
    dw2 = torch.zeros((kb, n), dtype=torch.float32, device="cuda:0")
    db = torch.zeros((n,), dtype=torch.float32, device="cuda:0")
    tess.linear_bwd_dw_bias(desc, list(x), list(dy), dw2, db, accumulate=True, workspace=ws)
    # input gradient through a GELU whose pre-activation is a seeded N(0, 1.5^2) block
    g = torch.Generator().manual_seed(99)
    z = (torch.randn((m, kb), generator=g) * 1.5).to(torch.bfloat16)
    dz = torch.full((m, kb), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    tess.linear_bwd_dx_act(desc, list(dy), list(wt), dev(z), B.ACT_GELU_ERF, dz, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(dw2, dw)
    want = orc.bias_grad_panels([np.ascontiguousarray(p) for p in dyw])
    e = errs["db"] = rel_err(db[c0:c0 + cw2], want)
    assert e <= 1e-4, ("db", e)
    assert not torch.isnan(dz).any()
    want = orc.bwd_dx_act_panels(dys, wrows, f64(z[rows][:, u0:u0 + uw]), orc.ACT_GELU_ERF)
    e = rel_err(dz[rows][:, u0:u0 + uw], want)
    assert e <= TOL["bf16"], ("dz", e)
    # one line per case for the results table (shown with pytest -s)
    print(f"\nPARITY {wname} {lname} " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()) + f" dz={e:.2e}")


def test_config1_full_grid_fp32():
    """q=2, d=1, fp32, X[256,256], W[256,1024], zero bias: all four processors, outputs
    reassembled and compared with the unpartitioned products (seed 0)."""
    w = wl.WORKLOADS[0]
    L = w.layers[0]
    q, d, a, b, c = w.q, w.d, L.a, L.b, L.c
    X, W, bias, dY = wl.full_grid_inputs(a, b, c, dtype="f32", seed=0, bias_std=0.0)
    Xd, Wd, bd, dYd = dev(X), dev(W), dev(bias), dev(dY)
    Y = torch.full((a, c), float("nan"), device="cuda:0")
    dX = torch.full((a, b), float("nan"), device="cuda:0")
    dW = torch.zeros((b, c), device="cuda:0")
    n = c // q
    for i, j, k in itertools.product(range(q), range(q), range(d)):
        desc = B.make_desc(q, d, i, j, k, a, b, c, B.F32, B.F32)
        assert tess.block_shape(desc) == (L.m, L.kb, L.n)
        a_p, b_p = P.fwd_panels(Xd, Wd, q, d, i, j, k)
        tess.linear_fwd(desc, a_p, b_p, bd[j * n:(j + 1) * n], B.ACT_NONE, P.out_block(Y, q, d, i, j, k))
        dy_p, w_p = P.dx_panels(dYd, Wd, q, d, i, j, k)
        tess.linear_bwd_dx(desc, dy_p, w_p, P.out_block(dX, q, d, i, j, k))
        x_p, dy2_p = P.dw_panels(Xd, dYd, q, d, i, j, k)
        tess.linear_bwd_dw(desc, x_p, dy2_p, P.weight_block(dW, q, i, j), accumulate=True)
    torch.cuda.synchronize()
    X64, W64, dY64 = f64(X), f64(W), f64(dY)
    assert rel_err(Y, orc.matmul_nn(X64, W64)) <= TOL["f32"]
    assert rel_err(dX, orc.matmul_nt(dY64, W64)) <= TOL["f32"]
    assert rel_err(dW, orc.matmul_tn(X64, dY64)) <= TOL["f32"]


def test_config2_full_grid_bf16():
    """q=2, d=2, bf16 MLP up-projection: all eight processors on strided views of the
    global X[8192,1024], W[1024,4096], dY[8192,4096]; sampled rows of the reassembled
    Y, dX and of the depth-summed dW against the unpartitioned definition."""
    w = wl.WORKLOADS[1]
    L = w.layers[0]
    q, d, a, b, c = w.q, w.d, L.a, L.b, L.c
    X, W, bias, dY = wl.full_grid_inputs(a, b, c, dtype="bf16", seed=0, bias_std=L.bias_std)
    Xd, Wd, bd, dYd = dev(X), dev(W), dev(bias), dev(dY)
    Y = torch.full((a, c), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    dX = torch.full((a, b), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    dW = torch.zeros((b, c), dtype=torch.float32, device="cuda:0")
    n = c // q
    nbytes = 0
    for i, j, k in itertools.product(range(q), range(q), range(d)):
        desc = B.make_desc(q, d, i, j, k, a, b, c, B.BF16, B.BF16)
        nbytes = max(nbytes, *(tess.workspace_bytes(desc, op) for op in (0, 1, 2)))
    ws = torch.empty(max(nbytes, 4) // 4, dtype=torch.float32, device="cuda:0")
    for i, j, k in itertools.product(range(q), range(q), range(d)):
        desc = B.make_desc(q, d, i, j, k, a, b, c, B.BF16, B.BF16)
        a_p, b_p = P.fwd_panels(Xd, Wd, q, d, i, j, k)
        tess.linear_fwd(desc, a_p, b_p, bd[j * n:(j + 1) * n], B.ACT_GELU_ERF,
                        P.out_block(Y, q, d, i, j, k), workspace=ws)
        dy_p, w_p = P.dx_panels(dYd, Wd, q, d, i, j, k)
        tess.linear_bwd_dx(desc, dy_p, w_p, P.out_block(dX, q, d, i, j, k), workspace=ws)
        x_p, dy2_p = P.dw_panels(Xd, dYd, q, d, i, j, k)
        tess.linear_bwd_dw(desc, x_p, dy2_p, P.weight_block(dW, q, i, j), accumulate=True,
                           workspace=ws)
    torch.cuda.synchronize()
    assert not torch.isnan(Y).any() and not torch.isnan(dX).any()
    X64, W64, dY64 = f64(X), f64(W), f64(dY)
    rows = _sample(a, 96, 3)
    # the unpartitioned definition = one panel per operand
    want = orc.fwd_panels([X64], [W64], bias=f64(bias), act=orc.ACT_GELU_ERF, rows=rows)
    assert rel_err(Y[rows], want) <= TOL["bf16"]
    want = orc.bwd_dx_panels([dY64], [W64], rows=rows)
    assert rel_err(dX[rows], want) <= TOL["bf16"]
    urows = _sample(b, 48, 4)
    want = orc.bwd_dw_panels([X64], [dY64], rows=urows)
    assert rel_err(dW[urows], want) <= 1e-3
