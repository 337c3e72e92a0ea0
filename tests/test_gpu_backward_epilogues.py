"""GPU parity of the two backward epilogues next to the path: the input gradient taken
through the MLP's middle activation (dX times act'(Z), Section 2.4) and the bias gradient
computed from the dY panels that the weight-gradient call streams (Section 3.2, bias-add).
Both against the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import tess_workloads as wl
import paper_2105_14500_amd as tess
from paper_2105_14500_amd import binding as B
from oracle import tess_oracle as orc
from gpu_util import TOL, f64, dev, rel_err, workspace, code, tdtype, share_desc

pytestmark = pytest.mark.gpu

ACTS = {"none": (B.ACT_NONE, orc.ACT_NONE), "gelu_erf": (B.ACT_GELU_ERF, orc.ACT_GELU_ERF),
        "gelu_tanh": (B.ACT_GELU_TANH, orc.ACT_GELU_TANH)}
# (q, d, m, kb, n): one tile, several tiles with ragged edges, a K-split shape, unaligned
SHAPES = [(2, 1, 128, 128, 64), (2, 2, 320, 200, 136), (3, 2, 264, 520, 192), (2, 2, 512, 256, 2048),
          (2, 1, 4096, 128, 128), (2, 1, 50, 36, 28)]


def _z(m, kb, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn((m, kb), generator=g) * 1.5).to(tdtype(dtype))


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("dtype,out", [("bf16", "bf16"), ("bf16", "f32"), ("f32", "f32")])
@pytest.mark.parametrize("act", ["gelu_erf", "gelu_tanh", "none"])
def test_dx_through_activation(shape, dtype, out, act):
    q, d, m, kb, n = shape
    inp = wl.share_inputs(q, m, kb, n, dtype=dtype, seed=31, w_std=0.1)
    z = _z(m, kb, dtype, 32)
    desc = share_desc(q, d, m, kb, n, dtype, out)
    dyd, wd = dev(inp["dy"]), dev(inp["w"])
    dz = torch.full((m, kb), float("nan"), dtype=tdtype(out), device="cuda:0")
    tess.linear_bwd_dx_act(desc, list(dyd), list(wd), dev(z), ACTS[act][0], dz,
                           workspace=workspace(desc, B.OP_BWD_DX))
    torch.cuda.synchronize()
    want = orc.bwd_dx_act_panels([f64(inp["dy"][t]) for t in range(q)],
                                 [f64(inp["w"][t]) for t in range(q)], f64(z), ACTS[act][1])
    assert rel_err(dz, want) <= (TOL["bf16"] if out == "bf16" else 1e-5)
    if act == "none":
        # identical to the plain call, bit for bit
        dx = torch.empty_like(dz)
        tess.linear_bwd_dx(desc, list(dyd), list(wd), dx, workspace=workspace(desc, B.OP_BWD_DX))
        torch.cuda.synchronize()
        assert torch.equal(dx, dz)


def test_dx_activation_gradient_of_exact_sums_bf16_out():
    """Sums that carry no rounding (dY multiples of 1/8, W in {-1,0,1}) leave the erf-form
    derivative as the only arithmetic: against the fp64 definition rounded to bf16 the output
    differs by at most one bf16 step plus the 1e-6 of the approximation, and rarely."""
    q, d, m, kb, n = 2, 2, 256, 256, 64
    r = np.random.default_rng(41)
    dy = torch.tensor(r.integers(-8, 9, size=(q, m, n)) / 8.0, dtype=torch.bfloat16)
    w = torch.tensor(r.integers(-1, 2, size=(q, kb, n)).astype(np.float64), dtype=torch.bfloat16)
    z = torch.tensor(r.integers(-48, 49, size=(m, kb)) / 8.0, dtype=torch.bfloat16)
    desc = share_desc(q, d, m, kb, n, "bf16", "bf16")
    dz = torch.full((m, kb), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    tess.linear_bwd_dx_act(desc, list(dev(dy)), list(dev(w)), dev(z), B.ACT_GELU_ERF, dz,
                           workspace=workspace(desc, B.OP_BWD_DX))
    torch.cuda.synchronize()
    dx = orc.bwd_dx_panels([f64(dy[t]) for t in range(q)], [f64(w[t]) for t in range(q)])
    exact = dx * orc.gelu_erf_grad(f64(z))
    want = orc.round_bf16(exact)
    got = f64(dz)
    step = np.maximum(np.abs(want), 2.0 ** -126) * 2.0 ** -7
    assert np.all(np.abs(got - want) <= step + 1e-6 * np.maximum(np.abs(dx), 1.0))
    body = np.abs(want) >= 1e-2
    assert body.mean() > 0.3 and np.mean(got[body] != want[body]) < 1e-2


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_dw_with_bias_gradient(shape, dtype):
    q, d, m, kb, n = shape
    inp = wl.share_inputs(q, m, kb, n, dtype=dtype, seed=33, w_std=0.1)
    desc = share_desc(q, d, m, kb, n, dtype, "f32")
    xd, dyd = dev(inp["x"]), dev(inp["dy"])
    ws = workspace(desc, B.OP_BWD_DW)
    dw = torch.full((kb, n), float("nan"), device="cuda:0")
    db = torch.full((n,), float("nan"), device="cuda:0")
    tess.linear_bwd_dw_bias(desc, list(xd), list(dyd), dw, db, workspace=ws)
    torch.cuda.synchronize()
    xs = [f64(inp["x"][t]) for t in range(q)]
    dys = [f64(inp["dy"][t]) for t in range(q)]
    want_dw, want_db = orc.bwd_dw_panels(xs, dys), orc.bias_grad_panels(dys)
    assert rel_err(dw, want_dw) <= 1e-5
    assert rel_err(db, want_db) <= 1e-5
    # the weight gradient is the plain call's, bit for bit
    dw2 = torch.empty_like(dw)
    tess.linear_bwd_dw(desc, list(xd), list(dyd), dw2, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(dw, dw2)
    # depth accumulation: a second layer's panels are added to both outputs
    inp2 = wl.share_inputs(q, m, kb, n, dtype=dtype, seed=34, w_std=0.1)
    tess.linear_bwd_dw_bias(desc, list(dev(inp2["x"])), list(dev(inp2["dy"])), dw, db,
                            accumulate=True, workspace=ws)
    torch.cuda.synchronize()
    dys2 = [f64(inp2["dy"][t]) for t in range(q)]
    orc.bias_grad_panels(dys2, accumulate_into=want_db)
    orc.bwd_dw_panels([f64(inp2["x"][t]) for t in range(q)], dys2, accumulate_into=want_dw)
    assert rel_err(dw, want_dw) <= 1e-5
    assert rel_err(db, want_db) <= 1e-5


def test_bias_gradient_of_integers_is_exact():
    q, d, m, kb, n = 2, 2, 384, 256, 320
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=35, integers=True)
    desc = share_desc(q, d, m, kb, n, "bf16", "f32")
    dw = torch.empty((kb, n), device="cuda:0")
    db = torch.empty((n,), device="cuda:0")
    tess.linear_bwd_dw_bias(desc, list(dev(inp["x"])), list(dev(inp["dy"])), dw, db,
                            workspace=workspace(desc, B.OP_BWD_DW))
    torch.cuda.synchronize()
    want = orc.bias_grad_panels([f64(inp["dy"][t]) for t in range(q)])
    assert np.array_equal(f64(db), want)


def test_new_entry_points_reject_bad_arguments():
    q, d, m, kb, n = 2, 2, 128, 64, 128
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=36)
    desc = share_desc(q, d, m, kb, n, "bf16", "bf16")
    dz = torch.full((m, kb), 7.0, dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(B.TessError) as e:
        tess.linear_bwd_dx_act(desc, list(dev(inp["dy"])), list(dev(inp["w"])), None, B.ACT_GELU_ERF, dz)
    assert e.value.status == 1
    with pytest.raises(B.TessError) as e:
        tess.linear_bwd_dx_act(desc, list(dev(inp["dy"])), list(dev(inp["w"])), dz.clone(), 9, dz)
    assert e.value.status == 5
    dw = torch.full((kb, n), 7.0, device="cuda:0")
    with pytest.raises(B.TessError) as e:
        tess.linear_bwd_dw_bias(desc, list(dev(inp["x"])), list(dev(inp["dy"])), dw, None, accumulate=True)
    assert e.value.status == 1
    torch.cuda.synchronize()
    assert torch.all(dz == 7.0) and torch.all(dw == 7.0)


@pytest.mark.parametrize("shape", [(2, 2, 128, 128, 64), (3, 1, 264, 200, 136), (2, 1, 512, 256, 2048),
                                   (2, 1, 4096, 128, 128), (2, 1, 50, 36, 28)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_stepwise_partial_products(shape, dtype):
    """Section 3.1's own wording of the backward: one step's partial product on single blocks,
    fp32 out, against the plain block products; accumulated over the q members of the reduce
    group it reproduces the owner-computes calls."""
    q, d, m, kb, n = shape
    inp = wl.share_inputs(q, m, kb, n, dtype=dtype, seed=51, w_std=0.1)
    desc = share_desc(q, d, m, kb, n, dtype, "f32")
    xd, wd, dyd = dev(inp["x"]), dev(inp["w"]), dev(inp["dy"])
    # one step each
    p = torch.full((m, kb), float("nan"), device="cuda:0")
    tess.linear_bwd_dx_step(desc, dyd[0], wd[0], p, workspace=workspace(desc, B.OP_BWD_DX_STEP))
    pw = torch.full((kb, n), float("nan"), device="cuda:0")
    tess.linear_bwd_dw_step(desc, xd[0], dyd[0], pw, workspace=workspace(desc, B.OP_BWD_DW_STEP))
    torch.cuda.synchronize()
    assert rel_err(p, orc.matmul_nt(f64(inp["dy"][0]), f64(inp["w"][0]))) <= 1e-5
    assert rel_err(pw, orc.matmul_tn(f64(inp["x"][0]), f64(inp["dy"][0]))) <= 1e-5
    # the reduce group played on one GPU: partials of members 1..q-1 added to member 0's
    for t in range(1, q):
        tess.linear_bwd_dx_step(desc, dyd[t], wd[t], p, accumulate=True,
                                workspace=workspace(desc, B.OP_BWD_DX_STEP))
        tess.linear_bwd_dw_step(desc, xd[t], dyd[t], pw, accumulate=True,
                                workspace=workspace(desc, B.OP_BWD_DW_STEP))
    torch.cuda.synchronize()
    dys = [f64(inp["dy"][t]) for t in range(q)]
    assert rel_err(p, orc.bwd_dx_panels(dys, [f64(inp["w"][t]) for t in range(q)])) <= 1e-5
    assert rel_err(pw, orc.bwd_dw_panels([f64(inp["x"][t]) for t in range(q)], dys)) <= 1e-5
