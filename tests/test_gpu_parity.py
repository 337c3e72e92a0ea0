"""GPU parity: the HIP library (through the C ABI) against the CPU fp64 oracle,
element by element on the same seeded inputs.  Sizes span several tiles and
ragged tails and are small enough for the oracle to finish in seconds; the
full-size configurations are in test_gpu_configs.py."""
import itertools

import numpy as np
import pytest
import torch

import tess_workloads as wl
import paper_2105_14500_amd as tess
from paper_2105_14500_amd import binding as B, partition as P
from oracle import tess_oracle as orc
from gpu_util import TOL, f64, dev, run_share, oracle_share, rel_err, workspace, code, tdtype

pytestmark = pytest.mark.gpu


# (q, d, m, kb, n, dtype): what each shape exercises
SHAPES = [
    (2, 1, 256, 128, 256, "bf16"),    # direct 128x128 tiles, fwd split
    (2, 2, 512, 256, 512, "bf16"),    # several 128-tiles per side
    (3, 2, 200, 72, 136, "bf16"),     # ragged M/N/K tails, register-staged loader
    (2, 2, 264, 64, 520, "bf16"),     # K % 64 == 0 (direct), ragged M and N
    (1, 1, 128, 192, 128, "bf16"),    # q = d = 1: plain matmul
    (4, 3, 40, 8, 16, "bf16"),        # tiny: one partial tile
    (2, 2, 33, 17, 29, "bf16"),       # no 8-alignment: generic kernel, bf16 inputs
    (2, 2, 130, 70, 100, "f32"),      # fp32 generic kernel, ragged
    (3, 1, 64, 64, 64, "f32"),
    (2, 2, 1024, 1024, 1024, "bf16"),  # 256x256 tiles
    (2, 1, 2048, 256, 2048, "bf16"),   # 256x256 tiles, many of them
    (16, 1, 64, 64, 128, "bf16"),      # the largest grid dimension the ABI takes: 16 panels per operand
    (8, 8, 128, 64, 256, "bf16"),      # d = q (the 3-D end of the family)
    (16, 2, 24, 40, 56, "f32"),        # 16 panels through the fp32 kernel
]


@pytest.mark.parametrize("q,d,m,kb,n,dtype", SHAPES)
def test_share_matches_oracle(q, d, m, kb, n, dtype):
    inp = wl.share_inputs(q, m, kb, n, dtype=dtype, seed=1234 + m + kb + n, w_std=0.05)
    got = run_share(q, d, inp["x"], inp["w"], inp["bias"], inp["dy"], dtype, dtype,
                    act="gelu_erf", want_preact=True)
    want = oracle_share(inp["x"], inp["w"], inp["bias"], inp["dy"], act="gelu_erf")
    for key in ("y", "preact", "dx", "dw"):
        e = rel_err(got[key], want[key])
        assert e <= TOL[dtype], (key, e)


@pytest.mark.parametrize("q,d,m,kb,n,dtype", SHAPES)
def test_small_integers_are_bit_exact(q, d, m, kb, n, dtype):
    """Inputs in {-2..2}: every product and partial sum is exactly representable
    in fp32, so the fp32 outputs must equal the oracle bit for bit."""
    inp = wl.share_inputs(q, m, kb, n, dtype=dtype, seed=99, integers=True)
    got = run_share(q, d, inp["x"], inp["w"], inp["bias"], inp["dy"], dtype, "f32", act="none")
    want = oracle_share(inp["x"], inp["w"], inp["bias"], inp["dy"], act="none")
    for key in ("y", "dx", "dw"):
        assert np.array_equal(f64(got[key]), want[key]), key


# Launch shapes that the cost model does not pick for any shape above, forced with the
# diagnostic override: (tile, K splits, (q, d, m, kb, n)).  tests/test_plan_coverage.py checks
# on the host that, with these, every kernel variant x split / no split x call is exercised.
FORCED = [
    (128, 3, (3, 2, 200, 72, 136)),        # register-staged loader (ragged K) with K splits
    (128, 1, (2, 2, 264, 64, 520)),
    (256, 2, (2, 2, 1024, 1024, 1024)),    # 256 x 256 tiles, K split, several tiles
    (256, 1, (2, 2, 1024, 1024, 1024)),
    (256, 3, (2, 1, 576, 320, 832)),       # ragged M and N edges on 256 x 256 tiles, uneven split
    (256, 5, (4, 1, 512, 512, 768)),       # five parts
    (256, 8, (4, 1, 512, 512, 512)),
]


@pytest.mark.parametrize("tile,splits,shape", FORCED)
def test_forced_launch_shapes_are_bit_exact(tile, splits, shape):
    q, d, m, kb, n = shape
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=17, integers=True)
    try:
        B.set_plan_override(tile=tile, k_splits=splits)
        desc = B.make_desc(q, d, 0, 0, 0, m * q * d, kb * q, n * q, B.BF16, B.F32)
        for op in (B.OP_FWD, B.OP_BWD_DX, B.OP_BWD_DW):
            assert tess.plan(desc, op) == (tile, tile, splits)
        got = run_share(q, d, inp["x"], inp["w"], inp["bias"], inp["dy"], "bf16", "f32", act="none")
    finally:
        B.set_plan_override(0, 0)
    want = oracle_share(inp["x"], inp["w"], inp["bias"], inp["dy"], act="none")
    for key in ("y", "dx", "dw"):
        assert np.array_equal(f64(got[key]), want[key]), key


@pytest.mark.parametrize("act", ["none", "gelu_erf", "gelu_tanh"])
@pytest.mark.parametrize("dtype,shape", [("bf16", (2, 2, 256, 128, 384)), ("f32", (2, 2, 96, 80, 72))])
def test_epilogue_forms(act, dtype, shape):
    q, d, m, kb, n = shape
    inp = wl.share_inputs(q, m, kb, n, dtype=dtype, seed=7, w_std=0.1, bias_std=0.5)
    got = run_share(q, d, inp["x"], inp["w"], inp["bias"], inp["dy"], dtype, "f32", act=act,
                    want_preact=True)
    xs = [f64(inp["x"][t]) for t in range(q)]
    ws = [f64(inp["w"][t]) for t in range(q)]
    oact = {"none": orc.ACT_NONE, "gelu_erf": orc.ACT_GELU_ERF, "gelu_tanh": orc.ACT_GELU_TANH}[act]
    y, z = orc.fwd_panels(xs, ws, bias=f64(inp["bias"]), act=oact, want_z=True)
    # fp32 outputs: only accumulation-order and erf/tanh rounding remain
    assert rel_err(got["y"], y) <= 1e-5
    assert rel_err(got["preact"], z) <= 1e-5
    # no bias pointer == zero bias
    got0 = run_share(q, d, inp["x"], inp["w"], None, inp["dy"], dtype, "f32", act=act)
    y0 = orc.fwd_panels(xs, ws, bias=None, act=oact)
    assert rel_err(got0["y"], y0) <= 1e-5


def test_bf16_output_is_rne_of_fp32_result():
    """Down-cast decision taken in the kernel's precision: the bf16 output must be
    the round-to-nearest-even of the same kernel's fp32 output."""
    q, d, m, kb, n = 2, 2, 256, 128, 256
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=5, w_std=0.1)
    g32 = run_share(q, d, inp["x"], inp["w"], inp["bias"], inp["dy"], "bf16", "f32")
    g16 = run_share(q, d, inp["x"], inp["w"], inp["bias"], inp["dy"], "bf16", "bf16")
    for key in ("y", "dx", "dw"):
        want = orc.round_bf16(g32[key].numpy())
        assert np.array_equal(f64(g16[key]), want), key


@pytest.mark.parametrize("tile,splits", [(0, 0), (256, 1), (256, 2), (128, 3)])
def test_bf16_gelu_output_does_not_depend_on_asking_for_the_preactivation(tile, splits):
    """The MLP chain keeps the up-projection's pre-activation; a plain call does not.  Both must
    produce the same H, bit for bit, in every launch shape (own drain, K-split reduction)."""
    q, d, m, kb, n = 2, 2, 512, 256, 768
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=21, w_std=0.1, bias_std=0.5)
    try:
        B.set_plan_override(tile=tile, k_splits=splits)
        a = run_share(q, d, inp["x"], inp["w"], inp["bias"], inp["dy"], "bf16", "bf16", act="gelu_erf")
        b = run_share(q, d, inp["x"], inp["w"], inp["bias"], inp["dy"], "bf16", "bf16", act="gelu_erf",
                      want_preact=True)
    finally:
        B.set_plan_override(0, 0)
    assert torch.equal(a["y"], b["y"])
    z = orc.fwd_panels([f64(inp["x"][t]) for t in range(q)], [f64(inp["w"][t]) for t in range(q)],
                       bias=f64(inp["bias"]), act=orc.ACT_NONE)
    assert rel_err(b["preact"], z) <= TOL["bf16"]


def test_gelu_of_exact_preactivations_bf16_out():
    """The 2-byte-output GELU epilogue on pre-activations that carry no rounding: inputs are
    multiples of 1/8 and weights are -1, 0, 1, so every sum is exact in fp32 and the only
    arithmetic left is the kernel's erf, whose absolute error is below 1e-6.  Against the
    fp64 definition rounded to bf16 the output may therefore differ by one bf16 step where
    the exact value sits next to a rounding boundary (plus that 1e-6 in the far negative
    tail, where a bf16 step is smaller still), nowhere by more, and only rarely."""
    q, d, m, kb, n = 2, 2, 256, 128, 256
    r = np.random.default_rng(11)
    x = torch.tensor(r.integers(-4, 5, size=(q, m, kb)) / 8.0, dtype=torch.bfloat16)
    w = torch.tensor(r.integers(-1, 2, size=(q, kb, n)).astype(np.float64), dtype=torch.bfloat16)
    bias = torch.tensor(r.integers(-8, 9, size=(n,)) / 8.0, dtype=torch.bfloat16)
    dy = torch.zeros((q, m, n), dtype=torch.bfloat16)
    got = f64(run_share(q, d, x, w, bias, dy, "bf16", "bf16", act="gelu_erf")["y"])
    y, z = orc.fwd_panels([f64(x[t]) for t in range(q)], [f64(w[t]) for t in range(q)],
                          bias=f64(bias), act=orc.ACT_GELU_ERF, want_z=True)
    assert np.abs(z).max() >= 6.0 and np.abs(z).min() == 0.0          # both tails and the middle
    want = orc.round_bf16(y)
    step = np.maximum(np.abs(want), 2.0 ** -126) * 2.0 ** -7             # >= one bf16 step at |want|
    assert np.all(np.abs(got - want) <= step + 1e-6)
    body = np.abs(want) >= 1e-2
    assert body.mean() > 0.5 and np.mean(got[body] != want[body]) < 5e-3
    assert rel_err(got, y) <= 3e-3                                       # bf16 rounding alone


@pytest.mark.parametrize("dtype,dims", [("bf16", (2, 2, 128, 64, 128)), ("bf16", (3, 3, 24, 40, 56)),
                                        ("f32", (2, 2, 20, 12, 28))])
def test_full_grid_emulation_small(dtype, dims):
    """Every processor of the grid on strided views of the global matrices; the
    reassembled C, dX and the depth-summed dW equal the unpartitioned products."""
    q, d, m, kb, n = dims
    a, b, c = m * q * d, kb * q, n * q
    X, W, bias, dY = wl.full_grid_inputs(a, b, c, dtype=dtype, seed=3, bias_std=0.02, w_std=0.05)
    Xd, Wd, bd, dYd = dev(X), dev(W), dev(bias), dev(dY)
    odt = tdtype(dtype)
    Y = torch.full((a, c), float("nan"), dtype=odt, device="cuda:0")
    dX = torch.full((a, b), float("nan"), dtype=odt, device="cuda:0")
    dW = torch.zeros((b, c), dtype=torch.float32, device="cuda:0")
    for i, j, k in itertools.product(range(q), range(q), range(d)):
        desc = B.make_desc(q, d, i, j, k, a, b, c, code(dtype), code(dtype))
        a_p, b_p = P.fwd_panels(Xd, Wd, q, d, i, j, k)
        tess.linear_fwd(desc, a_p, b_p, bd[j * n:(j + 1) * n], B.ACT_NONE,
                        P.out_block(Y, q, d, i, j, k), workspace=workspace(desc, B.OP_FWD))
        dy_p, w_p = P.dx_panels(dYd, Wd, q, d, i, j, k)
        tess.linear_bwd_dx(desc, dy_p, w_p, P.out_block(dX, q, d, i, j, k),
                           workspace=workspace(desc, B.OP_BWD_DX))
        x_p, dy2_p = P.dw_panels(Xd, dYd, q, d, i, j, k)
        tess.linear_bwd_dw(desc, x_p, dy2_p, P.weight_block(dW, q, i, j), accumulate=True,
                           workspace=workspace(desc, B.OP_BWD_DW))
    torch.cuda.synchronize()
    X64, W64, dY64 = f64(X), f64(W), f64(dY)
    assert rel_err(Y, orc.matmul_nn(X64, W64) + f64(bias)[None, :]) <= TOL[dtype]
    assert rel_err(dX, orc.matmul_nt(dY64, W64)) <= TOL[dtype]
    assert rel_err(dW, orc.matmul_tn(X64, dY64)) <= (1e-5 if dtype == "f32" else 1e-4)


def test_dw_depth_accumulation_order():
    """d calls with accumulate=1, k ascending, into one fp32 buffer."""
    q, d, m, kb, n = 2, 2, 192, 128, 256
    acc = torch.zeros((kb, n), dtype=torch.float32, device="cuda:0")
    want = np.zeros((kb, n))
    for k in range(d):
        inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=50 + k)
        run_share(q, d, inp["x"], inp["w"], None, inp["dy"], "bf16", "bf16", dw_accumulate_into=acc)
        orc.bwd_dw_panels([f64(inp["x"][t]) for t in range(q)], [f64(inp["dy"][t]) for t in range(q)],
                          accumulate_into=want)
    assert rel_err(acc, want) <= 1e-5


def test_run_to_run_determinism():
    q, d, m, kb, n = 4, 2, 256, 512, 256     # split-K path
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=8)
    r1 = run_share(q, d, inp["x"], inp["w"], inp["bias"], inp["dy"], "bf16", "f32", act="gelu_erf")
    r2 = run_share(q, d, inp["x"], inp["w"], inp["bias"], inp["dy"], "bf16", "f32", act="gelu_erf")
    for key in ("y", "dx", "dw"):
        assert torch.equal(r1[key], r2[key]), key


def test_empty_and_error_paths_leave_outputs_untouched():
    q, d, m, kb, n = 2, 2, 64, 64, 64
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=1)
    xd, wd = dev(inp["x"]), dev(inp["w"])
    y = torch.full((m, n), 7.0, dtype=torch.bfloat16, device="cuda:0")
    bad = B.make_desc(q, 3, 0, 0, 0, m * q * 3, kb * q, n * q, B.BF16, B.BF16)   # d > q
    with pytest.raises(tess.TessError) as ei:
        tess.linear_fwd(bad, list(xd), list(wd), None, B.ACT_NONE, y)
    assert ei.value.status == 2
    torch.cuda.synchronize()
    assert torch.all(y == 7.0)


def test_mfma_rate_probe_runs():
    """The measurement loop launches, fills its sink and reports its flop count."""
    sink = torch.full((8 * 256,), float("nan"), dtype=torch.float32, device="cuda:0")
    for real in (False, True):
        sink.fill_(float("nan"))
        flop = B.probe_mfma_rate(sink, 8, 10, real_data=real)
        torch.cuda.synchronize()
        assert flop == 8 * 4 * 10 * 16 * 32768.0
        assert torch.isfinite(sink).all()


def test_calls_can_be_recorded_into_a_hip_graph():
    """The library only enqueues kernels on the stream it is given (no allocation, no memset,
    no synchronisation), so its calls can be recorded into a HIP graph.  Several replays, with
    eager work and synchronisations in between, must reproduce the eager results bit for bit;
    the shape makes the input-gradient call take the K-split path (workspace + reduction)."""
    q, d, m, kb, n = 2, 2, 512, 256, 2048
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=61, w_std=0.1)
    desc = B.make_desc(q, d, 0, 0, 0, m * q * d, kb * q, n * q, B.BF16, B.BF16)
    assert tess.plan(desc, B.OP_BWD_DX)[2] > 1
    x, w, bias, dy = (dev(inp[k]) for k in ("x", "w", "bias", "dy"))
    xl, wl_, dyl = list(x), list(w), list(dy)
    nbytes = max(tess.workspace_bytes(desc, op) for op in (0, 1, 2))
    ws = torch.empty(max(nbytes, 4) // 4, dtype=torch.float32, device="cuda:0")
    y = torch.empty((m, n), dtype=torch.bfloat16, device="cuda:0")
    dx = torch.empty((m, kb), dtype=torch.bfloat16, device="cuda:0")
    dw = torch.empty((kb, n), dtype=torch.bfloat16, device="cuda:0")

    def calls():
        tess.linear_fwd(desc, xl, wl_, bias, B.ACT_GELU_ERF, y, workspace=ws)
        tess.linear_bwd_dx(desc, dyl, wl_, dx, workspace=ws)
        tess.linear_bwd_dw(desc, xl, dyl, dw, workspace=ws)

    calls()
    torch.cuda.synchronize()
    want = [t.clone() for t in (y, dx, dw)]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        calls()
    for rep in range(3):
        for t in (y, dx, dw):
            t.fill_(float("nan"))                       # eager work between the replays
        scratch = torch.randn(1 << 20, device="cuda:0").sum()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, ref in zip((y, dx, dw), want):
            assert torch.equal(got, ref), rep
        assert torch.isfinite(scratch)


def _random_shapes(count, seed):
    r = np.random.default_rng(seed)
    shapes = []
    for _ in range(count):
        q = int(r.integers(1, 6))
        d = int(r.integers(1, q + 1))
        # multiples of 8 (MFMA path, ragged tiles) with an occasional odd size (fp32-FMA path)
        dims = [int(r.integers(1, 90)) * 8 for _ in range(3)]
        if r.random() < 0.2:
            dims[int(r.integers(0, 3))] += int(r.integers(1, 8))
        shapes.append((q, d, *dims))
    return shapes


@pytest.mark.parametrize("q,d,m,kb,n", _random_shapes(24, 2024))
def test_random_block_shapes(q, d, m, kb, n):
    """Seeded random block shapes: ragged tile edges in every direction, contraction lengths
    that are and are not multiples of the 64-deep stage, K-split and single-launch plans."""
    inp = wl.share_inputs(q, m, kb, n, dtype="bf16", seed=m * 7 + kb * 3 + n, w_std=0.05)
    got = run_share(q, d, inp["x"], inp["w"], inp["bias"], inp["dy"], "bf16", "f32", act="gelu_erf")
    want = oracle_share(inp["x"], inp["w"], inp["bias"], inp["dy"], act="gelu_erf")
    for key in ("y", "dx", "dw"):
        e = rel_err(got[key], want[key])
        assert e <= 1e-5, (key, e)
