"""Pins of the CPU oracle to things other than itself (no GPU needed).

Each test ties one part of oracle/tess_oracle.c to a fact that the paper or
the mathematics fixes: the unpartitioned product from numpy's fp64 matmul
(Alg. 3 "combine all C_ij into C"; the Experiment section's own check), the
SUMMA gradient equation, the depth sum of Section 3.1, the adjoint identity,
hand-written block tables, exact integer arithmetic, textbook normal-CDF
values, and bit patterns for bfloat16 rounding.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import tess_oracle as orc

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
GRIDS = [(q, d) for q in range(1, 5) for d in range(1, q + 1)]


def _rng(seed):
    return np.random.default_rng(seed)


def _sizes(q, d, seed):
    """Non-square blocks: m, kb, n all different."""
    r = _rng(seed)
    m, kb, n = (int(v) for v in r.choice(np.arange(2, 9), size=3, replace=False))
    return m * q * d, kb * q, n * q, m, kb, n


def _read_table(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            left, _, right = line.partition("|")
            rows.append((left.split(), right.split()))
    return rows


# ---------------------------------------------------------------- plain products

def test_unpartitioned_products_match_numpy():
    r = _rng(1)
    A = r.standard_normal((7, 5))
    B = r.standard_normal((5, 9))
    np.testing.assert_allclose(orc.matmul_nn(A, B), A @ B, rtol=1e-13, atol=1e-13)
    Bt = r.standard_normal((9, 5))
    np.testing.assert_allclose(orc.matmul_nt(A, Bt), A @ Bt.T, rtol=1e-13, atol=1e-13)
    At = r.standard_normal((5, 7))
    np.testing.assert_allclose(orc.matmul_tn(At, B), At.T @ B, rtol=1e-13, atol=1e-13)


def test_products_brute_force_tiny():
    """Definition by Python loops on a 2x3 * 3x2 integer case worked by hand."""
    A = np.array([[1., 2., 3.], [4., 5., 6.]])
    B = np.array([[1., -1.], [0., 2.], [3., 1.]])
    want = np.array([[10., 6.], [22., 12.]])
    assert np.array_equal(orc.matmul_nn(A, B), want)
    assert np.array_equal(orc.matmul_nt(A, B.T.copy()), want)
    assert np.array_equal(orc.matmul_tn(A.T.copy(), B), want)


# ---------------------------------------------------------------- Alg. 3 forward

@pytest.mark.parametrize("q,d", GRIDS)
def test_forward_reassembles_to_full_product(q, d):
    a, b, c, m, kb, n = _sizes(q, d, 10 * q + d)
    r = _rng(100 + q * 7 + d)
    A = r.standard_normal((a, b))
    B = r.standard_normal((b, c))
    C = np.full((a, c), np.nan)
    for i, j, k in itertools.product(range(q), range(q), range(d)):
        h = i + k * q                      # Alg. 3 set-up loop
        blk = orc.tess_fwd(q, d, i, j, k, A, B)
        assert blk.shape == (m, n)
        C[h * m:(h + 1) * m, j * n:(j + 1) * n] = blk
    np.testing.assert_allclose(C, A @ B, rtol=1e-12, atol=1e-12)


def test_forward_block_table_by_hand():
    """tests/golden/partition_q2_d2.txt: B = I makes C_{i,j,k} the stored block of A."""
    A = np.array([[10.0 * r + u for u in range(4)] for r in range(8)])
    B = np.eye(4)
    table = _read_table("partition_q2_d2.txt")
    assert len(table) == 8
    for (i, j, k), vals in table:
        blk = orc.tess_fwd(2, 2, int(i), int(j), int(k), A, B)
        want = np.array([float(v) for v in vals]).reshape(2, 2)
        assert np.array_equal(blk, want), (i, j, k)


def test_block_row_map():
    assert orc.block_row(2, 1, 1) == 3
    assert orc.block_row(4, 3, 2) == 11
    assert orc.block_row(4, 0, 0) == 0


def test_forward_special_cases():
    r = _rng(3)
    A = r.standard_normal((6, 4))
    B = r.standard_normal((4, 10))
    # q = d = 1 is the plain matmul (the [1,1,1] row of the weak-scaling table)
    np.testing.assert_allclose(orc.tess_fwd(1, 1, 0, 0, 0, A, B), A @ B, rtol=1e-13, atol=1e-13)
    # d = 1 is SUMMA: block (i,j) of C = sum_t A_it B_tj
    q = 2
    for i, j in itertools.product(range(q), range(q)):
        want = sum(A[3 * i:3 * i + 3, 2 * t:2 * t + 2] @ B[2 * t:2 * t + 2, 5 * j:5 * j + 5]
                   for t in range(q))
        np.testing.assert_allclose(orc.tess_fwd(q, 1, i, j, 0, A, B), want, rtol=1e-13, atol=1e-13)


def test_forward_bias_is_column_slice_and_precedes_activation():
    q, d = 2, 2
    r = _rng(4)
    A = r.standard_normal((8, 6))
    B = r.standard_normal((6, 4))
    bias = np.array([100.0, 200.0, 300.0, 400.0])
    full = A @ B + bias[None, :]
    for i, j, k in itertools.product(range(q), range(q), range(d)):
        h = i + k * q
        y, z = orc.tess_fwd(q, d, i, j, k, A, B, bias=bias, act=orc.ACT_NONE, want_z=True)
        np.testing.assert_allclose(y, full[2 * h:2 * h + 2, 2 * j:2 * j + 2], rtol=1e-12)
        np.testing.assert_allclose(z, y, rtol=0, atol=0)
    # activation acts on (Z + bias): a large bias turns GELU into the identity,
    # a large negative one into zero -- wrong order (act before bias) fails both
    y = orc.tess_fwd(q, d, 0, 0, 0, A, B, bias=np.full(4, 50.0), act=orc.ACT_GELU_ERF)
    np.testing.assert_allclose(y, (A @ B)[0:2, 0:2] + 50.0, rtol=1e-12)
    y = orc.tess_fwd(q, d, 0, 0, 0, A, B, bias=np.full(4, -50.0), act=orc.ACT_GELU_ERF)
    assert np.all(np.abs(y) < 1e-300)


# ---------------------------------------------------------------- gradients

@pytest.mark.parametrize("q,d", GRIDS)
def test_dx_reassembles_to_dy_wT(q, d):
    a, b, c, m, kb, n = _sizes(q, d, 20 * q + d)
    r = _rng(200 + q * 7 + d)
    dY = r.standard_normal((a, c))
    W = r.standard_normal((b, c))
    dX = np.full((a, b), np.nan)
    for i, j, k in itertools.product(range(q), range(q), range(d)):
        h = i + k * q
        blk = orc.tess_bwd_dx(q, d, i, j, k, dY, W)
        assert blk.shape == (m, kb)
        dX[h * m:(h + 1) * m, j * kb:(j + 1) * kb] = blk
    np.testing.assert_allclose(dX, dY @ W.T, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("q,d", GRIDS)
def test_dw_depth_sum_is_xT_dy(q, d):
    a, b, c, m, kb, n = _sizes(q, d, 30 * q + d)
    r = _rng(300 + q * 7 + d)
    X = r.standard_normal((a, b))
    dY = r.standard_normal((a, c))
    full = X.T @ dY
    dW = np.full((b, c), np.nan)
    dW_acc = np.zeros((b, c))
    for i, j in itertools.product(range(q), range(q)):
        parts = [orc.tess_bwd_dw(q, d, i, j, k, X, dY) for k in range(d)]
        assert parts[0].shape == (kb, n)
        dW[i * kb:(i + 1) * kb, j * n:(j + 1) * n] = sum(parts)
        acc = np.zeros((kb, n))
        for k in range(d):                       # the accumulate form of the depth sum
            orc.tess_bwd_dw(q, d, i, j, k, X, dY, accumulate_into=acc)
        dW_acc[i * kb:(i + 1) * kb, j * n:(j + 1) * n] = acc
        if d > 1:                                # one slice alone is NOT the gradient
            assert not np.allclose(parts[0], full[i * kb:(i + 1) * kb, j * n:(j + 1) * n])
    np.testing.assert_allclose(dW, full, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dW_acc, full, rtol=1e-12, atol=1e-12)


def test_dw_one_hot_lands_on_one_processor():
    """A single non-zero in X and dY at the same row: only the depth layer that
    holds that row contributes, at block (u0 // kb, s0 // n)."""
    q, d, m, kb, n = 2, 2, 3, 2, 4
    a, b, c = m * q * d, kb * q, n * q
    r0, u0, s0 = 10, 3, 5            # row 10 -> block row h = 3 = i + k*q -> (t=1, k=1)
    X = np.zeros((a, b)); X[r0, u0] = 2.0
    dY = np.zeros((a, c)); dY[r0, s0] = 3.0
    for i, j, k in itertools.product(range(q), range(q), range(d)):
        blk = orc.tess_bwd_dw(q, d, i, j, k, X, dY)
        want = np.zeros((kb, n))
        if (i, j, k) == (1, 1, 1):
            want[u0 - kb, s0 - n] = 6.0
        assert np.array_equal(blk, want), (i, j, k)


def test_adjoint_identity():
    q, d = 3, 2
    a, b, c, m, kb, n = _sizes(q, d, 77)
    r = _rng(5)
    X = r.standard_normal((a, b)); W = r.standard_normal((b, c)); dY = r.standard_normal((a, c))
    Y = np.zeros((a, c)); dX = np.zeros((a, b)); dW = np.zeros((b, c))
    for i, j, k in itertools.product(range(q), range(q), range(d)):
        h = i + k * q
        Y[h * m:(h + 1) * m, j * n:(j + 1) * n] = orc.tess_fwd(q, d, i, j, k, X, W)
        dX[h * m:(h + 1) * m, j * kb:(j + 1) * kb] = orc.tess_bwd_dx(q, d, i, j, k, dY, W)
        dW[i * kb:(i + 1) * kb, j * n:(j + 1) * n] += orc.tess_bwd_dw(q, d, i, j, k, X, dY)
    s0 = np.sum(dY * Y)
    assert abs(np.sum(dX * X) - s0) <= 1e-11 * abs(s0)
    assert abs(np.sum(dW * W) - s0) <= 1e-11 * abs(s0)


def test_small_integer_inputs_are_exact():
    """Inputs in {-2..2}: every product and partial sum is an integer far below
    2^53, so the blocked sums equal numpy's integer matmul exactly."""
    q, d, m, kb, n = 3, 2, 4, 5, 6
    a, b, c = m * q * d, kb * q, n * q
    r = _rng(6)
    X = r.integers(-2, 3, (a, b)); W = r.integers(-2, 3, (b, c)); dY = r.integers(-2, 3, (a, c))
    Y = X @ W; dX = dY @ W.T; dW = X.T @ dY
    for i, j, k in itertools.product(range(q), range(q), range(d)):
        h = i + k * q
        assert np.array_equal(orc.tess_fwd(q, d, i, j, k, X, W),
                              Y[h * m:(h + 1) * m, j * n:(j + 1) * n])
        assert np.array_equal(orc.tess_bwd_dx(q, d, i, j, k, dY, W),
                              dX[h * m:(h + 1) * m, j * kb:(j + 1) * kb])
    for i, j in itertools.product(range(q), range(q)):
        acc = np.zeros((kb, n))
        for k in range(d):
            orc.tess_bwd_dw(q, d, i, j, k, X, dY, accumulate_into=acc)
        assert np.array_equal(acc, dW[i * kb:(i + 1) * kb, j * n:(j + 1) * n])


def test_panel_forms_match_global_forms_and_row_subsets():
    q, d, i, j, k = 3, 2, 1, 2, 1
    a, b, c, m, kb, n = _sizes(q, d, 88)
    r = _rng(7)
    X = r.standard_normal((a, b)); W = r.standard_normal((b, c)); dY = r.standard_normal((a, c))
    bias = r.standard_normal(c)
    h = i + k * q
    # panels as strided views of the global matrices
    a_p = [X[h * m:(h + 1) * m, t * kb:(t + 1) * kb] for t in range(q)]
    b_p = [W[t * kb:(t + 1) * kb, j * n:(j + 1) * n] for t in range(q)]
    y = orc.fwd_panels(a_p, b_p, bias=bias[j * n:(j + 1) * n], act=orc.ACT_GELU_ERF)
    np.testing.assert_array_equal(y, orc.tess_fwd(q, d, i, j, k, X, W, bias=bias,
                                                  act=orc.ACT_GELU_ERF))
    rows = np.array([m - 1, 0])
    np.testing.assert_array_equal(
        orc.fwd_panels(a_p, b_p, bias=bias[j * n:(j + 1) * n], act=orc.ACT_GELU_ERF, rows=rows),
        y[rows])
    dy_p = [dY[h * m:(h + 1) * m, t * n:(t + 1) * n] for t in range(q)]
    w_p = [W[j * kb:(j + 1) * kb, t * n:(t + 1) * n] for t in range(q)]
    dx = orc.bwd_dx_panels(dy_p, w_p)
    np.testing.assert_array_equal(dx, orc.tess_bwd_dx(q, d, i, j, k, dY, W))
    np.testing.assert_array_equal(orc.bwd_dx_panels(dy_p, w_p, rows=rows), dx[rows])
    x_p = [X[(t + k * q) * m:(t + k * q + 1) * m, i * kb:(i + 1) * kb] for t in range(q)]
    dy2_p = [dY[(t + k * q) * m:(t + k * q + 1) * m, j * n:(j + 1) * n] for t in range(q)]
    dw = orc.bwd_dw_panels(x_p, dy2_p)
    np.testing.assert_array_equal(dw, orc.tess_bwd_dw(q, d, i, j, k, X, dY))
    urows = np.array([kb - 1, 1])
    np.testing.assert_array_equal(orc.bwd_dw_panels(x_p, dy2_p, rows=urows), dw[urows])


# ---------------------------------------------------------------- shapes, grid rules

def test_block_shapes_and_memory_closed_form():
    """Section 3.1 memory model: ab/p + bcd/p + ac/p elements per processor."""
    import tess_workloads as wl
    table = {left[0]: ([int(v) for v in left[1:]], [int(v) for v in right])
             for left, right in _read_table("block_shapes.txt")}
    seen = 0
    for w in wl.WORKLOADS:
        for L in w.layers:
            (q, d, a, b, c), (m, kb, n) = table[f"{w.name}/{L.name}"]
            assert (w.q, w.d, L.a, L.b, L.c, L.m, L.kb, L.n) == (q, d, a, b, c, m, kb, n)
            p = d * q * q
            assert m * kb * p == a * b and kb * n * p == b * c * d and m * n * p == a * c
            assert orc.check_grid(q, d, 0, 0, 0, a, b, c) == 0
            X = np.zeros((a // 64, b // 64)); W = np.zeros((b // 64, c // 64))
            assert orc.tess_fwd(q, d, 0, 0, 0, X, W).shape == (m // 64, n // 64)
            seen += 1
    assert seen == len(table) == 8


def test_grid_rules():
    ok = orc.check_grid
    assert ok(2, 2, 1, 1, 1, 8, 4, 6) == 0
    assert ok(2, 3, 0, 0, 0, 12, 4, 6) != 0          # d > q is outside 1 <= d <= q
    assert ok(0, 1, 0, 0, 0, 8, 4, 6) != 0
    assert ok(2, 0, 0, 0, 0, 8, 4, 6) != 0
    assert ok(2, 2, 2, 0, 0, 8, 4, 6) != 0           # coordinate outside the grid
    assert ok(2, 2, 0, 0, 2, 8, 4, 6) != 0
    assert ok(2, 2, 0, 0, 0, 6, 4, 6) != 0           # a not divisible by q*d
    assert ok(2, 2, 0, 0, 0, 8, 3, 6) != 0
    assert ok(2, 2, 0, 0, 0, 8, 4, 5) != 0


# ---------------------------------------------------------------- scalar helpers

def test_gelu_against_normal_cdf_table():
    seen = 0
    with open(os.path.join(GOLDEN, "normal_cdf.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            x, phi = (float(v) for v in line.split())
            assert abs(orc.gelu_erf(x) - x * phi) <= 2e-15 * max(1.0, abs(x))
            seen += 1
    assert seen == 7


def test_gelu_identities():
    assert orc.gelu_erf(0.0) == 0.0 and orc.gelu_tanh(0.0) == 0.0
    for x in (0.1, 0.7, 1.3, 2.9, 6.0):
        assert abs(orc.gelu_erf(x) - orc.gelu_erf(-x) - x) < 1e-15 * max(1, x)
        assert abs(orc.gelu_tanh(x) - orc.gelu_tanh(-x) - x) < 1e-15 * max(1, x)
    assert orc.gelu_erf(12.0) == 12.0 and abs(orc.gelu_erf(-12.0)) < 1e-30
    # the tanh form is a different function: close to, but not, the erf form
    assert 1e-5 < abs(orc.gelu_tanh(1.0) - orc.gelu_erf(1.0)) < 1e-3
    # value of the tanh form at 1 from its formula evaluated independently
    want = 0.5 * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * 1.044715))
    assert abs(orc.gelu_tanh(1.0) - want) < 1e-15


def test_gelu_tanh_form_against_library_routine_and_its_gap_to_the_exact_form():
    """The tanh form is pinned to things other than its own formula: (1) PyTorch's CPU
    fp64 `gelu(approximate="tanh")`, a library routine; (2) the largest distance between
    the tanh form and the exact form x Phi(x) (itself pinned by the normal-CDF table) over
    [-8, 8]: 4.732e-4, reached at |x| = 2.699 -- a mistyped cubic coefficient moves it well
    outside the band (0.04715 gives 1.5e-3, 0.045 gives 5.6e-4), a low digit of sqrt(2/pi)
    moves it too; (3) the tails: identity for large x, zero for very negative x."""
    torch = pytest.importorskip("torch")
    xs = np.linspace(-8.0, 8.0, 160001)
    got = np.array([orc.gelu_tanh(float(x)) for x in xs[::40]])
    lib = torch.nn.functional.gelu(torch.from_numpy(xs[::40].copy()), approximate="tanh").numpy()
    assert np.max(np.abs(got - lib)) < 2e-14
    gt = np.array([orc.gelu_tanh(float(x)) for x in xs])
    ge = np.array([orc.gelu_erf(float(x)) for x in xs])
    gap = np.abs(gt - ge)
    i = int(np.argmax(gap))
    assert abs(gap[i] - 4.732e-4) < 2e-6, gap[i]
    assert abs(abs(xs[i]) - 2.699) < 0.01, xs[i]
    assert orc.gelu_tanh(9.0) == 9.0 and abs(orc.gelu_tanh(-9.0)) < 1e-30
    assert abs(orc.gelu_tanh(40.0) - 40.0) == 0.0 and orc.gelu_tanh(-40.0) == 0.0


def test_gelu_tanh_derivative_against_autograd_and_its_gap_to_the_exact_derivative():
    """Same for the derivative: PyTorch's fp64 autograd through its own tanh-form GELU,
    and the largest distance to the exact derivative Phi(x) + x phi(x) (pinned above by
    tabulated values): 8.685e-4 at |x| = 2.019."""
    torch = pytest.importorskip("torch")
    xs = np.linspace(-8.0, 8.0, 160001)
    xt = torch.from_numpy(xs[::40].copy()).requires_grad_()
    torch.nn.functional.gelu(xt, approximate="tanh").sum().backward()
    got = np.array([float(orc.gelu_tanh_grad(float(x))) for x in xs[::40]])
    assert np.max(np.abs(got - xt.grad.numpy())) < 2e-14
    xe = torch.from_numpy(xs[::40].copy()).requires_grad_()
    torch.nn.functional.gelu(xe).sum().backward()
    gote = np.array([float(orc.gelu_erf_grad(float(x))) for x in xs[::40]])
    assert np.max(np.abs(gote - xe.grad.numpy())) < 2e-14
    dt = np.array([float(orc.gelu_tanh_grad(float(x))) for x in xs])
    de = np.array([float(orc.gelu_erf_grad(float(x))) for x in xs])
    gap = np.abs(dt - de)
    i = int(np.argmax(gap))
    assert abs(gap[i] - 8.685e-4) < 2e-6, gap[i]
    assert abs(abs(xs[i]) - 2.019) < 0.01, xs[i]
    assert float(orc.gelu_tanh_grad(9.0)) == 1.0 and abs(float(orc.gelu_tanh_grad(-9.0))) < 1e-30


def test_bf16_rounding_bit_patterns():
    def f(bits):
        return np.array([bits], dtype=np.uint32).view(np.float32)[0]

    def bits_of(x):
        return int(np.array([x], dtype=np.float32).view(np.uint32)[0])

    cases = [
        (0x3F800000, 0x3F800000),   # 1.0 stays
        (0x3F808000, 0x3F800000),   # exact tie, even mantissa below -> down
        (0x3F818000, 0x3F820000),   # exact tie, odd mantissa below -> up
        (0x3F808001, 0x3F810000),   # just above the tie -> up
        (0x3F807FFF, 0x3F800000),   # just below the tie -> down
        (0xBF818000, 0xBF820000),   # sign carried
        (0x7F7FFFFF, 0x7F800000),   # largest fp32 rounds to +inf
        (0x00000000, 0x00000000),
        (0x80000000, 0x80000000),
    ]
    for src, want in cases:
        got = orc.round_bf16(np.array([f(src)], dtype=np.float32))[0]
        assert bits_of(np.float32(got)) == want, hex(src)
    # the result is always representable in bfloat16 (low 16 bits clear)
    x = _rng(9).standard_normal(1000).astype(np.float32)
    y = orc.round_bf16(x).astype(np.float32)
    assert np.all((y.view(np.uint32) & 0xFFFF) == 0)
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -8)


def test_rel_frobenius():
    O = np.array([[3.0, 4.0]])
    G = np.array([[3.0, 4.5]])
    assert abs(orc.rel_frobenius(G, O) - 0.1) < 1e-15
    assert orc.rel_frobenius(O, O) == 0.0


def test_planted_mistakes_are_caught():
    """A transposed block map (h = i*d + k) or a dropped step disagrees with numpy."""
    q, d, m, kb, n = 2, 2, 2, 3, 2
    a, b, c = m * q * d, kb * q, n * q
    r = _rng(11)
    A = r.standard_normal((a, b)); B = r.standard_normal((b, c))
    full = A @ B
    wrong = 0
    for i, j, k in itertools.product(range(q), range(q), range(d)):
        h_bad = i * d + k
        blk = orc.tess_fwd(q, d, i, j, k, A, B)
        if not np.allclose(blk, full[h_bad * m:(h_bad + 1) * m, j * n:(j + 1) * n]):
            wrong += 1
    assert wrong > 0


# ------------------------------------------------- backward epilogues next to the path
def test_gelu_derivatives_against_central_differences():
    """The derivative formulas against central differences of the GELU forms that the
    tests above pin (step 1e-5: truncation ~1e-11, rounding ~1e-11)."""
    h = 1e-5
    for x in np.linspace(-6.0, 6.0, 97):
        fd = (orc.gelu_erf(x + h) - orc.gelu_erf(x - h)) / (2 * h)
        assert abs(float(orc.gelu_erf_grad(x)) - float(fd)) < 5e-10, x
        fd = (orc.gelu_tanh(x + h) - orc.gelu_tanh(x - h)) / (2 * h)
        assert abs(float(orc.gelu_tanh_grad(x)) - float(fd)) < 5e-10, x


def test_gelu_derivative_special_values():
    # at 0 only Phi(0) = 1/2 is left; far out the function is the identity or zero
    assert float(orc.gelu_erf_grad(0.0)) == 0.5 and float(orc.gelu_tanh_grad(0.0)) == 0.5
    assert abs(float(orc.gelu_erf_grad(12.0)) - 1.0) < 1e-15 and abs(float(orc.gelu_erf_grad(-12.0))) < 1e-15
    # Phi(x) + x phi(x) at x = 1 and -1 from the tabulated Phi(1) and phi(1) = e^{-1/2}/sqrt(2 pi)
    phi1 = np.exp(-0.5) / np.sqrt(2 * np.pi)
    assert abs(float(orc.gelu_erf_grad(1.0)) - (0.841344746068543 + phi1)) < 1e-14
    assert abs(float(orc.gelu_erf_grad(-1.0)) - (0.158655253931457 - phi1)) < 1e-14
    # symmetry that follows from Phi(-x) = 1 - Phi(x): g'(x) + g'(-x) = 1
    for x in (0.3, 1.7, 4.0):
        assert abs(float(orc.gelu_erf_grad(x)) + float(orc.gelu_erf_grad(-x)) - 1.0) < 1e-15
        assert abs(float(orc.gelu_tanh_grad(x)) + float(orc.gelu_tanh_grad(-x)) - 1.0) < 1e-15
    # GELU has its minimum where the derivative changes sign: bracket it and check that
    # the function is indeed smallest there
    lo, hi = -1.0, -0.5
    assert orc.gelu_erf_grad(lo) < 0 < orc.gelu_erf_grad(hi)
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        lo, hi = (mid, hi) if orc.gelu_erf_grad(mid) < 0 else (lo, mid)
    xs = np.linspace(-3, 3, 6001)
    assert abs(xs[np.argmin(orc.gelu_erf(xs))] - lo) < 2e-3


def test_dx_with_activation_gradient():
    q, m, kb, n = 3, 5, 4, 6
    r = _rng(21)
    dys = [r.standard_normal((m, n)) for _ in range(q)]
    ws = [r.standard_normal((kb, n)) for _ in range(q)]
    z = r.standard_normal((m, kb)) * 2
    dx = orc.bwd_dx_panels(dys, ws)
    # identity activation changes nothing; GELU scales element by element
    assert np.array_equal(orc.bwd_dx_act_panels(dys, ws, z, orc.ACT_NONE), dx)
    got = orc.bwd_dx_act_panels(dys, ws, z, orc.ACT_GELU_ERF)
    assert np.allclose(got, dx * orc.gelu_erf_grad(z), rtol=0, atol=1e-14)
    rows = np.array([4, 0, 2])
    assert np.array_equal(orc.bwd_dx_act_panels(dys, ws, z, orc.ACT_GELU_ERF, rows=rows), got[rows])
    # chain rule end to end: loss = sum(dOut * gelu(Z)) has dL/dZ = dOut * gelu'(Z);
    # with dOut = dX this is a directional derivative that central differences reproduce
    e = r.standard_normal((m, kb))
    h = 1e-6
    fd = (np.sum(dx * orc.gelu_erf(z + h * e)) - np.sum(dx * orc.gelu_erf(z - h * e))) / (2 * h)
    assert abs(fd - np.sum(got * e)) < 1e-7 * max(1.0, abs(fd))


def test_bias_gradient():
    q, m, n = 3, 4, 5
    r = _rng(22)
    dys = [r.standard_normal((m, n)) for _ in range(q)]
    db = orc.bias_grad_panels(dys)
    # brute force, one column at a time
    for s in range(n):
        tot = 0.0
        for t in range(q):
            for row in range(m):
                tot += dys[t][row, s]
        assert abs(db[s] - tot) < 1e-14
    # all-ones dY counts the rows; the grand total is the sum of everything
    ones = [np.ones((m, n)) for _ in range(q)]
    assert np.array_equal(orc.bias_grad_panels(ones), np.full(n, float(q * m)))
    assert abs(db.sum() - sum(p.sum() for p in dys)) < 1e-13
    # depth layers add up
    acc = np.zeros(n)
    orc.bias_grad_panels(dys, accumulate_into=acc)
    orc.bias_grad_panels(ones, accumulate_into=acc)
    assert np.allclose(acc, db + q * m, rtol=0, atol=1e-14)
    # it is the gradient of the bias: <db, e> equals the change of sum(dY * (Z + e)) along e,
    # which does not depend on Z
    e = r.standard_normal(n)
    assert abs(sum((p * e[None, :]).sum() for p in dys) - db @ e) < 1e-13


def test_bias_gradient_of_the_full_grid_is_the_column_sum_of_dy():
    """Row 0 of the grid ends up with the column sums of the unpartitioned dY, slice j:
    for every depth layer k the q panels are block rows t + k q of block column j."""
    q, d, m, n = 2, 2, 3, 4
    a, c = m * q * d, n * q
    dY = _rng(23).standard_normal((a, c))
    for j in range(q):
        acc = np.zeros(n)
        for k in range(d):
            panels = [np.ascontiguousarray(dY[(t + k * q) * m:(t + k * q + 1) * m, j * n:(j + 1) * n])
                      for t in range(q)]
            orc.bias_grad_panels(panels, accumulate_into=acc)
        assert np.allclose(acc, dY[:, j * n:(j + 1) * n].sum(axis=0), rtol=0, atol=1e-13)


# --------------------------------------- the backward as Section 3.1 words it, step by step
@pytest.mark.parametrize("q,d", [(2, 1), (2, 2), (3, 2)])
def test_stepwise_partials_reduce_to_the_owner_computes_sums(q, d):
    """Processor (i,j,k) multiplies ITS dY block by the block it receives at step t and the
    partials are reduced along the grid row (input gradient, owner (i,t,k)) or the grid column
    (weight gradient, owner (t,j,k)).  Written with the plain products on blocks of the global
    matrices, both reductions must give the blocks of dY W^T and, summed over depth, X^T dY."""
    a, b, c, m, kb, n = _sizes(q, d, 50 + q * 7 + d)
    r = _rng(60 + q + d)
    X, W, dY = r.standard_normal((a, b)), r.standard_normal((b, c)), r.standard_normal((a, c))
    dX_full, dW_full = dY @ W.T, X.T @ dY
    blkA = lambda M_, h, col, w_: np.ascontiguousarray(M_[h * m:(h + 1) * m, col * w_:(col + 1) * w_])
    blkW = lambda u, v: np.ascontiguousarray(W[u * kb:(u + 1) * kb, v * n:(v + 1) * n])
    dW_acc = np.zeros((b, c))
    for k in range(d):
        for i in range(q):
            h = orc.block_row(q, i, k)
            for t in range(q):
                # input gradient of block (h, t): sum over the row's processors j
                part = sum(orc.matmul_nt(blkA(dY, h, j, n), blkW(t, j)) for j in range(q))
                assert np.allclose(part, dX_full[h * m:(h + 1) * m, t * kb:(t + 1) * kb], atol=1e-12)
                # the same block from the owner-computes formula
                own = orc.tess_bwd_dx(q, d, i, t, k, dY, W)
                assert np.allclose(part, own, atol=1e-12)
        for j in range(q):
            for t in range(q):
                # weight gradient of block (t, j), depth layer k: sum over the column's processors i
                part = sum(orc.matmul_tn(blkA(X, orc.block_row(q, i, k), t, kb),
                                         blkA(dY, orc.block_row(q, i, k), j, n)) for i in range(q))
                dW_acc[t * kb:(t + 1) * kb, j * n:(j + 1) * n] += part
                assert np.allclose(part, orc.tess_bwd_dw(q, d, t, j, k, X, dY), atol=1e-12)
    assert np.allclose(dW_acc, dW_full, atol=1e-11)


# ----------------------------------------------- layer normalisation, local partial sums
def test_row_sums_and_layernorm_against_numpy():
    """Sums of q column blocks add up to the sums of the whole row, and normalising each block
    with the summed numbers is numpy's (x - mean) / sqrt(var + eps) on the whole row."""
    q, m, w = 3, 5, 4
    r = _rng(70)
    X = r.standard_normal((m, q * w)) * 3 + 1.5
    acc = np.zeros((m, 2))
    for j in range(q):
        orc.row_sums(np.ascontiguousarray(X[:, j * w:(j + 1) * w]), accumulate_into=acc)
    assert np.allclose(acc[:, 0], X.sum(axis=1), atol=1e-12)
    assert np.allclose(acc[:, 1], (X * X).sum(axis=1), atol=1e-11)
    one = orc.row_sums(np.ascontiguousarray(X[:, :w]))
    assert np.allclose(one[:, 0], X[:, :w].sum(axis=1), atol=1e-12)
    eps = 1e-5
    want = (X - X.mean(axis=1, keepdims=True)) / np.sqrt(X.var(axis=1, keepdims=True) + eps)
    for j in range(q):
        got = orc.layernorm_from_sums(np.ascontiguousarray(X[:, j * w:(j + 1) * w]), acc, q * w, eps)
        assert np.allclose(got, want[:, j * w:(j + 1) * w], atol=1e-12)
    # rows of the result have mean 0 and variance var / (var + eps)
    full = np.concatenate([orc.layernorm_from_sums(np.ascontiguousarray(X[:, j * w:(j + 1) * w]), acc,
                                                   q * w, eps) for j in range(q)], axis=1)
    assert np.allclose(full.mean(axis=1), 0.0, atol=1e-13)
    v = X.var(axis=1)
    assert np.allclose(full.var(axis=1), v / (v + eps), atol=1e-12)
    # a constant row has no variance: everything is (x - x) / sqrt(eps) = 0
    C = np.full((2, w), 7.0)
    assert np.array_equal(orc.layernorm_from_sums(C, orc.row_sums(C), w, eps), np.zeros((2, w)))
    # hand-computed: row (1, 2, 3, 6): sum 12, squares 50, mean 3, variance 50/4 - 9 = 3.5
    s = orc.row_sums(np.array([[1.0, 2.0, 3.0, 6.0]]))
    assert s.tolist() == [[12.0, 50.0]]
    got = orc.layernorm_from_sums(np.array([[1.0, 2.0, 3.0, 6.0]]), s, 4, 0.0)
    assert np.allclose(got, np.array([[-2.0, -1.0, 0.0, 3.0]]) / np.sqrt(3.5), atol=1e-15)


def test_layernorm_variance_is_never_negative():
    """Var[X] = E[X^2] - E[X]^2 (Section 3.2, "Other procedure") is a variance: where the
    difference of the two moments rounds below zero it is taken as zero.  Sums whose
    difference is slightly negative must give the result of a zero variance, not the NaN
    of a negative one (eps smaller than the deficit)."""
    x = np.array([[3.0, 3.0, 3.0, 3.0 + 1e-3]])
    sums = np.array([[12.0 + 1e-3, 36.0 - 1e-3]])       # sum of squares too small by more than eps * n
    out = orc.layernorm_from_sums(x, sums, 4, 1e-9)
    assert np.isfinite(out).all()
    mean = (12.0 + 1e-3) / 4
    assert np.allclose(out, (x - mean) / np.sqrt(1e-9), rtol=1e-12)


def test_layernorm_backward_against_central_differences():
    """X' of the paper's formula is the gradient of J = sum(c * xhat(X)) for fixed weights c
    (so dJ/dxhat = c): central differences of the oracle's own forward, element by element,
    with the hidden dimension spread over q blocks."""
    q, m, w = 2, 3, 4
    n, eps = q * w, 1e-3
    r = _rng(71)
    X = r.standard_normal((m, n)) * 2 + 0.5
    C = r.standard_normal((m, n))

    def forward(Xm):
        s = np.zeros((m, 2))
        for j in range(q):
            orc.row_sums(np.ascontiguousarray(Xm[:, j * w:(j + 1) * w]), accumulate_into=s)
        xh = np.concatenate([orc.layernorm_from_sums(np.ascontiguousarray(Xm[:, j * w:(j + 1) * w]), s, n, eps)
                             for j in range(q)], axis=1)
        return xh, s

    xhat, s_fwd = forward(X)
    s_bwd = np.zeros((m, 2))
    for j in range(q):
        orc.row_sums_bwd(np.ascontiguousarray(xhat[:, j * w:(j + 1) * w]),
                         np.ascontiguousarray(C[:, j * w:(j + 1) * w]), accumulate_into=s_bwd)
    assert np.allclose(s_bwd[:, 0], (xhat * C).sum(axis=1), atol=1e-13)
    assert np.allclose(s_bwd[:, 1], C.sum(axis=1), atol=1e-13)
    got = np.concatenate([orc.layernorm_bwd_from_sums(np.ascontiguousarray(xhat[:, j * w:(j + 1) * w]),
                                                      np.ascontiguousarray(C[:, j * w:(j + 1) * w]),
                                                      s_bwd, s_fwd, n, eps) for j in range(q)], axis=1)
    h = 1e-6
    for rr in range(m):
        for u in range(n):
            Xp, Xm = X.copy(), X.copy()
            Xp[rr, u] += h
            Xm[rr, u] -= h
            fd = (np.sum(C * forward(Xp)[0]) - np.sum(C * forward(Xm)[0])) / (2 * h)
            assert abs(fd - got[rr, u]) < 1e-7, (rr, u)
    # the gradient is orthogonal to the all-ones direction (shifting a row changes nothing)
    assert np.allclose(got.sum(axis=1), 0.0, atol=1e-12)
