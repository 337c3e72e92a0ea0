"""GPU parity of the local layer-normalisation parts (Section 3.2, "Other procedure"): per-row
sum and sum of squares of one processor's block, accumulated over the q blocks of a grid row
on one GPU, and the normalisation from the reduced sums; against the fp64 oracle."""
import numpy as np
import pytest
import torch

from paper_2105_14500_amd import binding as B
from oracle import tess_oracle as orc
from gpu_util import TOL, f64, dev, rel_err, tdtype

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("q,m,w", [(1, 7, 33), (2, 5, 8), (4, 256, 1024), (3, 130, 72), (8, 1024, 1536)])
def test_row_sums_and_normalize(dtype, q, m, w):
    g = torch.Generator().manual_seed(5 + q + m)
    X = (torch.randn((m, q * w), generator=g) * 3 + 1.5).to(tdtype(dtype))     # the whole rows
    Xd = dev(X)
    sums = torch.full((m, 2), float("nan"), device="cuda:0")
    for j in range(q):                                   # strided column blocks, ld = q*w
        B.layernorm_row_sums(Xd[:, j * w:(j + 1) * w], sums, accumulate=(j > 0))
    eps = 1e-5
    out = torch.full((m, q * w), float("nan"), dtype=tdtype(dtype), device="cuda:0")
    for j in range(q):
        B.layernorm_normalize(Xd[:, j * w:(j + 1) * w], sums, q * w, eps, out[:, j * w:(j + 1) * w])
    torch.cuda.synchronize()
    X64 = f64(X)
    want_s = np.zeros((m, 2))
    for j in range(q):
        orc.row_sums(np.ascontiguousarray(X64[:, j * w:(j + 1) * w]), accumulate_into=want_s)
    assert rel_err(sums, want_s) <= 1e-5
    want = np.concatenate([orc.layernorm_from_sums(np.ascontiguousarray(X64[:, j * w:(j + 1) * w]),
                                                   want_s, q * w, eps) for j in range(q)], axis=1)
    assert rel_err(out, want) <= (TOL["bf16"] if dtype == "bf16" else 1e-5)
    assert not torch.isnan(out).any()


def test_constant_rows_with_a_large_mean_stay_finite():
    """Rows whose mean dwarfs their spread: in fp32 the difference of the two moments can
    round below zero by more than eps, and an unclamped variance would then give NaN.  A
    constant row has variance 0: its normalised values are exactly 0."""
    m, w = 16, 512
    X = torch.full((m, w), 1000.0, dtype=torch.float32)
    X[8:] += torch.arange(w, dtype=torch.float32)[None, :] * 1e-3        # tiny spread on half the rows
    Xd = dev(X)
    sums = torch.empty((m, 2), device="cuda:0")
    B.layernorm_row_sums(Xd, sums)
    for eps in (1e-5, 1e-12):
        out = torch.full((m, w), float("nan"), device="cuda:0")
        B.layernorm_normalize(Xd, sums, w, eps, out)
        torch.cuda.synchronize()
        assert torch.isfinite(out).all()
        assert torch.all(out[:8] == 0.0)
    want = orc.layernorm_from_sums(f64(X[:8]), orc.row_sums(f64(X[:8])), w, 1e-5)
    assert np.all(want == 0.0)


def test_row_sums_of_integers_are_exact_and_errors_are_reported():
    m, w = 64, 520
    r = np.random.default_rng(3)
    X = torch.tensor(r.integers(-3, 4, size=(m, w)).astype(np.float32)).to(torch.bfloat16)
    sums = torch.empty((m, 2), device="cuda:0")
    B.layernorm_row_sums(dev(X), sums)
    torch.cuda.synchronize()
    assert np.array_equal(f64(sums), orc.row_sums(f64(X)))
    L = B.lib()
    assert L.tess_layernorm_row_sums(None, 4, 4, 4, B.BF16, None, 0, None) == 1
    assert L.tess_layernorm_row_sums(sums.data_ptr(), 4, 8, 4, B.BF16, sums.data_ptr(), 0, None) == 3
    assert L.tess_layernorm_normalize(sums.data_ptr(), 4, 8, 8, 7, sums.data_ptr(), 8, 1e-5,
                                      sums.data_ptr(), 8, None) == 5


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("q,m,w", [(1, 7, 33), (2, 5, 8), (4, 256, 1024), (3, 130, 72)])
def test_backward_row_sums_and_apply(dtype, q, m, w):
    """The backward of the normalisation on the q column blocks of whole rows: partial sums
    accumulated over the blocks, then X' per block, against the fp64 oracle."""
    g_ = torch.Generator().manual_seed(15 + q + m)
    X = (torch.randn((m, q * w), generator=g_) * 2 + 0.5).to(tdtype(dtype))
    G = torch.randn((m, q * w), generator=g_).to(tdtype(dtype))
    n, eps = q * w, 1e-5
    Xd, Gd = dev(X), dev(G)
    s_fwd = torch.empty((m, 2), device="cuda:0")
    for j in range(q):
        B.layernorm_row_sums(Xd[:, j * w:(j + 1) * w], s_fwd, accumulate=(j > 0))
    xhat = torch.empty_like(Xd)
    for j in range(q):
        B.layernorm_normalize(Xd[:, j * w:(j + 1) * w], s_fwd, n, eps, xhat[:, j * w:(j + 1) * w])
    s_bwd = torch.full((m, 2), float("nan"), device="cuda:0")
    for j in range(q):
        B.layernorm_bwd_row_sums(xhat[:, j * w:(j + 1) * w], Gd[:, j * w:(j + 1) * w], s_bwd,
                                 accumulate=(j > 0))
    dx = torch.full((m, n), float("nan"), dtype=tdtype(dtype), device="cuda:0")
    for j in range(q):
        B.layernorm_bwd_apply(xhat[:, j * w:(j + 1) * w], Gd[:, j * w:(j + 1) * w], s_bwd, s_fwd, n, eps,
                              dx[:, j * w:(j + 1) * w])
    torch.cuda.synchronize()
    # the oracle takes the GPU-independent inputs: X, G, and ITS OWN forward
    X64, G64 = f64(X), f64(G)
    blk = lambda M_, j: np.ascontiguousarray(M_[:, j * w:(j + 1) * w])
    sf = np.zeros((m, 2))
    for j in range(q):
        orc.row_sums(blk(X64, j), accumulate_into=sf)
    xh = np.concatenate([orc.layernorm_from_sums(blk(X64, j), sf, n, eps) for j in range(q)], axis=1)
    sb = np.zeros((m, 2))
    for j in range(q):
        orc.row_sums_bwd(blk(xh, j), blk(G64, j), accumulate_into=sb)
    want = np.concatenate([orc.layernorm_bwd_from_sums(blk(xh, j), blk(G64, j), sb, sf, n, eps)
                           for j in range(q)], axis=1)
    tol = TOL["bf16"] if dtype == "bf16" else 1e-4
    assert rel_err(s_bwd, sb) <= tol          # xhat is rounded to the storage dtype on the GPU
    assert rel_err(dx, want) <= tol
    assert not torch.isnan(dx).any()


def test_in_place_variants():
    """xhat_out may be x itself and dx_out may be g itself (each element is read once, by the lane
    that overwrites it)."""
    m, w, eps = 96, 520, 1e-5
    g_ = torch.Generator().manual_seed(9)
    X = (torch.randn((m, w), generator=g_) * 2 + 1).to(torch.bfloat16)
    G = torch.randn((m, w), generator=g_).to(torch.bfloat16)
    Xd, Gd = dev(X), dev(G)
    s_fwd = torch.empty((m, 2), device="cuda:0")
    B.layernorm_row_sums(Xd, s_fwd)
    out = torch.empty_like(Xd)
    B.layernorm_normalize(Xd, s_fwd, w, eps, out)
    inplace = Xd.clone()
    B.layernorm_normalize(inplace, s_fwd, w, eps, inplace)
    s_bwd = torch.empty((m, 2), device="cuda:0")
    B.layernorm_bwd_row_sums(out, Gd, s_bwd)
    dx = torch.empty_like(Gd)
    B.layernorm_bwd_apply(out, Gd, s_bwd, s_fwd, w, eps, dx)
    g_inplace = Gd.clone()
    B.layernorm_bwd_apply(out, g_inplace, s_bwd, s_fwd, w, eps, g_inplace)
    torch.cuda.synchronize()
    assert torch.equal(inplace, out) and torch.equal(g_inplace, dx)
