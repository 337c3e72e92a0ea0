"""One processor's MLP as a chain of library calls (up-projection with bias and GELU, its
pre-activation kept; down-projection; then the backward through both, with the GELU
derivative fused into the down-projection's input gradient and the bias gradients fused
into the weight-gradient calls) against the same chain written with the fp64 oracle.
The intermediates H and dZ1 are bf16 on the GPU and fp64 in the oracle, so every output is
compared at the bf16 bound."""
import numpy as np
import pytest
import torch

from paper_2105_14500_amd import binding as B
from paper_2105_14500_amd.mlp import MlpShare
from oracle import tess_oracle as orc
from gpu_util import TOL, f64, dev, rel_err

pytestmark = pytest.mark.gpu


def _panels(gen, q, r, c, std):
    return [(torch.randn((r, c), generator=gen) * std).to(torch.bfloat16) for _ in range(q)]


@pytest.mark.parametrize("q,d,m,h_q,f_q,own", [(2, 2, 128, 64, 256, 0), (3, 1, 192, 128, 512, 2),
                                               (2, 1, 256, 256, 1024, 1)])
def test_mlp_chain_matches_oracle_chain(q, d, m, h_q, f_q, own):
    g = torch.Generator().manual_seed(77)
    x = _panels(g, q, m, h_q, 1.0)
    w1 = _panels(g, q, h_q, f_q, 0.05)          # column block j of W1 (forward operand)
    w1t = _panels(g, q, h_q, f_q, 0.05)         # row block of W1 (dX operand)
    w2 = _panels(g, q, f_q, h_q, 0.05)
    w2t = _panels(g, q, f_q, h_q, 0.05)
    b1 = (torch.randn((f_q,), generator=g) * 0.1).to(torch.bfloat16)
    b2 = (torch.randn((h_q,), generator=g) * 0.1).to(torch.bfloat16)
    h_in = _panels(g, q, m, f_q, 0.5)           # peers' blocks of H (slot `own` is replaced)
    dy = _panels(g, q, m, h_q, 1.0)
    dz_in = _panels(g, q, m, f_q, 0.5)          # peers' blocks of dZ1

    mlp = MlpShare(q, d, m, h_q, f_q, act=B.ACT_GELU_ERF, own=own)
    D = lambda ps: [dev(p) for p in ps]
    xd, hd, dyd, dzd = D(x), D(h_in), D(dy), D(dz_in)
    y = mlp.forward(xd, D(w1), dev(b1), hd, D(w2), dev(b2))
    dx = mlp.backward(xd, D(w1t), hd, D(w2t), dyd, dzd, accumulate=False)
    torch.cuda.synchronize()

    F = lambda ps: [f64(p) for p in ps]
    h, z1 = orc.fwd_panels(F(x), F(w1), bias=f64(b1), act=orc.ACT_GELU_ERF, want_z=True)
    hp = F(h_in); hp[own] = h
    y_o = orc.fwd_panels(hp, F(w2), bias=f64(b2))
    dw2_o = orc.bwd_dw_panels(hp, F(dy))
    db2_o = orc.bias_grad_panels(F(dy))
    dz1 = orc.bwd_dx_act_panels(F(dy), F(w2t), z1, orc.ACT_GELU_ERF)
    dzp = F(dz_in); dzp[own] = dz1
    dw1_o = orc.bwd_dw_panels(F(x), dzp)
    db1_o = orc.bias_grad_panels(dzp)
    dx_o = orc.bwd_dx_panels(dzp, F(w1t))

    tol = TOL["bf16"]
    errs = {"z1": rel_err(mlp.z1, z1), "h": rel_err(mlp.h, h), "y": rel_err(y, y_o),
            "dz1": rel_err(mlp.dz1, dz1), "dx": rel_err(dx, dx_o),
            "dw2": rel_err(mlp.dw2, dw2_o), "db2": rel_err(mlp.db2, db2_o),
            "dw1": rel_err(mlp.dw1, dw1_o), "db1": rel_err(mlp.db1, db1_o)}
    assert all(e <= tol for e in errs.values()), errs
    # the caller's panel lists are left as they were
    assert hd[own] is not mlp.h and dzd[own] is not mlp.dz1
