"""Helpers shared by the GPU parity tests: run the HIP library through its C ABI
binding and compare with the CPU fp64 oracle on the same seeded inputs."""
import numpy as np
import torch

import paper_2105_14500_amd as tess
from paper_2105_14500_amd import binding as B
from oracle import tess_oracle as orc

TOL = {"f32": 1e-5, "bf16": 2e-2}     # relative Frobenius bounds of the north-star
ACT = {"none": B.ACT_NONE, "gelu_erf": B.ACT_GELU_ERF, "gelu_tanh": B.ACT_GELU_TANH}
ORC_ACT = {"none": orc.ACT_NONE, "gelu_erf": orc.ACT_GELU_ERF, "gelu_tanh": orc.ACT_GELU_TANH}


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def dev(t):
    return t.to("cuda:0")


def workspace(desc, op):
    nbytes = tess.workspace_bytes(desc, op)
    if nbytes == 0:
        return None
    return torch.empty(nbytes // 4, dtype=torch.float32, device="cuda:0")


def code(dtype_name):
    return {"f32": B.F32, "bf16": B.BF16}[dtype_name]


def tdtype(dtype_name):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype_name]


def share_desc(q, d, m, kb, n, in_dtype, out_dtype):
    """Descriptor of processor (0,0,0) for block shape (m, kb, n)."""
    return B.make_desc(q, d, 0, 0, 0, m * q * d, kb * q, n * q, code(in_dtype), code(out_dtype))


def run_share(q, d, x, w, bias, dy, in_dtype, out_dtype, act="none", want_preact=False,
              dw_accumulate_into=None):
    """One processor's fwd, dX and dW on packed panels x[q,m,kb], w[q,kb,n], dy[q,m,n]
    (CPU tensors).  Returns device results as CPU tensors."""
    _, m, kb = x.shape
    n = w.shape[2]
    desc = share_desc(q, d, m, kb, n, in_dtype, out_dtype)
    xd, wd, dyd = dev(x), dev(w), dev(dy)
    bd = dev(bias) if bias is not None else None
    odt = tdtype(out_dtype)
    y = torch.full((m, n), float("nan"), dtype=odt, device="cuda:0")
    pre = torch.full((m, n), float("nan"), dtype=odt, device="cuda:0") if want_preact else None
    tess.linear_fwd(desc, list(xd), list(wd), bd, ACT[act], y, preact_out=pre,
                    workspace=workspace(desc, B.OP_FWD))
    dx = torch.full((m, kb), float("nan"), dtype=odt, device="cuda:0")
    tess.linear_bwd_dx(desc, list(dyd), list(wd), dx, workspace=workspace(desc, B.OP_BWD_DX))
    if dw_accumulate_into is not None:
        dw = dw_accumulate_into
        tess.linear_bwd_dw(desc, list(xd), list(dyd), dw, accumulate=True,
                           workspace=workspace(desc, B.OP_BWD_DW))
    else:
        dw = torch.full((kb, n), float("nan"), dtype=odt, device="cuda:0")
        tess.linear_bwd_dw(desc, list(xd), list(dyd), dw, workspace=workspace(desc, B.OP_BWD_DW))
    torch.cuda.synchronize()
    out = {"y": y.cpu(), "dx": dx.cpu(), "dw": dw.cpu() if dw_accumulate_into is None else dw}
    if want_preact:
        out["preact"] = pre.cpu()
    return out


def oracle_share(x, w, bias, dy, act="none"):
    """Oracle results for the same packed panels (full outputs)."""
    q = x.shape[0]
    xs = [f64(x[t]) for t in range(q)]
    ws = [f64(w[t]) for t in range(q)]
    dys = [f64(dy[t]) for t in range(q)]
    b64 = f64(bias) if bias is not None else None
    y, z = orc.fwd_panels(xs, ws, bias=b64, act=ORC_ACT[act], want_z=True)
    return {"y": y, "preact": z, "dx": orc.bwd_dx_panels(dys, ws), "dw": orc.bwd_dw_panels(xs, dys)}


def rel_err(got, want):
    return orc.rel_frobenius(f64(got) if isinstance(got, torch.Tensor) else got, want)
