"""Seeded synthetic inputs and the workload table for the Tesseract linear hot path.

This module serves both the HIP path and the CPU oracle and therefore holds
none of the method's arithmetic: it only names the benchmark configurations
(grid [q,q,d], global layer sizes, the per-processor block shapes they imply,
dtype, epilogue) and draws random matrices.  The paper itself checks the method
on randomly generated matrices (Experiment section); the distributions here
are N(0,1) activations and output gradients and N(0,0.02) weights and biases.

Draw order per generator call (CPU torch.Generator, fp32, then cast): X, W,
bias, dY.  One processor's share of an i.i.d. matrix is again i.i.d., so the
one-share generators draw the q panels of each operand directly at the block
shape instead of slicing a global matrix.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import torch


@dataclass(frozen=True)
class Layer:
    """One linear layer of a workload: global sizes A[a,b], B[b,c], C[a,c]."""
    name: str
    a: int
    b: int
    c: int
    m: int          # rows per block     = a / (q d)
    kb: int         # block width of A   = b / q
    n: int          # block width of B,C = c / q
    act: str        # "none" | "gelu_erf"
    bias_std: float  # 0.0 -> zero bias


@dataclass(frozen=True)
class Workload:
    name: str
    q: int
    d: int
    dtype: str      # "f32" | "bf16"
    mode: str       # "full_grid" | "one_share"
    layers: List[Layer] = field(default_factory=list)


WORKLOADS = [
    Workload("cfg1_q2d1_f32_fullgrid", 2, 1, "f32", "full_grid",
             [Layer("linear", 256, 256, 1024, 128, 128, 512, "none", 0.0)]),
    Workload("cfg2_q2d2_bf16_mlp_up_h1024", 2, 2, "bf16", "one_share",
             [Layer("up", 8192, 1024, 4096, 2048, 512, 2048, "gelu_erf", 0.02)]),
    Workload("cfg3_q4d2_bf16_mlp_h4096", 4, 2, "bf16", "one_share",
             [Layer("up", 32768, 4096, 16384, 4096, 1024, 4096, "gelu_erf", 0.02),
              Layer("down", 32768, 16384, 4096, 4096, 4096, 1024, "none", 0.0)]),
    Workload("cfg4_q4d4_bf16_attn_h8192", 4, 4, "bf16", "one_share",
             [Layer("qkv", 131072, 8192, 24576, 8192, 2048, 6144, "none", 0.0),
              Layer("out", 131072, 8192, 8192, 8192, 2048, 2048, "none", 0.0)]),
    Workload("cfg5_q8d2_bf16_mlp_h12288", 8, 2, "bf16", "one_share",
             [Layer("up", 32768, 12288, 49152, 2048, 1536, 6144, "gelu_erf", 0.02),
              Layer("down", 32768, 49152, 12288, 2048, 6144, 1536, "none", 0.0)]),
]


# The grids and Transformer sizes of the paper's own experiments (Tables 1 and 2: GPU shape,
# batch size, hidden size), turned into per-processor block shapes.  The paper gives no
# sequence length: SEQ_LEN is this build's choice.  Table 2's batch sizes give b/(dq) = 48
# sequences per processor (its text says 24; the table is followed).  Four linear layers per
# Transformer layer (Section 3.2): QKV h -> 3h, attention output h -> h, MLP h -> 4h -> h.
SEQ_LEN = 512
PAPER_TABLE_GRIDS = [
    # (table, q, d, batch, hidden)
    ("strong", 2, 1, 12, 3072), ("strong", 2, 2, 12, 3072), ("strong", 4, 1, 12, 3072),
    ("strong", 4, 2, 12, 3072), ("strong", 4, 4, 16, 3072), ("strong", 8, 1, 12, 3072),
    ("weak", 1, 1, 48, 1024), ("weak", 2, 1, 96, 2048), ("weak", 2, 2, 192, 2048),
    ("weak", 4, 1, 192, 4096), ("weak", 4, 2, 384, 4096), ("weak", 4, 4, 768, 4096),
    ("weak", 8, 1, 384, 8192),
]


def _transformer_layers(q, d, batch, h):
    a = batch * SEQ_LEN
    spec = [("qkv", h, 3 * h, "none", 0.02), ("out", h, h, "none", 0.02),
            ("up", h, 4 * h, "gelu_erf", 0.02), ("down", 4 * h, h, "none", 0.02)]
    return [Layer(name, a, b, c, a // (q * d), b // q, c // q, act, bstd)
            for name, b, c, act, bstd in spec]


PAPER_TABLE_WORKLOADS = [
    Workload(f"{table}_q{q}d{d}_b{batch}_h{h}", q, d, "bf16", "one_share",
             _transformer_layers(q, d, batch, h))
    for table, q, d, batch, h in PAPER_TABLE_GRIDS
]


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def _normal(g, shape, std, dtype):
    if std == 0.0:
        return torch.zeros(shape, dtype=dtype)
    x = torch.randn(shape, generator=g, dtype=torch.float32)
    if std != 1.0:
        x = x * std
    return x.to(dtype)


def _small_ints(g, shape, dtype, lo=-2, hi=2):
    return torch.randint(lo, hi + 1, shape, generator=g).to(dtype)


def full_grid_inputs(a, b, c, dtype="f32", seed=0, bias_std=0.0, w_std=0.02, integers=False):
    """Global X[a,b], W[b,c], bias[c], dY[a,c] on the CPU."""
    g = _gen(seed)
    dt = torch_dtype(dtype)
    if integers:
        return (_small_ints(g, (a, b), dt), _small_ints(g, (b, c), dt),
                _small_ints(g, (c,), dt), _small_ints(g, (a, c), dt))
    X = _normal(g, (a, b), 1.0, dt)
    W = _normal(g, (b, c), w_std, dt)
    bias = _normal(g, (c,), bias_std, dt)
    dY = _normal(g, (a, c), 1.0, dt)
    return X, W, bias, dY


def share_inputs(q, m, kb, n, dtype="bf16", seed=0, bias_std=0.02, w_std=0.02, integers=False,
                 want=("x", "w", "bias", "dy")):
    """One processor's panels at the block shape: q X-panels [m,kb], q W-panels
    [kb,n], a bias slice [n], q dY-panels [m,n].  The forward uses (X, W, bias),
    the input gradient (dY, W), the weight gradient (X, dY).  Each operand is one
    packed [q, rows, cols] tensor; panel t is operand[t]."""
    g = _gen(seed)
    dt = torch_dtype(dtype)
    out = {}
    if integers:
        out["x"] = _small_ints(g, (q, m, kb), dt)
        out["w"] = _small_ints(g, (q, kb, n), dt)
        out["bias"] = _small_ints(g, (n,), dt)
        out["dy"] = _small_ints(g, (q, m, n), dt)
        return out
    # operands a caller does not want are not drawn; later operands then come
    # from another position of the same seeded stream, still i.i.d.
    out["x"] = _normal(g, (q, m, kb), 1.0, dt) if "x" in want else None
    out["w"] = _normal(g, (q, kb, n), w_std, dt) if "w" in want else None
    out["bias"] = _normal(g, (n,), bias_std, dt) if "bias" in want else None
    out["dy"] = _normal(g, (q, m, n), 1.0, dt) if "dy" in want else None
    return out


def workload_by_name(name: str) -> Optional[Workload]:
    for w in WORKLOADS + PAPER_TABLE_WORKLOADS:
        if w.name == name:
            return w
    return None
