"""Host-only: which kernel variant each shape of the GPU suite takes.  The launch plan is
pure host arithmetic (tess_linear_plan), so this runs without a GPU and fails when a
retuned cost model silently moves the GPU tests off a code path: every combination of
{256 x 256 direct, 128 x 128 direct, 128 x 128 register-staged} x {no K split, K split} x
{forward, input gradient, weight gradient} must be taken by at least one GPU test shape."""
import itertools

import tess_workloads as wl
from paper_2105_14500_amd import binding as B

import test_gpu_configs
import test_gpu_parity
import test_gpu_tile_grids


def _variants(q, d, m, kb, n):
    desc = B.make_desc(q, d, 0, 0, 0, m * q * d, kb * q, n * q, B.BF16, B.BF16)
    out = []
    for op, name, kp in ((B.OP_FWD, "fwd", kb), (B.OP_BWD_DX, "dx", n), (B.OP_BWD_DW, "dw", m)):
        tile, _, splits = B.plan(desc, op)
        if tile:
            out.append(((tile, "direct" if kp % 64 == 0 else "staged"), "split" if splits > 1 else "whole", name))
    return out


def test_gpu_suite_reaches_every_kernel_variant():
    seen = {}
    for q, d, m, kb, n, dtype in test_gpu_parity.SHAPES:
        if dtype == "bf16":
            for v in _variants(q, d, m, kb, n):
                seen.setdefault(v, ("test_gpu_parity.SHAPES", (q, d, m, kb, n)))
    for wname, lname in test_gpu_configs.CASES:
        w = wl.workload_by_name(wname)
        L = next(l for l in w.layers if l.name == lname)
        for v in _variants(w.q, w.d, L.m, L.kb, L.n):
            seen.setdefault(v, ("test_gpu_configs.CASES", (wname, lname)))
    try:
        for tile, splits, (q, d, m, kb, n) in test_gpu_parity.FORCED:
            B.set_plan_override(tile=tile, k_splits=splits)
            for v in _variants(q, d, m, kb, n):
                assert v[0][0] == tile and (v[1] == "split") == (splits > 1)
                seen.setdefault(v, ("test_gpu_parity.FORCED", (tile, splits, q, d, m, kb, n)))
    finally:
        B.set_plan_override(0, 0)
    want = set(itertools.product([(256, "direct"), (128, "direct"), (128, "staged")], ["whole", "split"],
                                 ["fwd", "dx", "dw"]))
    missing = sorted(want - set(seen))
    assert not missing, missing


def test_full_size_plans_of_the_configurations_match_the_exact_grid_tests():
    """The whole-output exact tests force the K-split count that the full-size call of the
    same output shape takes; if the cost model changes that count, this says which."""
    planned = set()
    for w in wl.WORKLOADS:
        if w.dtype != "bf16" or w.name.startswith("cfg2"):
            continue
        for L in w.layers:
            desc = B.make_desc(w.q, w.d, 0, 0, 0, L.a, L.b, L.c, B.BF16, B.BF16)
            for op, name, (M, N) in ((B.OP_FWD, "fwd", (L.m, L.n)), (B.OP_BWD_DX, "dx", (L.m, L.kb)),
                                     (B.OP_BWD_DW, "dw", (L.kb, L.n))):
                tile, _, splits = B.plan(desc, op)
                assert tile == 256
                planned.add((name, w.q, M, N, splits))
    assert planned == set(test_gpu_tile_grids.GRIDS), sorted(planned ^ set(test_gpu_tile_grids.GRIDS))
