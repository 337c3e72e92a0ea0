"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before any HIP call (so this runs on
a machine without a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2105_14500_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    for header in ("tesseract.h", "tesseract_diag.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(tess_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = _declared_symbols()
    assert set(B.EXPORTS) == set(names)
    for name in names:
        assert getattr(L, name) is not None


def test_version_and_status_strings():
    assert re.match(r"^\d+\.\d+$", B.version())
    assert B.status_string(0) == "TESS_OK"
    assert B.status_string(2) == "TESS_ERR_GRID"
    assert B.status_string(99).startswith("TESS_ERR")


def test_descriptor_rules():
    ok = B.make_desc(2, 2, 1, 1, 1, 8, 4, 6)
    assert B.desc_check(ok) == 0
    assert B.block_shape(ok) == (2, 2, 3)
    assert B.desc_check(B.make_desc(2, 3, 0, 0, 0, 12, 4, 6)) == 2      # d > q
    assert B.desc_check(B.make_desc(0, 1, 0, 0, 0, 8, 4, 6)) == 2
    assert B.desc_check(B.make_desc(17, 1, 0, 0, 0, 17, 17, 17)) == 2   # q > TESS_MAX_Q
    assert B.desc_check(B.make_desc(2, 2, 2, 0, 0, 8, 4, 6)) == 2       # i outside
    assert B.desc_check(B.make_desc(2, 2, 0, 0, 2, 8, 4, 6)) == 2       # k outside
    assert B.desc_check(B.make_desc(2, 2, 0, 0, 0, 6, 4, 6)) == 3       # a % (q d)
    assert B.desc_check(B.make_desc(2, 2, 0, 0, 0, 8, 3, 6)) == 3
    assert B.desc_check(B.make_desc(2, 2, 0, 0, 0, 8, 4, 5)) == 3
    assert B.desc_check(B.make_desc(2, 2, 0, 0, 0, 8, 4, 6, 5, 0)) == 5  # dtype
    assert B.lib().tess_desc_check(None) == 1


def test_entry_points_validate_before_touching_the_gpu():
    """Bad arguments must come back as status codes without a GPU present."""
    L = B.lib()
    d = B.make_desc(2, 2, 0, 0, 0, 8, 4, 6)
    fake = ctypes.c_void_p(0x1000)        # never dereferenced: validation fails first
    two = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    holes = (ctypes.c_void_p * 2)(0x1000, None)
    ref = ctypes.byref
    # null descriptor / panel arrays / a hole in the panel array / null output
    assert L.tess_linear_fwd(None, two, 2, two, 3, None, 0, fake, 3, None, None, 0, None) == 1
    assert L.tess_linear_fwd(ref(d), None, 2, two, 3, None, 0, fake, 3, None, None, 0, None) == 1
    assert L.tess_linear_fwd(ref(d), holes, 2, two, 3, None, 0, fake, 3, None, None, 0, None) == 1
    assert L.tess_linear_fwd(ref(d), two, 2, two, 3, None, 0, None, 3, None, None, 0, None) == 1
    # leading dimensions shorter than a row
    assert L.tess_linear_fwd(ref(d), two, 1, two, 3, None, 0, fake, 3, None, None, 0, None) == 3
    assert L.tess_linear_fwd(ref(d), two, 2, two, 2, None, 0, fake, 3, None, None, 0, None) == 3
    assert L.tess_linear_fwd(ref(d), two, 2, two, 3, None, 0, fake, 2, None, None, 0, None) == 3
    # unknown activation
    assert L.tess_linear_fwd(ref(d), two, 2, two, 3, None, 9, fake, 3, None, None, 0, None) == 5
    # dX / dW
    assert L.tess_linear_bwd_dx(ref(d), two, 2, two, 3, fake, 2, None, 0, None) == 3   # lddy < n
    assert L.tess_linear_bwd_dx(ref(d), two, 3, two, 3, None, 2, None, 0, None) == 1
    assert L.tess_linear_bwd_dw(ref(d), two, 2, two, 3, fake, 3, 2, None, 0, None) == 5  # accumulate
    assert L.tess_linear_bwd_dw(ref(d), two, 1, two, 3, fake, 3, 0, None, 0, None) == 3
    bad = B.make_desc(2, 3, 0, 0, 0, 12, 4, 6)
    assert L.tess_linear_bwd_dw(ref(bad), two, 2, two, 3, fake, 3, 0, None, 0, None) == 2


def test_workspace_query_and_enforcement():
    # a long-K, small-output bf16 problem needs split-K scratch
    d = B.make_desc(8, 2, 0, 0, 0, 2048 * 16, 6144 * 8, 1536 * 8, B.BF16, B.BF16)
    need = B.workspace_bytes(d, B.OP_FWD)
    assert need > 0 and need % 4 == 0
    assert B.workspace_bytes(d, 7) == 0
    # fp32 problems use the plain kernel: no scratch
    d32 = B.make_desc(2, 1, 0, 0, 0, 256, 256, 1024, B.F32, B.F32)
    assert [B.workspace_bytes(d32, op) for op in (0, 1, 2)] == [0, 0, 0]
    L = B.lib()
    q = 8
    arr = (ctypes.c_void_p * q)(*[0x10000 * (t + 1) for t in range(q)])
    fake = ctypes.c_void_p(0x1000)
    st = L.tess_linear_fwd(ctypes.byref(d), arr, 6144, arr, 1536, None, 0, fake, 1536, None,
                           None, 0, None)
    assert st == 6
    st = L.tess_linear_fwd(ctypes.byref(d), arr, 6144, arr, 1536, None, 0, fake, 1536, None,
                           ctypes.c_void_p(0x100000), need - 1, None)
    assert st == 6


def test_misaligned_bf16_operands_are_refused_not_rerouted():
    """A bf16 block whose shape selects the matrix-core kernel must not drop silently to the
    plain fp32 kernel when a pointer or a leading dimension is misaligned."""
    L = B.lib()
    d = B.make_desc(2, 2, 0, 0, 0, 64 * 4, 64 * 2, 64 * 2, B.BF16, B.BF16)
    assert B.plan(d, B.OP_FWD)[0] > 0
    ok = (ctypes.c_void_p * 2)(0x10000, 0x20000)
    odd = (ctypes.c_void_p * 2)(0x10000, 0x20008)          # second panel 8-byte aligned only
    out = ctypes.c_void_p(0x90000)
    ref = ctypes.byref
    assert L.tess_linear_fwd(ref(d), odd, 64, ok, 64, None, 0, out, 64, None, None, 0, None) == 4
    assert L.tess_linear_fwd(ref(d), ok, 64, odd, 64, None, 0, out, 64, None, None, 0, None) == 4
    assert L.tess_linear_fwd(ref(d), ok, 68, ok, 64, None, 0, out, 64, None, None, 0, None) == 4   # lda % 8
    assert L.tess_linear_bwd_dx(ref(d), ok, 64, odd, 64, out, 64, None, 0, None) == 4
    assert L.tess_linear_bwd_dw(ref(d), odd, 64, ok, 64, out, 64, 0, None, 0, None) == 4
    assert B.status_string(4) == "TESS_ERR_ALIGN"
    # a block whose extents are no multiple of 8 is planned for the plain kernel (tile 0 x 0),
    # which takes any alignment: the plan says so up front
    ragged = B.make_desc(2, 2, 0, 0, 0, 33 * 4, 17 * 2, 29 * 2, B.BF16, B.BF16)
    assert B.plan(ragged, B.OP_FWD) == (0, 0, 1) and B.plan(ragged, B.OP_BWD_DW) == (0, 0, 1)
    f32 = B.make_desc(2, 1, 0, 0, 0, 256, 256, 1024, B.F32, B.F32)
    assert B.plan(f32, B.OP_FWD) == (0, 0, 1)


def test_plan_override_is_explicit_and_reversible():
    d = B.make_desc(4, 2, 0, 0, 0, 4096 * 8, 1024 * 4, 4096 * 4, B.BF16, B.BF16)
    base = B.plan(d, B.OP_BWD_DX)
    try:
        B.set_plan_override(tile=128, k_splits=2)
        assert B.plan(d, B.OP_BWD_DX) == (128, 128, 2)
        B.set_plan_override(tile=256, k_splits=3)
        t = B.plan(d, B.OP_BWD_DX)
        assert t == (256, 256, 3) and B.workspace_bytes(d, B.OP_BWD_DX) >= 3 * 16 * 4 * 256 * 256 * 4
        with pytest.raises(B.TessError):
            B.set_plan_override(tile=64)
    finally:
        B.set_plan_override(0, 0)
    assert B.plan(d, B.OP_BWD_DX) == base
    # the environment no longer steers the product path
    os.environ["TESS_SPLITS"] = "7"
    try:
        assert B.plan(d, B.OP_BWD_DX) == base
    finally:
        del os.environ["TESS_SPLITS"]


def test_binding_refuses_tensors_of_the_wrong_dtype():
    """The library reads raw memory in the descriptor's dtypes; the binding must refuse a
    tensor of another element size before the call (it would be read or written past its
    end).  CPU tensors suffice: the dtype check comes first."""
    import torch
    q, d, m, kb, n = 2, 2, 16, 8, 24
    desc = B.make_desc(q, d, 0, 0, 0, m * q * d, kb * q, n * q, B.BF16, B.BF16)
    bf, f32 = torch.bfloat16, torch.float32
    x = [torch.zeros(m, kb, dtype=bf) for _ in range(q)]
    w = [torch.zeros(kb, n, dtype=bf) for _ in range(q)]
    dy = [torch.zeros(m, n, dtype=bf) for _ in range(q)]
    x32 = [t.float() for t in x]
    with pytest.raises(ValueError, match="dtype"):
        B.linear_fwd(desc, x32, w, None, B.ACT_NONE, torch.zeros(m, n, dtype=bf))
    with pytest.raises(ValueError, match="dtype"):
        B.linear_fwd(desc, x, w, None, B.ACT_NONE, torch.zeros(m, n, dtype=f32))
    with pytest.raises(ValueError, match="dtype"):
        B.linear_fwd(desc, x, w, torch.zeros(n, dtype=f32), B.ACT_NONE, torch.zeros(m, n, dtype=bf))
    with pytest.raises(ValueError, match="dtype"):
        B.linear_bwd_dx(desc, dy, w, torch.zeros(m, kb, dtype=f32))
    with pytest.raises(ValueError, match="dtype"):     # accumulate needs an fp32 buffer
        B.linear_bwd_dw(desc, x, dy, torch.zeros(kb, n, dtype=bf), accumulate=True)
    with pytest.raises(ValueError, match="dtype"):     # ... and overwrite needs out_dtype
        B.linear_bwd_dw(desc, x, dy, torch.zeros(kb, n, dtype=f32), accumulate=False)
    with pytest.raises(ValueError, match="dtype"):
        B.linear_bwd_dw_bias(desc, x, dy, torch.zeros(kb, n, dtype=bf), torch.zeros(n), accumulate=True)
    with pytest.raises(ValueError, match="dtype"):     # step partials are always fp32
        B.linear_bwd_dx_step(desc, dy[0], w[0], torch.zeros(m, kb, dtype=bf))
    with pytest.raises(ValueError, match="dtype"):
        B.linear_bwd_dw_step(desc, x[0], dy[0], torch.zeros(kb, n, dtype=bf))
    with pytest.raises(ValueError, match="dtype"):
        B.linear_bwd_dx_act(desc, dy, w, torch.zeros(m, kb, dtype=f32), B.ACT_GELU_ERF,
                            torch.zeros(m, kb, dtype=bf))
    # right dtypes get past the dtype check and stop at the device check
    with pytest.raises(ValueError, match="device"):
        B.linear_fwd(desc, x, w, None, B.ACT_NONE, torch.zeros(m, n, dtype=bf))


def test_build_check_of_m0_writes():
    """The build refuses device code in which anything but the loader's own statement
    (s_mov_b32 m0 followed by s_nop 0) writes M0."""
    from paper_2105_14500_amd import build as bld
    ok = "\n".join(["s_mov_b32 m0, s12", "s_nop 0", "buffer_load_dwordx4 v1, s[4:7], s9 offen lds",
                    "v_readlane_b32 s3, v2, m0", "ds_read_b128 v[0:3], v9"])
    assert bld.check_m0_writes(ok) == []
    assert bld.check_m0_writes("s_mov_b32 m0, s12\nv_add_f32 v1, v1, v2") != []     # no s_nop 0 behind it
    assert bld.check_m0_writes("s_add_u32 m0, s1, s2\ns_nop 0") != []
    assert bld.check_m0_writes("s_lshl_b32 m0, s1, 2") != []


def test_partition_helpers_match_block_table():
    """Views produced for processor (i,j,k) are the blocks of the hand-written table
    tests/golden/partition_q2_d2.txt (Alg. 3, h = i + k*q)."""
    import torch
    from paper_2105_14500_amd import partition as P
    A = torch.tensor([[10.0 * r + u for u in range(4)] for r in range(8)])
    with open(os.path.join(ROOT, "tests", "golden", "partition_q2_d2.txt")) as f:
        rows = [l.split("|") for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 8
    for left, right in rows:
        i, j, k = (int(v) for v in left.split())
        want = torch.tensor([float(v) for v in right.split()]).reshape(2, 2)
        assert torch.equal(P.out_block(A, 2, 2, i, j, k), want)
        a_p, _ = P.fwd_panels(A, torch.eye(4), 2, 2, i, j, k)
        assert torch.equal(a_p[j], want)
    with pytest.raises(ValueError):
        P.block_dims(2, 3, 12, 4, 4)


@pytest.mark.parametrize("tiles_m,tiles_n", [(1, 1), (1, 7), (5, 3), (8, 8), (16, 16), (17, 16), (16, 17),
                                             (32, 24), (32, 8), (8, 24), (33, 35), (3, 50), (50, 3),
                                             (31, 47), (64, 5)])
def test_block_to_tile_map_is_a_bijection(tiles_m, tiles_n):
    seen = set()
    for b in range(tiles_m * tiles_n):
        tm, tn = B.tile_of_block(b, tiles_m, tiles_n)
        assert 0 <= tm < tiles_m and 0 <= tn < tiles_n
        seen.add((tm, tn))
    assert len(seen) == tiles_m * tiles_n


def test_block_to_tile_map_gives_each_xcd_a_compact_block():
    """Of 256 consecutive workgroups (one per compute unit) of a 32 x 24 tile grid, the 32
    that land on one XCD (every eighth block id) cover 8 tile rows x 4 tile columns."""
    for rnd in range(3):
        tiles = [B.tile_of_block(b, 32, 24) for b in range(256 * rnd, 256 * (rnd + 1))]
        for xcd in range(8):
            mine = tiles[xcd::8]
            assert len(set(mine)) == 32
            assert len({t[0] for t in mine}) == 8 and len({t[1] for t in mine}) == 4
    assert B.lib().tess_tile_of_block(32 * 24, 32, 24, None, None) != 0
