"""ctypes binding of the C ABI in include/tesseract.h.

Argument marshalling only: tensors are turned into device pointers, leading
dimensions and a stream handle; every step of the computation runs in the HIP
library.  There is no CPU fallback: a missing library raises at first use.
PyTorch is used for device memory and streams.
"""
import ctypes
import os

import torch

F32, BF16 = 0, 1
ACT_NONE, ACT_GELU_ERF, ACT_GELU_TANH = 0, 1, 2
OP_FWD, OP_BWD_DX, OP_BWD_DW, OP_BWD_DX_STEP, OP_BWD_DW_STEP = 0, 1, 2, 3, 4
MAX_Q = 16

_HERE = os.path.dirname(os.path.abspath(__file__))
# TESS_LIB_PATH: another build of the same sources (the host-only sanitizer build of the tests)
LIB_PATH = os.environ.get("TESS_LIB_PATH") or os.path.join(_HERE, "libtesseract_hip.so")

EXPORTS = ["tess_linear_fwd", "tess_linear_bwd_dx", "tess_linear_bwd_dw",
           "tess_linear_bwd_dx_act", "tess_linear_bwd_dw_bias",
           "tess_linear_bwd_dw_noalloc", "tess_noalloc_scratch_bytes",
           "tess_linear_bwd_dx_step", "tess_linear_bwd_dw_step",
           "tess_layernorm_row_sums", "tess_layernorm_normalize",
           "tess_layernorm_bwd_row_sums", "tess_layernorm_bwd_apply",
           "tess_linear_workspace_bytes", "tess_linear_plan", "tess_probe_mfma_rate",
           "tess_tile_of_block", "tess_diag_set_plan_override", "tess_desc_check", "tess_block_shape",
           "tess_status_string", "tess_version"]


class TessDesc(ctypes.Structure):
    """Mirror of `tess_desc`: grid [q,q,d], coordinates (i,j,k), global sizes a,b,c."""
    _fields_ = [("q", ctypes.c_int32), ("d", ctypes.c_int32),
                ("i", ctypes.c_int32), ("j", ctypes.c_int32), ("k", ctypes.c_int32),
                ("a", ctypes.c_int64), ("b", ctypes.c_int64), ("c", ctypes.c_int64),
                ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32)]


class TessError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def lib():
    """Load the HIP library (built in-tree by paper_2105_14500_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2105_14500_amd.build` "
                               "(or __graft_entry__.build()) first; there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, cint, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
        dp = ctypes.POINTER(TessDesc)
        pp = ctypes.POINTER(ctypes.c_void_p)
        L.tess_linear_fwd.restype = cint
        L.tess_linear_fwd.argtypes = [dp, pp, i64, pp, i64, vp, cint, vp, i64, vp, vp, sz, vp]
        L.tess_linear_bwd_dx.restype = cint
        L.tess_linear_bwd_dx.argtypes = [dp, pp, i64, pp, i64, vp, i64, vp, sz, vp]
        L.tess_linear_bwd_dw.restype = cint
        L.tess_linear_bwd_dw.argtypes = [dp, pp, i64, pp, i64, vp, i64, cint, vp, sz, vp]
        L.tess_linear_bwd_dw_noalloc.restype = cint
        L.tess_linear_bwd_dw_noalloc.argtypes = [dp, pp, i64, pp, i64, vp, i64, cint, vp]
        L.tess_noalloc_scratch_bytes.restype = sz
        L.tess_noalloc_scratch_bytes.argtypes = []
        L.tess_linear_bwd_dx_act.restype = cint
        L.tess_linear_bwd_dx_act.argtypes = [dp, pp, i64, pp, i64, vp, i64, cint, vp, i64, vp, sz, vp]
        L.tess_linear_bwd_dw_bias.restype = cint
        L.tess_linear_bwd_dw_bias.argtypes = [dp, pp, i64, pp, i64, vp, i64, vp, cint, vp, sz, vp]
        for name in ("tess_linear_bwd_dx_step", "tess_linear_bwd_dw_step"):
            getattr(L, name).restype = cint
            getattr(L, name).argtypes = [dp, vp, i64, vp, i64, vp, i64, cint, vp, sz, vp]
        L.tess_layernorm_row_sums.restype = cint
        L.tess_layernorm_row_sums.argtypes = [vp, i64, i64, i64, cint, vp, cint, vp]
        L.tess_layernorm_normalize.restype = cint
        L.tess_layernorm_normalize.argtypes = [vp, i64, i64, i64, cint, vp, i64, ctypes.c_float, vp, i64, vp]
        L.tess_layernorm_bwd_row_sums.restype = cint
        L.tess_layernorm_bwd_row_sums.argtypes = [vp, i64, vp, i64, i64, i64, cint, vp, cint, vp]
        L.tess_layernorm_bwd_apply.restype = cint
        L.tess_layernorm_bwd_apply.argtypes = [vp, i64, vp, i64, i64, i64, cint, vp, vp, i64,
                                               ctypes.c_float, vp, i64, vp]
        L.tess_linear_workspace_bytes.restype = sz
        L.tess_linear_workspace_bytes.argtypes = [dp, cint]
        i32p = ctypes.POINTER(ctypes.c_int32)
        L.tess_linear_plan.restype = cint
        L.tess_linear_plan.argtypes = [dp, cint, i32p, i32p, i32p]
        L.tess_probe_mfma_rate.restype = cint
        L.tess_probe_mfma_rate.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp]
        L.tess_diag_set_plan_override.restype = cint
        L.tess_diag_set_plan_override.argtypes = [ctypes.c_int32, ctypes.c_int32]
        L.tess_tile_of_block.restype = cint
        L.tess_tile_of_block.argtypes = [ctypes.c_int32] * 3 + [ctypes.POINTER(ctypes.c_int32)] * 2
        L.tess_desc_check.restype = cint
        L.tess_desc_check.argtypes = [dp]
        L.tess_block_shape.restype = cint
        L.tess_block_shape.argtypes = [dp, ctypes.POINTER(i64), ctypes.POINTER(i64),
                                       ctypes.POINTER(i64)]
        L.tess_status_string.restype = ctypes.c_char_p
        L.tess_status_string.argtypes = [cint]
        L.tess_version.restype = ctypes.c_char_p
        L.tess_version.argtypes = []
        _lib = L
    return _lib


def status_string(status):
    return lib().tess_status_string(int(status)).decode()


def version():
    return lib().tess_version().decode()


def dtype_code(dt):
    if dt == torch.float32:
        return F32
    if dt == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {dt}")


def make_desc(q, d, i, j, k, a, b, c, in_dtype=BF16, out_dtype=BF16):
    return TessDesc(q, d, i, j, k, a, b, c, in_dtype, out_dtype)


def desc_check(desc):
    return lib().tess_desc_check(ctypes.byref(desc))


def block_shape(desc):
    m, kb, n = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    st = lib().tess_block_shape(ctypes.byref(desc), ctypes.byref(m), ctypes.byref(kb),
                                ctypes.byref(n))
    if st:
        raise TessError(st, "tess_block_shape")
    return m.value, kb.value, n.value


def workspace_bytes(desc, op):
    return lib().tess_linear_workspace_bytes(ctypes.byref(desc), op)


def plan(desc, op):
    """(tile_m, tile_n, k_splits) of the launch the library would choose."""
    tm, tn, ks = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    st = lib().tess_linear_plan(ctypes.byref(desc), op, ctypes.byref(tm), ctypes.byref(tn),
                                ctypes.byref(ks))
    if st:
        raise TessError(st, "tess_linear_plan")
    return tm.value, tn.value, ks.value


def tile_of_block(block, tiles_m, tiles_n):
    """tess_tile_of_block: (tile row, tile column) of one workgroup."""
    tm, tn = ctypes.c_int32(), ctypes.c_int32()
    st = lib().tess_tile_of_block(block, tiles_m, tiles_n, ctypes.byref(tm), ctypes.byref(tn))
    if st:
        raise TessError(st, "tess_tile_of_block")
    return tm.value, tn.value


def probe_mfma_rate(sink, workgroups, iters, real_data=False, stream=None):
    """tess_probe_mfma_rate: enqueue the register-resident MFMA loop; returns its flop count.
    real_data: operands distributed like the workloads' instead of small integers."""
    if sink.numel() < workgroups * 256 or sink.dtype != torch.float32 or not sink.is_cuda:
        raise ValueError("sink: need a device float32 tensor of workgroups*256 elements")
    st = lib().tess_probe_mfma_rate(ctypes.c_void_p(sink.data_ptr()), workgroups, iters,
                                    1 if real_data else 0, _stream(stream))
    if st:
        raise TessError(st, "tess_probe_mfma_rate")
    return workgroups * 4 * iters * 16 * 32768.0


def set_plan_override(tile=0, k_splits=0):
    """tess_diag_set_plan_override: force tile (128/256) and K splits of later calls; 0 = cost model."""
    st = lib().tess_diag_set_plan_override(tile, k_splits)
    if st:
        raise TessError(st, "tess_diag_set_plan_override")


def layernorm_row_sums(x, sums_out, accumulate=False, stream=None):
    """tess_layernorm_row_sums: sums_out[m, 2] (+)= per-row sum and sum of squares of x[m, w]."""
    m, w = x.shape
    xp, ldx = _out(x, m, w, "x")
    if sums_out.dtype != torch.float32 or tuple(sums_out.shape) != (m, 2) or not sums_out.is_contiguous():
        raise ValueError("sums_out: need a contiguous device float32 tensor of shape (m, 2)")
    st = lib().tess_layernorm_row_sums(xp, m, w, ldx, dtype_code(x.dtype),
                                       ctypes.c_void_p(sums_out.data_ptr()), 1 if accumulate else 0,
                                       _stream(stream))
    if st:
        raise TessError(st, "tess_layernorm_row_sums")


def layernorm_normalize(x, sums, n_total, eps, xhat_out, stream=None):
    """tess_layernorm_normalize: xhat_out = (x - mean) / sqrt(var + eps) from the reduced sums."""
    m, w = x.shape
    xp, ldx = _out(x, m, w, "x")
    op, ldo = _out(xhat_out, m, w, "xhat_out")
    if xhat_out.dtype != x.dtype:
        raise ValueError("xhat_out: same dtype as x")
    if sums.dtype != torch.float32 or tuple(sums.shape) != (m, 2) or not sums.is_contiguous():
        raise ValueError("sums: need a contiguous device float32 tensor of shape (m, 2)")
    st = lib().tess_layernorm_normalize(xp, m, w, ldx, dtype_code(x.dtype),
                                        ctypes.c_void_p(sums.data_ptr()), n_total, float(eps), op, ldo,
                                        _stream(stream))
    if st:
        raise TessError(st, "tess_layernorm_normalize")


def _sums(t, m, what):
    if t.dtype != torch.float32 or tuple(t.shape) != (m, 2) or not t.is_contiguous() or not t.is_cuda:
        raise ValueError(f"{what}: need a contiguous device float32 tensor of shape (m, 2)")
    return ctypes.c_void_p(t.data_ptr())


def layernorm_bwd_row_sums(xhat, g, sums_out, accumulate=False, stream=None):
    """tess_layernorm_bwd_row_sums: sums_out[m, 2] (+)= per-row sum(xhat * g), sum(g)."""
    m, w = xhat.shape
    xp, ldx = _out(xhat, m, w, "xhat")
    gp, ldg = _out(g, m, w, "g")
    st = lib().tess_layernorm_bwd_row_sums(xp, ldx, gp, ldg, m, w, dtype_code(xhat.dtype),
                                           _sums(sums_out, m, "sums_out"), 1 if accumulate else 0,
                                           _stream(stream))
    if st:
        raise TessError(st, "tess_layernorm_bwd_row_sums")


def layernorm_bwd_apply(xhat, g, sums_bwd, sums_fwd, n_total, eps, dx_out, stream=None):
    """tess_layernorm_bwd_apply: dx_out = (g - (xhat * A + B) / n) / sqrt(var + eps)."""
    m, w = xhat.shape
    xp, ldx = _out(xhat, m, w, "xhat")
    gp, ldg = _out(g, m, w, "g")
    op, ldo = _out(dx_out, m, w, "dx_out")
    st = lib().tess_layernorm_bwd_apply(xp, ldx, gp, ldg, m, w, dtype_code(xhat.dtype),
                                        _sums(sums_bwd, m, "sums_bwd"), _sums(sums_fwd, m, "sums_fwd"),
                                        n_total, float(eps), op, ldo, _stream(stream))
    if st:
        raise TessError(st, "tess_layernorm_bwd_apply")


_TORCH_DTYPE = {F32: torch.float32, BF16: torch.bfloat16}


def _want_dtype(t, code, what):
    """The library reads and writes raw memory in the descriptor's dtypes: a tensor of another
    element size would be read or written past its end, so it is refused here."""
    if code is not None and t.dtype != _TORCH_DTYPE[code]:
        raise ValueError(f"{what} has dtype {t.dtype}, the call needs {_TORCH_DTYPE[code]}")


def _dtypes(**groups):
    """All dtype checks of a call, before anything else is looked at: each keyword is
    `name=(dtype code, tensor or list of tensors or None)`."""
    for what, (code, ts) in groups.items():
        if ts is None:
            continue
        for t in (ts if isinstance(ts, (list, tuple)) else [ts]):
            _want_dtype(t, code, what)


def _panel_array(panels, rows, cols, what, dtype=None):
    """q 2-D device tensors with unit column stride and one common row stride ->
    (host array of device pointers, leading dimension in elements)."""
    ld = None
    ptrs = (ctypes.c_void_p * len(panels))()
    for t, p in enumerate(panels):
        _want_dtype(p, dtype, f"{what}[{t}]")
        if p.dim() != 2 or tuple(p.shape) != (rows, cols):
            raise ValueError(f"{what}[{t}] has shape {tuple(p.shape)}, expected {(rows, cols)}")
        if not p.is_cuda:
            raise ValueError(f"{what}[{t}] is not a device tensor")
        if p.stride(1) != 1 and cols > 1:
            raise ValueError(f"{what}[{t}] rows are not contiguous")
        l = p.stride(0) if rows > 1 else max(p.stride(0), cols)
        if ld is None:
            ld = l
        elif l != ld:
            raise ValueError(f"{what}: panels differ in leading dimension")
        ptrs[t] = p.data_ptr()
    return ptrs, ld


def _out(t, rows, cols, what, dtype=None):
    _want_dtype(t, dtype, what)
    if t.dim() != 2 or tuple(t.shape) != (rows, cols) or not t.is_cuda or (cols > 1 and t.stride(1) != 1):
        raise ValueError(f"{what}: need a device tensor of shape {(rows, cols)} with contiguous rows")
    return ctypes.c_void_p(t.data_ptr()), (t.stride(0) if rows > 1 else max(t.stride(0), cols))


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _ws(workspace):
    if workspace is None:
        return None, 0
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace: need a contiguous device tensor")
    return ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def linear_fwd(desc, a_panels, b_panels, bias, act, c_out, preact_out=None, workspace=None,
               stream=None):
    """tess_linear_fwd: c_out = act(sum_t a_panels[t] @ b_panels[t] + bias)."""
    m, kb, n = block_shape(desc)
    _dtypes(a_panels=(desc.in_dtype, a_panels), b_panels=(desc.in_dtype, b_panels),
            bias=(desc.in_dtype, bias), c_out=(desc.out_dtype, c_out),
            preact_out=(desc.out_dtype, preact_out))
    ap, lda = _panel_array(a_panels, m, kb, "a_panels", desc.in_dtype)
    bp, ldb = _panel_array(b_panels, kb, n, "b_panels", desc.in_dtype)
    cp, ldc = _out(c_out, m, n, "c_out", desc.out_dtype)
    pre = None
    if preact_out is not None:
        pre, ldp = _out(preact_out, m, n, "preact_out", desc.out_dtype)
        if ldp != ldc:
            raise ValueError("preact_out must share c_out's leading dimension")
    if bias is not None:
        _want_dtype(bias, desc.in_dtype, "bias")
        if tuple(bias.shape) != (n,) or not bias.is_cuda or not bias.is_contiguous():
            raise ValueError(f"bias: need a contiguous device tensor of shape {(n,)}")
    bptr = ctypes.c_void_p(bias.data_ptr()) if bias is not None else None
    wsp, wsb = _ws(workspace)
    st = lib().tess_linear_fwd(ctypes.byref(desc), ap, lda, bp, ldb, bptr, act, cp, ldc, pre,
                               wsp, wsb, _stream(stream))
    if st:
        raise TessError(st, "tess_linear_fwd")


def linear_bwd_dx(desc, dy_panels, w_panels, dx_out, workspace=None, stream=None):
    """tess_linear_bwd_dx: dx_out = sum_t dy_panels[t] @ w_panels[t]^T."""
    m, kb, n = block_shape(desc)
    _dtypes(dy_panels=(desc.in_dtype, dy_panels), w_panels=(desc.in_dtype, w_panels),
            dx_out=(desc.out_dtype, dx_out))
    dyp, lddy = _panel_array(dy_panels, m, n, "dy_panels", desc.in_dtype)
    wp, ldw = _panel_array(w_panels, kb, n, "w_panels", desc.in_dtype)
    op, ldo = _out(dx_out, m, kb, "dx_out", desc.out_dtype)
    wsp, wsb = _ws(workspace)
    st = lib().tess_linear_bwd_dx(ctypes.byref(desc), dyp, lddy, wp, ldw, op, ldo, wsp, wsb,
                                  _stream(stream))
    if st:
        raise TessError(st, "tess_linear_bwd_dx")


def linear_bwd_dx_act(desc, dy_panels, w_panels, preact, act, dz_out, workspace=None, stream=None):
    """tess_linear_bwd_dx_act: dz_out = (sum_t dy_panels[t] @ w_panels[t]^T) * act'(preact)."""
    m, kb, n = block_shape(desc)
    _dtypes(dy_panels=(desc.in_dtype, dy_panels), w_panels=(desc.in_dtype, w_panels),
            preact=(desc.in_dtype, preact), dz_out=(desc.out_dtype, dz_out))
    dyp, lddy = _panel_array(dy_panels, m, n, "dy_panels", desc.in_dtype)
    wp, ldw = _panel_array(w_panels, kb, n, "w_panels", desc.in_dtype)
    op, ldo = _out(dz_out, m, kb, "dz_out", desc.out_dtype)
    zp, ldz = _out(preact, m, kb, "preact", desc.in_dtype) if preact is not None else (None, 0)
    wsp, wsb = _ws(workspace)
    st = lib().tess_linear_bwd_dx_act(ctypes.byref(desc), dyp, lddy, wp, ldw, zp, ldz, act, op, ldo,
                                      wsp, wsb, _stream(stream))
    if st:
        raise TessError(st, "tess_linear_bwd_dx_act")


def linear_bwd_dw_bias(desc, x_panels, dy_panels, dw_out, dbias_out, accumulate=False,
                       workspace=None, stream=None):
    """tess_linear_bwd_dw_bias: linear_bwd_dw plus dbias_out (+)= column sums of the dy panels."""
    m, kb, n = block_shape(desc)
    _dtypes(x_panels=(desc.in_dtype, x_panels), dy_panels=(desc.in_dtype, dy_panels),
            dw_out=(F32 if accumulate else desc.out_dtype, dw_out))
    xp, ldx = _panel_array(x_panels, m, kb, "x_panels", desc.in_dtype)
    dyp, lddy = _panel_array(dy_panels, m, n, "dy_panels", desc.in_dtype)
    op, ldo = _out(dw_out, kb, n, "dw_out", F32 if accumulate else desc.out_dtype)
    if dbias_out is not None and (dbias_out.dtype != torch.float32 or tuple(dbias_out.shape) != (n,)
                                  or not dbias_out.is_cuda or not dbias_out.is_contiguous()):
        raise ValueError(f"dbias_out: need a contiguous device float32 tensor of shape {(n,)}")
    bp = ctypes.c_void_p(dbias_out.data_ptr()) if dbias_out is not None else None
    wsp, wsb = _ws(workspace)
    st = lib().tess_linear_bwd_dw_bias(ctypes.byref(desc), xp, ldx, dyp, lddy, op, ldo, bp,
                                       1 if accumulate else 0, wsp, wsb, _stream(stream))
    if st:
        raise TessError(st, "tess_linear_bwd_dw_bias")


def linear_bwd_dx_step(desc, dy_block, w_block, partial_out, accumulate=False, workspace=None,
                       stream=None):
    """tess_linear_bwd_dx_step: partial_out (fp32) (+)= dy_block @ w_block^T."""
    m, kb, n = block_shape(desc)
    _dtypes(dy_block=(desc.in_dtype, dy_block), w_block=(desc.in_dtype, w_block),
            partial_out=(F32, partial_out))
    ap, lda = _out(dy_block, m, n, "dy_block", desc.in_dtype)
    bp, ldb = _out(w_block, kb, n, "w_block", desc.in_dtype)
    op, ldo = _out(partial_out, m, kb, "partial_out", F32)
    wsp, wsb = _ws(workspace)
    st = lib().tess_linear_bwd_dx_step(ctypes.byref(desc), ap, lda, bp, ldb, op, ldo,
                                       1 if accumulate else 0, wsp, wsb, _stream(stream))
    if st:
        raise TessError(st, "tess_linear_bwd_dx_step")


def linear_bwd_dw_step(desc, x_block, dy_block, partial_out, accumulate=False, workspace=None,
                       stream=None):
    """tess_linear_bwd_dw_step: partial_out (fp32) (+)= x_block^T @ dy_block."""
    m, kb, n = block_shape(desc)
    _dtypes(x_block=(desc.in_dtype, x_block), dy_block=(desc.in_dtype, dy_block),
            partial_out=(F32, partial_out))
    ap, lda = _out(x_block, m, kb, "x_block", desc.in_dtype)
    bp, ldb = _out(dy_block, m, n, "dy_block", desc.in_dtype)
    op, ldo = _out(partial_out, kb, n, "partial_out", F32)
    wsp, wsb = _ws(workspace)
    st = lib().tess_linear_bwd_dw_step(ctypes.byref(desc), ap, lda, bp, ldb, op, ldo,
                                       1 if accumulate else 0, wsp, wsb, _stream(stream))
    if st:
        raise TessError(st, "tess_linear_bwd_dw_step")


def linear_bwd_dw(desc, x_panels, dy_panels, dw_out, accumulate=False, workspace=None,
                  stream=None):
    """tess_linear_bwd_dw: dw_out (+)= sum_t x_panels[t]^T @ dy_panels[t]."""
    m, kb, n = block_shape(desc)
    _dtypes(x_panels=(desc.in_dtype, x_panels), dy_panels=(desc.in_dtype, dy_panels),
            dw_out=(F32 if accumulate else desc.out_dtype, dw_out))
    xp, ldx = _panel_array(x_panels, m, kb, "x_panels", desc.in_dtype)
    dyp, lddy = _panel_array(dy_panels, m, n, "dy_panels", desc.in_dtype)
    op, ldo = _out(dw_out, kb, n, "dw_out", F32 if accumulate else desc.out_dtype)
    wsp, wsb = _ws(workspace)
    st = lib().tess_linear_bwd_dw(ctypes.byref(desc), xp, ldx, dyp, lddy, op, ldo,
                                  1 if accumulate else 0, wsp, wsb, _stream(stream))
    if st:
        raise TessError(st, "tess_linear_bwd_dw")


def linear_bwd_dw_noalloc(desc, x_panels, dy_panels, dw_out, accumulate=False, stream=None):
    """tess_linear_bwd_dw_noalloc: linear_bwd_dw with the library's own static scratch."""
    m, kb, n = block_shape(desc)
    _dtypes(x_panels=(desc.in_dtype, x_panels), dy_panels=(desc.in_dtype, dy_panels),
            dw_out=(F32 if accumulate else desc.out_dtype, dw_out))
    xp, ldx = _panel_array(x_panels, m, kb, "x_panels", desc.in_dtype)
    dyp, lddy = _panel_array(dy_panels, m, n, "dy_panels", desc.in_dtype)
    op, ldo = _out(dw_out, kb, n, "dw_out", F32 if accumulate else desc.out_dtype)
    st = lib().tess_linear_bwd_dw_noalloc(ctypes.byref(desc), xp, ldx, dyp, lddy, op, ldo,
                                          1 if accumulate else 0, _stream(stream))
    if st:
        raise TessError(st, "tess_linear_bwd_dw_noalloc")


def noalloc_scratch_bytes():
    return lib().tess_noalloc_scratch_bytes()
