"""numpy front-end of the C fp64 oracle (oracle/tess_oracle.c).

TEST INFRASTRUCTURE.  Only tests/, the smoke check and the benchmark's
cpu_baseline leg import this module.  It marshals numpy float64 arrays into
the C routines and contains no arithmetic of its own beyond slicing views.
"""
import ctypes
import os

import numpy as np

from . import build as _build

ACT_NONE, ACT_GELU_ERF, ACT_GELU_TANH = 0, 1, 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        # TESS_ORACLE_LIB: another build of the same source (the sanitizer build of the tests)
        path = os.environ.get("TESS_ORACLE_LIB") or _build.build(force=False)
        L = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        i64 = ctypes.c_int64
        L.orc_num_threads.restype = ctypes.c_int
        L.orc_gelu_erf.restype = ctypes.c_double
        L.orc_gelu_erf.argtypes = [ctypes.c_double]
        L.orc_gelu_tanh.restype = ctypes.c_double
        L.orc_gelu_tanh.argtypes = [ctypes.c_double]
        for name in ("orc_gelu_erf_grad", "orc_gelu_tanh_grad"):
            getattr(L, name).restype = ctypes.c_double
            getattr(L, name).argtypes = [ctypes.c_double]
        L.orc_round_bf16_scalar.restype = ctypes.c_float
        L.orc_round_bf16_scalar.argtypes = [ctypes.c_float]
        L.orc_round_bf16.argtypes = [ctypes.POINTER(ctypes.c_float), dp, i64]
        for name in ("orc_matmul_nn", "orc_matmul_nt", "orc_matmul_tn"):
            getattr(L, name).argtypes = [dp, dp, dp, i64, i64, i64]
            getattr(L, name).restype = None
        L.orc_block_row.restype = i64
        L.orc_block_row.argtypes = [ctypes.c_int] * 3
        L.orc_check_grid.restype = ctypes.c_int
        L.orc_check_grid.argtypes = [ctypes.c_int] * 5 + [i64] * 3
        pp = ctypes.POINTER(dp)
        ip = ctypes.POINTER(i64)
        L.orc_fwd_panels.argtypes = [ctypes.c_int, i64, i64, i64, pp, i64, pp, i64, dp,
                                     ctypes.c_int, ip, i64, dp, dp]
        L.orc_fwd_panels.restype = None
        L.orc_bwd_dx_panels.argtypes = [ctypes.c_int, i64, i64, i64, pp, i64, pp, i64,
                                        ip, i64, dp]
        L.orc_bwd_dx_panels.restype = None
        L.orc_bwd_dw_panels.argtypes = [ctypes.c_int, i64, i64, i64, pp, i64, pp, i64,
                                        ip, i64, ctypes.c_int, dp]
        L.orc_bwd_dw_panels.restype = None
        L.orc_bwd_dx_act_panels.argtypes = [ctypes.c_int, i64, i64, i64, pp, i64, pp, i64,
                                            dp, i64, ctypes.c_int, ctypes.POINTER(i64), i64, dp]
        L.orc_bwd_dx_act_panels.restype = None
        L.orc_bias_grad_panels.argtypes = [ctypes.c_int, i64, i64, pp, i64, ctypes.c_int, dp]
        L.orc_bias_grad_panels.restype = None
        L.orc_row_sums.argtypes = [dp, i64, i64, i64, ctypes.c_int, dp]
        L.orc_row_sums.restype = None
        L.orc_layernorm_from_sums.argtypes = [dp, i64, i64, i64, dp, i64, ctypes.c_double, dp]
        L.orc_layernorm_from_sums.restype = None
        L.orc_row_sums_bwd.argtypes = [dp, dp, i64, i64, i64, i64, ctypes.c_int, dp]
        L.orc_row_sums_bwd.restype = None
        L.orc_layernorm_bwd_from_sums.argtypes = [dp, dp, i64, i64, i64, i64, dp, dp, i64,
                                                  ctypes.c_double, dp]
        L.orc_layernorm_bwd_from_sums.restype = None
        L.orc_tess_fwd.argtypes = [ctypes.c_int] * 5 + [i64] * 3 + [dp, dp, dp, ctypes.c_int,
                                                                   dp, dp]
        L.orc_tess_fwd.restype = ctypes.c_int
        L.orc_tess_bwd_dx.argtypes = [ctypes.c_int] * 5 + [i64] * 3 + [dp, dp, dp]
        L.orc_tess_bwd_dx.restype = ctypes.c_int
        L.orc_tess_bwd_dw.argtypes = [ctypes.c_int] * 5 + [i64] * 3 + [dp, dp, ctypes.c_int, dp]
        L.orc_tess_bwd_dw.restype = ctypes.c_int
        L.orc_rel_frobenius.argtypes = [dp, dp, i64]
        L.orc_rel_frobenius.restype = ctypes.c_double
        _lib = L
    return _lib


_DP = ctypes.POINTER(ctypes.c_double)


def _f64(x):
    x = np.ascontiguousarray(x, dtype=np.float64)
    return x


def _p(x):
    return x.ctypes.data_as(_DP) if x is not None else None


def num_threads():
    return lib().orc_num_threads()


def _scalar_fn(name, x):
    """Apply a double -> double routine of the library to a scalar or element-wise."""
    f = getattr(lib(), name)
    if np.ndim(x) == 0:
        return f(float(x))
    return np.vectorize(f, otypes=[np.float64])(x)


def gelu_erf(x):
    return _scalar_fn("orc_gelu_erf", x)


def gelu_tanh(x):
    return _scalar_fn("orc_gelu_tanh", x)


def gelu_erf_grad(x):
    return _scalar_fn("orc_gelu_erf_grad", x)


def gelu_tanh_grad(x):
    return _scalar_fn("orc_gelu_tanh_grad", x)


def round_bf16(x):
    """fp32 array -> nearest bf16 values (ties to even), returned as float64."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.float64)
    lib().orc_round_bf16(x.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), _p(out), x.size)
    return out


def matmul_nn(A, B):
    A, B = _f64(A), _f64(B)
    M, K = A.shape
    N = B.shape[1]
    assert B.shape[0] == K
    C = np.empty((M, N))
    lib().orc_matmul_nn(_p(A), _p(B), _p(C), M, N, K)
    return C


def matmul_nt(A, B):
    A, B = _f64(A), _f64(B)
    M, K = A.shape
    N = B.shape[0]
    assert B.shape[1] == K
    C = np.empty((M, N))
    lib().orc_matmul_nt(_p(A), _p(B), _p(C), M, N, K)
    return C


def matmul_tn(A, B):
    A, B = _f64(A), _f64(B)
    K, M = A.shape
    N = B.shape[1]
    assert B.shape[0] == K
    C = np.empty((M, N))
    lib().orc_matmul_tn(_p(A), _p(B), _p(C), M, N, K)
    return C


def block_row(q, i, k):
    return lib().orc_block_row(q, i, k)


def check_grid(q, d, i, j, k, a, b, c):
    return lib().orc_check_grid(q, d, i, j, k, a, b, c)


def _panel_ptrs(panels):
    """panels: list of 2-D float64 arrays whose rows are contiguous (views allowed)."""
    ld = None
    for p in panels:
        assert p.dtype == np.float64 and p.ndim == 2 and p.strides[1] == 8
        l = p.strides[0] // 8
        assert ld is None or l == ld, "panels of one operand share a leading dimension"
        ld = l
    arr = (_DP * len(panels))(*[p.ctypes.data_as(_DP) for p in panels])
    return arr, ld


def _rows(rows):
    if rows is None:
        return None, 0, None
    r = np.ascontiguousarray(rows, dtype=np.int64)
    return r.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), r.size, r


def fwd_panels(a_panels, b_panels, bias=None, act=ACT_NONE, rows=None, want_z=False):
    q = len(a_panels)
    assert len(b_panels) == q
    m, kb = a_panels[0].shape
    n = b_panels[0].shape[1]
    assert all(p.shape == (m, kb) for p in a_panels) and all(p.shape == (kb, n) for p in b_panels)
    ap, lda = _panel_ptrs(a_panels)
    bp, ldb = _panel_ptrs(b_panels)
    rp, nr, keep = _rows(rows)
    R = nr if rows is not None else m
    y = np.empty((R, n))
    z = np.empty((R, n)) if want_z else None
    bias64 = _f64(bias) if bias is not None else None
    lib().orc_fwd_panels(q, m, kb, n, ap, lda, bp, ldb, _p(bias64), act, rp, nr, _p(y), _p(z))
    return (y, z) if want_z else y


def bwd_dx_panels(dy_panels, w_panels, rows=None):
    q = len(dy_panels)
    assert len(w_panels) == q
    m, n = dy_panels[0].shape
    kb = w_panels[0].shape[0]
    assert all(p.shape == (m, n) for p in dy_panels) and all(p.shape == (kb, n) for p in w_panels)
    dyp, lddy = _panel_ptrs(dy_panels)
    wp, ldw = _panel_ptrs(w_panels)
    rp, nr, keep = _rows(rows)
    R = nr if rows is not None else m
    dx = np.empty((R, kb))
    lib().orc_bwd_dx_panels(q, m, kb, n, dyp, lddy, wp, ldw, rp, nr, _p(dx))
    return dx


def bwd_dx_act_panels(dy_panels, w_panels, z, act, rows=None):
    """dX of bwd_dx_panels times act'(z); z is the FULL [m, kb] pre-activation."""
    q = len(dy_panels)
    m, n = dy_panels[0].shape
    kb = w_panels[0].shape[0]
    assert all(p.shape == (m, n) for p in dy_panels) and all(p.shape == (kb, n) for p in w_panels)
    z = _f64(z)
    assert z.shape == (m, kb)
    dyp, lddy = _panel_ptrs(dy_panels)
    wp, ldw = _panel_ptrs(w_panels)
    rp, nr, keep = _rows(rows)
    R = nr if rows is not None else m
    dz = np.empty((R, kb))
    lib().orc_bwd_dx_act_panels(q, m, kb, n, dyp, lddy, wp, ldw, _p(z), kb, act, rp, nr, _p(dz))
    return dz


def bias_grad_panels(dy_panels, accumulate_into=None):
    q = len(dy_panels)
    m, n = dy_panels[0].shape
    assert all(p.shape == (m, n) for p in dy_panels)
    dyp, lddy = _panel_ptrs(dy_panels)
    if accumulate_into is not None:
        db = accumulate_into
        assert db.dtype == np.float64 and db.shape == (n,) and db.flags.c_contiguous
        acc = 1
    else:
        db = np.empty((n,))
        acc = 0
    lib().orc_bias_grad_panels(q, m, n, dyp, lddy, acc, _p(db))
    return db


def row_sums(x, accumulate_into=None):
    """[m, 2]: per row the sum and the sum of squares of the block x [m, w]."""
    x = _f64(x)
    m, w = x.shape
    if accumulate_into is not None:
        out = accumulate_into
        assert out.dtype == np.float64 and out.shape == (m, 2) and out.flags.c_contiguous
        acc = 1
    else:
        out = np.empty((m, 2))
        acc = 0
    lib().orc_row_sums(_p(x), m, w, w, acc, _p(out))
    return out


def layernorm_from_sums(x, sums, n_total, eps):
    x = _f64(x)
    sums = _f64(sums)
    m, w = x.shape
    assert sums.shape == (m, 2)
    out = np.empty((m, w))
    lib().orc_layernorm_from_sums(_p(x), m, w, w, _p(sums), n_total, float(eps), _p(out))
    return out


def row_sums_bwd(xhat, g, accumulate_into=None):
    """[m, 2]: per row sum(xhat * g) and sum(g) of one block."""
    xhat, g = _f64(xhat), _f64(g)
    m, w = xhat.shape
    assert g.shape == (m, w)
    if accumulate_into is not None:
        out = accumulate_into
        assert out.dtype == np.float64 and out.shape == (m, 2) and out.flags.c_contiguous
        acc = 1
    else:
        out = np.empty((m, 2))
        acc = 0
    lib().orc_row_sums_bwd(_p(xhat), _p(g), m, w, w, w, acc, _p(out))
    return out


def layernorm_bwd_from_sums(xhat, g, sums_bwd, sums_fwd, n_total, eps):
    xhat, g, sums_bwd, sums_fwd = _f64(xhat), _f64(g), _f64(sums_bwd), _f64(sums_fwd)
    m, w = xhat.shape
    out = np.empty((m, w))
    lib().orc_layernorm_bwd_from_sums(_p(xhat), _p(g), m, w, w, w, _p(sums_bwd), _p(sums_fwd), n_total,
                                      float(eps), _p(out))
    return out


def bwd_dw_panels(x_panels, dy_panels, rows=None, accumulate_into=None):
    q = len(x_panels)
    assert len(dy_panels) == q
    m, kb = x_panels[0].shape
    n = dy_panels[0].shape[1]
    assert all(p.shape == (m, kb) for p in x_panels) and all(p.shape == (m, n) for p in dy_panels)
    xp, ldx = _panel_ptrs(x_panels)
    dyp, lddy = _panel_ptrs(dy_panels)
    rp, nr, keep = _rows(rows)
    R = nr if rows is not None else kb
    if accumulate_into is not None:
        dw = accumulate_into
        assert dw.dtype == np.float64 and dw.shape == (R, n) and dw.flags.c_contiguous
        acc = 1
    else:
        dw = np.empty((R, n))
        acc = 0
    lib().orc_bwd_dw_panels(q, m, kb, n, xp, ldx, dyp, lddy, rp, nr, acc, _p(dw))
    return dw


def tess_fwd(q, d, i, j, k, A, B, bias=None, act=ACT_NONE, want_z=False):
    A, B = _f64(A), _f64(B)
    a, b = A.shape
    c = B.shape[1]
    assert B.shape[0] == b
    if check_grid(q, d, i, j, k, a, b, c):
        raise ValueError("inadmissible grid or sizes")
    y = np.empty((a // (q * d), c // q))
    z = np.empty_like(y) if want_z else None
    bias64 = _f64(bias) if bias is not None else None
    rc = lib().orc_tess_fwd(q, d, i, j, k, a, b, c, _p(A), _p(B), _p(bias64), act, _p(y), _p(z))
    assert rc == 0
    return (y, z) if want_z else y


def tess_bwd_dx(q, d, i, j, k, dY, W):
    dY, W = _f64(dY), _f64(W)
    a, c = dY.shape
    b = W.shape[0]
    assert W.shape[1] == c
    if check_grid(q, d, i, j, k, a, b, c):
        raise ValueError("inadmissible grid or sizes")
    dx = np.empty((a // (q * d), b // q))
    rc = lib().orc_tess_bwd_dx(q, d, i, j, k, a, b, c, _p(dY), _p(W), _p(dx))
    assert rc == 0
    return dx


def tess_bwd_dw(q, d, i, j, k, X, dY, accumulate_into=None):
    X, dY = _f64(X), _f64(dY)
    a, b = X.shape
    c = dY.shape[1]
    assert dY.shape[0] == a
    if check_grid(q, d, i, j, k, a, b, c):
        raise ValueError("inadmissible grid or sizes")
    if accumulate_into is not None:
        dw = accumulate_into
        assert dw.dtype == np.float64 and dw.shape == (b // q, c // q) and dw.flags.c_contiguous
        acc = 1
    else:
        dw = np.empty((b // q, c // q))
        acc = 0
    rc = lib().orc_tess_bwd_dw(q, d, i, j, k, a, b, c, _p(X), _p(dY), acc, _p(dw))
    assert rc == 0
    return dw


def rel_frobenius(G, O):
    G, O = _f64(G), _f64(O)
    assert G.shape == O.shape
    return lib().orc_rel_frobenius(_p(G), _p(O), G.size)
