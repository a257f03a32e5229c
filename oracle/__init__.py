"""RMSMP CPU oracle -- TEST INFRASTRUCTURE ONLY.

ctypes front-end of ``rmsmp_oracle.c`` (plain C, written from the paper: Section
3.1.1 / Eq. 1-2 Fixed quantizer, Section 3.1.2 / Eq. 3-4 PoT quantizer, Alg. 1
forward line for the layer output, Alg. 1 else-branch for the variance split).
Only the tests, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg may
import this package; the HIP library and its Python binding never do.

All arrays are numpy; integer tensors are int32, one code per element (no nibble
packing here -- packing is a storage detail of the HIP library).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rmsmp_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

FIXED4, POT4, FIXED8 = 0, 1, 2


def build(force=False):
    """Compile rmsmp_oracle.c with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-Wall", "-shared",
               "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "C", "H", "W", "KH", "KW", "stride", "pad")]


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_row_alpha.restype = ctypes.c_float
        _lib.oracle_conv_out_h.restype = ctypes.c_int64
        _lib.oracle_conv_out_w.restype = ctypes.c_int64
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _u8(a):
    return np.ascontiguousarray(a, dtype=np.uint8)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def num_threads():
    return int(_L().oracle_num_threads())


def set_threads(n):
    _L().oracle_set_threads(int(n))


def fixed_codes(w, alpha, m):
    """Fixed-m integer q in [-Q, Q], Q = 2^(m-1)-1 (Eq. 1-2), for every element of w."""
    w = _f32(w).ravel()
    q = np.empty(w.size, np.int32)
    _L().oracle_fixed_codes(_p(w, ctypes.c_float), ctypes.c_int64(w.size), ctypes.c_float(alpha),
                            ctypes.c_int(m), _p(q, ctypes.c_int32))
    return q


def pot4_ints(w, alpha):
    """PoT-4 signed integer sign*2^(6-k) or 0 (Eq. 3-4); level = alpha*2^-6 * value."""
    w = _f32(w).ravel()
    q = np.empty(w.size, np.int32)
    _L().oracle_pot4_ints(_p(w, ctypes.c_float), ctypes.c_int64(w.size), ctypes.c_float(alpha),
                          _p(q, ctypes.c_int32))
    return q


def quantize_rows(W, scheme, alpha=None, want_levels=True):
    """Row-wise mixed-scheme quantization.  Returns dict(wint, rowscale, alpha, what)."""
    W = _f32(W)
    M, K = W.shape
    scheme = _u8(scheme)
    assert scheme.shape == (M,)
    a_in = None if alpha is None else _f32(alpha)
    wint = np.empty((M, K), np.int32)
    rowscale = np.empty(M, np.float32)
    a_out = np.empty(M, np.float32)
    what = np.empty((M, K), np.float64) if want_levels else None
    rc = _L().oracle_quantize_rows(_p(W, ctypes.c_float), ctypes.c_int64(M), ctypes.c_int64(K),
                                   _p(scheme, ctypes.c_uint8), _p(a_in, ctypes.c_float),
                                   _p(wint, ctypes.c_int32), _p(rowscale, ctypes.c_float),
                                   _p(a_out, ctypes.c_float), _p(what, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle_quantize_rows: bad scheme code or alpha (rc=%d)" % rc)
    return dict(wint=wint, rowscale=rowscale, alpha=a_out, what=what)


def gemm_acc(wint, xq):
    """acc[M][N] = sum_k wint[M][K] * xq[N][K] in int32 (overflow checked)."""
    wint, xq = _i32(wint), _i32(xq)
    M, K = wint.shape
    N, K2 = xq.shape
    assert K == K2
    acc = np.empty((M, N), np.int32)
    rc = _L().oracle_gemm_acc(_p(wint, ctypes.c_int32), _p(xq, ctypes.c_int32), ctypes.c_int64(M),
                              ctypes.c_int64(K), ctypes.c_int64(N), _p(acc, ctypes.c_int32))
    if rc != 0:
        raise OverflowError("oracle_gemm_acc: int32 overflow")
    return acc


def gemm_acc_at(wint, xq, ms, ns):
    wint, xq, ms, ns = _i32(wint), _i32(xq), _i64(ms), _i64(ns)
    M, K = wint.shape
    N = xq.shape[0]
    out = np.empty(ms.size, np.int32)
    rc = _L().oracle_gemm_acc_at(_p(wint, ctypes.c_int32), _p(xq, ctypes.c_int32), ctypes.c_int64(M),
                                 ctypes.c_int64(K), ctypes.c_int64(N), _p(ms, ctypes.c_int64),
                                 _p(ns, ctypes.c_int64), ctypes.c_int64(ms.size), _p(out, ctypes.c_int32))
    if rc != 0:
        raise ValueError("oracle_gemm_acc_at: position out of range")
    return out


def gemm_acc_pot_shift(wint, scheme, xq):
    """PoT rows only, computed with shifts and adds; other rows are returned as zeros."""
    wint, xq, scheme = _i32(wint), _i32(xq), _u8(scheme)
    M, K = wint.shape
    N = xq.shape[0]
    acc = np.zeros((M, N), np.int32)
    rc = _L().oracle_gemm_acc_pot_shift(_p(wint, ctypes.c_int32), _p(scheme, ctypes.c_uint8),
                                        _p(xq, ctypes.c_int32), ctypes.c_int64(M), ctypes.c_int64(K),
                                        ctypes.c_int64(N), _p(acc, ctypes.c_int32))
    if rc != 0:
        raise ValueError("oracle_gemm_acc_pot_shift rc=%d" % rc)
    return acc


def rowsum(wint):
    wint = _i32(wint)
    M, K = wint.shape
    rs = np.empty(M, np.int32)
    _L().oracle_rowsum(_p(wint, ctypes.c_int32), ctypes.c_int64(M), ctypes.c_int64(K), _p(rs, ctypes.c_int32))
    return rs


def conv_desc(B, C, H, W, KH, KW, stride, pad):
    return ConvDesc(B, C, H, W, KH, KW, stride, pad)


def conv_out_hw(d):
    return int(_L().oracle_conv_out_h(ctypes.byref(d))), int(_L().oracle_conv_out_w(ctypes.byref(d)))


def conv_acc(wint, x, d, zpad=0):
    """Direct convolution.  wint [M][C][KH][KW], x [B][H][W][C] codes -> acc [M][B*OH*OW]."""
    wint, x = _i32(wint), _i32(x)
    M = wint.shape[0]
    assert wint.shape == (M, d.C, d.KH, d.KW) and x.shape == (d.B, d.H, d.W, d.C)
    OH, OW = conv_out_hw(d)
    acc = np.empty((M, d.B * OH * OW), np.int32)
    rc = _L().oracle_conv_acc(_p(wint, ctypes.c_int32), _p(x, ctypes.c_int32), ctypes.byref(d),
                              ctypes.c_int64(M), ctypes.c_int32(zpad), _p(acc, ctypes.c_int32))
    if rc != 0:
        raise OverflowError("oracle_conv_acc: int32 overflow")
    return acc


def conv_acc_at(wint, x, d, ms, ns, zpad=0):
    wint, x, ms, ns = _i32(wint), _i32(x), _i64(ms), _i64(ns)
    M = wint.shape[0]
    assert wint.shape == (M, d.C, d.KH, d.KW) and x.shape == (d.B, d.H, d.W, d.C)
    out = np.empty(ms.size, np.int32)
    rc = _L().oracle_conv_acc_at(_p(wint, ctypes.c_int32), _p(x, ctypes.c_int32), ctypes.byref(d),
                                 ctypes.c_int64(M), ctypes.c_int32(zpad), _p(ms, ctypes.c_int64),
                                 _p(ns, ctypes.c_int64), ctypes.c_int64(ms.size), _p(out, ctypes.c_int32))
    if rc != 0:
        raise ValueError("oracle_conv_acc_at: position out of range")
    return out


def epilogue(acc, rowsum_, z, rowscale, s_x, bias=None, relu=False, inv_s_out=None):
    """Zero-point correction, per-row dequant, bias, ReLU and (optional) 4-bit requant.

    Returns (acc_corr int32, y fp32, q uint8-or-None); q is one code per element."""
    acc = _i32(acc)
    M, N = acc.shape
    rs, sc = _i32(rowsum_), _f32(rowscale)
    b = None if bias is None else _f32(bias)
    acc_c = np.empty((M, N), np.int32)
    y = np.empty((M, N), np.float32)
    q = np.empty((M, N), np.uint8) if inv_s_out is not None else None
    _L().oracle_epilogue(_p(acc, ctypes.c_int32), ctypes.c_int64(M), ctypes.c_int64(N),
                         _p(rs, ctypes.c_int32), ctypes.c_int32(z), _p(sc, ctypes.c_float),
                         ctypes.c_float(s_x), _p(b, ctypes.c_float), ctypes.c_int(1 if relu else 0),
                         ctypes.c_float(0.0 if inv_s_out is None else inv_s_out),
                         _p(acc_c, ctypes.c_int32), _p(y, ctypes.c_float), _p(q, ctypes.c_uint8))
    return acc_c, y, q


def epilogue_gelu(acc, rowsum_, z, rowscale, s_x, bias, inv_s_out, z_out):
    """Zero-point correction, per-row dequant, bias, GELU and affine 4-bit requant.

    Returns (g fp32, q uint8), q one code per element."""
    acc = _i32(acc)
    M, N = acc.shape
    rs, sc = _i32(rowsum_), _f32(rowscale)
    b = None if bias is None else _f32(bias)
    g = np.empty((M, N), np.float32)
    q = np.empty((M, N), np.uint8)
    _L().oracle_epilogue_gelu(_p(acc, ctypes.c_int32), ctypes.c_int64(M), ctypes.c_int64(N),
                              _p(rs, ctypes.c_int32), ctypes.c_int32(z), _p(sc, ctypes.c_float),
                              ctypes.c_float(s_x), _p(b, ctypes.c_float), ctypes.c_float(inv_s_out),
                              ctypes.c_int32(z_out), _p(g, ctypes.c_float), _p(q, ctypes.c_uint8))
    return g, q


def gelu_codes(y, inv_s_out, z_out):
    """GELU and its affine 4-bit code for a list of fp32 pre-activations.  Returns (g fp32, q uint8)."""
    y = _f32(y).ravel()
    g = np.empty(y.size, np.float32)
    q = np.empty(y.size, np.uint8)
    _L().oracle_gelu_codes(_p(y, ctypes.c_float), ctypes.c_int64(y.size), ctypes.c_float(inv_s_out),
                           ctypes.c_int32(z_out), _p(g, ctypes.c_float), _p(q, ctypes.c_uint8))
    return g, q


def gemm_f64(what, xq, s_x, z=0, bias=None, relu=False):
    """The plain float64 definition sum_k what * (s_x*(xq - z)) (+bias, ReLU)."""
    what = np.ascontiguousarray(what, dtype=np.float64)
    xq = _i32(xq)
    M, K = what.shape
    N = xq.shape[0]
    b = None if bias is None else _f32(bias)
    y = np.empty((M, N), np.float64)
    _L().oracle_gemm_f64(_p(what, ctypes.c_double), _p(xq, ctypes.c_int32), ctypes.c_int64(M),
                         ctypes.c_int64(K), ctypes.c_int64(N), ctypes.c_double(s_x), ctypes.c_int32(z),
                         _p(b, ctypes.c_float), ctypes.c_int(1 if relu else 0), _p(y, ctypes.c_double))
    return y


def ratio_counts(M, pct_pot4, pct_fixed4, pct_fixed8):
    """Row counts (n_fixed4, n_pot4, n_fixed8) for the ratio PoT-4 : Fixed-4 : Fixed-8."""
    c = (ctypes.c_int64 * 3)()
    rc = _L().oracle_ratio_counts(ctypes.c_int64(M), int(pct_pot4), int(pct_fixed4), int(pct_fixed8), c)
    if rc != 0:
        raise ValueError("ratio must be non-negative and sum to 100")
    return int(c[0]), int(c[1]), int(c[2])


def assign_by_variance(W, scheme, n_pot4):
    """Alg. 1 else-branch: among rows not marked Fixed-8, lowest-variance n_pot4 rows -> PoT-4."""
    W = _f32(W)
    M, K = W.shape
    s = _u8(scheme).copy()
    rc = _L().oracle_assign_by_variance(_p(W, ctypes.c_float), ctypes.c_int64(M), ctypes.c_int64(K),
                                        ctypes.c_int64(n_pot4), _p(s, ctypes.c_uint8))
    if rc != 0:
        raise MemoryError("oracle_assign_by_variance")
    return s


def project_rows_f32(W, scheme, alpha=None):
    """Alg. 1 forward, weight side: proj_S(W) in fp32 (rowscale * integer level).  Returns (what, alpha)."""
    W = _f32(W)
    M, K = W.shape
    scheme = _u8(scheme)
    a_in = None if alpha is None else _f32(alpha)
    what = np.empty((M, K), np.float32)
    a_out = np.empty(M, np.float32)
    rc = _L().oracle_project_rows_f32(_p(W, ctypes.c_float), ctypes.c_int64(M), ctypes.c_int64(K),
                                      _p(scheme, ctypes.c_uint8), _p(a_in, ctypes.c_float),
                                      _p(what, ctypes.c_float), _p(a_out, ctypes.c_float))
    if rc != 0:
        raise ValueError("oracle_project_rows_f32: bad scheme code or alpha (rc=%d)" % rc)
    return what, a_out


def ste_backward(W, dwhat, alpha=None):
    """Eq. 5: gradient of the projected weights handed to the weights, zero where the clip was active."""
    W, dwhat = _f32(W), _f32(dwhat)
    M, K = W.shape
    assert dwhat.shape == (M, K)
    a_in = None if alpha is None else _f32(alpha)
    dw = np.empty((M, K), np.float32)
    _L().oracle_ste_backward(_p(W, ctypes.c_float), ctypes.c_int64(M), ctypes.c_int64(K), _p(a_in, ctypes.c_float),
                             _p(dwhat, ctypes.c_float), _p(dw, ctypes.c_float))
    return dw
