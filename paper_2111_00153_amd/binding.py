"""Thin ctypes binding of librmsmp.so: argument marshalling only.

Function names mirror include/rmsmp.h.  Device buffers are torch tensors (PyTorch is used
for device memory and streams, nothing else); host arrays are numpy.  Every computation of
the hot path happens inside the library's HIP kernels -- there is no Python or CPU fallback:
if the shared library is missing, importing this module raises.
"""
import ctypes
import os

import numpy as np
# torch ships its own copy of the HIP runtime: it has to be in the process before the library is
# loaded, so that both resolve to that one copy (two runtimes in one process do not see the GPU)
import torch  # noqa: F401

from . import build as _build

FIXED4, POT4, FIXED8 = 0, 1, 2
OUT_INT32, OUT_FP32, OUT_U4, OUT_GELU_U4 = 0, 1, 2, 3

_STATUS = {0: "OK", 1: "EINVAL", 2: "ESHAPE", 3: "ENOMEM", 4: "EHIP", 5: "EUNSUPPORTED", 6: "EWORKSPACE"}


class RmsmpError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("librmsmp %s: %s" % (_STATUS.get(code, code), msg))
        self.code = code


class Epilogue(ctypes.Structure):
    _fields_ = [("act_scale", ctypes.c_float), ("act_zero_point", ctypes.c_int32), ("act_bits", ctypes.c_int32),
                ("bias", ctypes.c_void_p), ("relu", ctypes.c_int32), ("out_kind", ctypes.c_int32),
                ("out_inv_scale", ctypes.c_float), ("out_zero_point", ctypes.c_int32)]


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "C", "H", "W", "KH", "KW", "stride", "pad")]


def _load():
    path = _build.LIB
    if not os.path.exists(path):
        raise ImportError("librmsmp.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no fallback implementation)")
    lib = ctypes.CDLL(path)
    lib.rmsmp_last_error.restype = ctypes.c_char_p
    lib.rmsmp_version.restype = ctypes.c_char_p
    return lib


_lib = _load()

EXPORTS = ["rmsmp_last_error", "rmsmp_version", "rmsmp_ratio_counts", "rmsmp_assign_by_variance",
           "rmsmp_pack_weights", "rmsmp_free_packed", "rmsmp_packed_info", "rmsmp_unpack_codes",
           "rmsmp_pack_roundtrip_host", "rmsmp_gemm", "rmsmp_conv2d", "rmsmp_conv2d_workspace_size",
           "rmsmp_fake_quant_rows", "rmsmp_ste_backward", "rmsmp_debug_set_wave_split",
           "rmsmp_debug_last_dispatch", "rmsmp_debug_measure_peaks", "rmsmp_init", "rmsmp_conv2d_static_workspace", "rmsmp_debug_gelu_breakpoints",
           "rmsmp_conv2d_pair", "rmsmp_pack_weights_opt"]


def _check(rc):
    if rc != 0:
        raise RmsmpError(rc, _lib.rmsmp_last_error().decode())


def _np(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _ptr(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _dev(t):
    """Device pointer of a torch tensor (must be contiguous and on the GPU)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous GPU tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def rmsmp_version():
    return _lib.rmsmp_version().decode()


def rmsmp_ratio_counts(M, pct_pot4, pct_fixed4, pct_fixed8):
    c = (ctypes.c_int64 * 3)()
    _check(_lib.rmsmp_ratio_counts(ctypes.c_int64(M), int(pct_pot4), int(pct_fixed4), int(pct_fixed8), c))
    return int(c[0]), int(c[1]), int(c[2])


def rmsmp_assign_by_variance(W, scheme, n_pot4):
    W = _np(W, np.float32)
    s = _np(scheme, np.uint8).copy()
    _check(_lib.rmsmp_assign_by_variance(_ptr(W), ctypes.c_int64(W.shape[0]), ctypes.c_int64(W.shape[1]),
                                         ctypes.c_int64(n_pot4), _ptr(s)))
    return s


class Packed:
    """Owner of an rmsmp_packed handle."""

    def __init__(self, handle, M, K, taps):
        self.handle = handle
        self.M, self.K, self.taps = M, K, taps
        counts = (ctypes.c_int64 * 3)()
        perm = ctypes.POINTER(ctypes.c_int32)()
        rs = ctypes.POINTER(ctypes.c_float)()
        rsum = ctypes.POINTER(ctypes.c_int32)()
        _check(_lib.rmsmp_packed_info(handle, None, None, counts, ctypes.byref(perm), ctypes.byref(rs),
                                      ctypes.byref(rsum)))
        self.counts = tuple(int(c) for c in counts)
        self.perm = np.ctypeslib.as_array(perm, (M,)).copy()
        self.rowscale = np.ctypeslib.as_array(rs, (M,)).copy()
        self.rowsum = np.ctypeslib.as_array(rsum, (M,)).copy()

    def free(self):
        if self.handle:
            _lib.rmsmp_free_packed(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


PACK_POT_AS_INT8 = 1  # RMSMP_PACK_POT_AS_INT8


def rmsmp_pack_weights(W, scheme, alpha=None, taps=1, in_perm=None, flags=0):
    """flags = 0: rmsmp_pack_weights; otherwise rmsmp_pack_weights_opt with those flags."""
    W = _np(W, np.float32)
    M, K = W.shape
    scheme = _np(scheme, np.uint8)
    if scheme.shape != (M,):
        raise ValueError("scheme must have one entry per row")
    alpha = None if alpha is None else _np(alpha, np.float32)
    in_perm = None if in_perm is None else _np(in_perm, np.int32)
    h = ctypes.c_void_p()
    if flags:
        _check(_lib.rmsmp_pack_weights_opt(_ptr(W), ctypes.c_int64(M), ctypes.c_int64(K), _ptr(scheme), _ptr(alpha),
                                           ctypes.c_int32(taps), _ptr(in_perm), ctypes.c_uint32(flags), ctypes.byref(h)))
    else:
        _check(_lib.rmsmp_pack_weights(_ptr(W), ctypes.c_int64(M), ctypes.c_int64(K), _ptr(scheme), _ptr(alpha),
                                       ctypes.c_int32(taps), _ptr(in_perm), ctypes.byref(h)))
    return Packed(h, M, K, taps)


def rmsmp_unpack_codes(p):
    out = np.empty((p.M, p.K), np.int8)
    _check(_lib.rmsmp_unpack_codes(p.handle, _ptr(out)))
    return out


def rmsmp_pack_roundtrip_host(W, scheme, alpha=None, taps=1, in_perm=None):
    """No GPU needed.  Returns dict(wint, rowscale, rowsum, perm)."""
    W = _np(W, np.float32)
    M, K = W.shape
    scheme = _np(scheme, np.uint8)
    alpha = None if alpha is None else _np(alpha, np.float32)
    in_perm = None if in_perm is None else _np(in_perm, np.int32)
    wint = np.empty((M, K), np.int8)
    rowscale = np.empty(M, np.float32)
    rowsum = np.empty(M, np.int32)
    perm = np.empty(M, np.int32)
    _check(_lib.rmsmp_pack_roundtrip_host(_ptr(W), ctypes.c_int64(M), ctypes.c_int64(K), _ptr(scheme), _ptr(alpha),
                                          ctypes.c_int32(taps), _ptr(in_perm), _ptr(wint), _ptr(rowscale),
                                          _ptr(rowsum), _ptr(perm)))
    return dict(wint=wint, rowscale=rowscale, rowsum=rowsum, perm=perm)


def make_epilogue(act_scale=1.0, act_zero_point=0, act_bits=4, bias=None, relu=False, out_kind=OUT_INT32,
                  out_inv_scale=1.0, out_zero_point=0):
    return Epilogue(float(act_scale), int(act_zero_point), int(act_bits),
                    None if bias is None else bias.data_ptr(), 1 if relu else 0, int(out_kind),
                    float(out_inv_scale), int(out_zero_point))


def rmsmp_gemm(p, X, N, ep, Y, stream=None):
    _check(_lib.rmsmp_gemm(p.handle, _dev(X), ctypes.c_int64(N), ctypes.byref(ep), _dev(Y), _stream(stream)))


def rmsmp_conv2d_workspace_size(p, d, act_bits=4):
    n = ctypes.c_size_t()
    _check(_lib.rmsmp_conv2d_workspace_size(p.handle, ctypes.byref(d), ctypes.c_int32(act_bits), ctypes.byref(n)))
    return int(n.value)


def rmsmp_conv2d(p, X, d, ep, Y, workspace=None, stream=None):
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.rmsmp_conv2d(p.handle, _dev(X), ctypes.byref(d), ctypes.byref(ep), _dev(Y), _dev(workspace),
                             ctypes.c_size_t(wbytes), _stream(stream)))


STATIC_WORKSPACE_BYTES = 16 << 20  # RMSMP_STATIC_WORKSPACE_BYTES


def rmsmp_init():
    _check(_lib.rmsmp_init())


def rmsmp_conv2d_static_workspace(p, X, d, ep, Y, stream=None):
    _check(_lib.rmsmp_conv2d_static_workspace(p.handle, _dev(X), ctypes.byref(d), ctypes.byref(ep), _dev(Y),
                                              _stream(stream)))


def rmsmp_conv2d_pair(pa, da, epa, Ya, pb, db, epb, Yb, X, stream=None):
    """Two convolutions on the same input X, enqueued together (one launch where the library can)."""
    _check(_lib.rmsmp_conv2d_pair(pa.handle, ctypes.byref(da), ctypes.byref(epa), _dev(Ya),
                                  pb.handle, ctypes.byref(db), ctypes.byref(epb), _dev(Yb), _dev(X), _stream(stream)))


def conv2d_pair_launcher(pa, da, epa, Ya, pb, db, epb, Yb, X, stream=None):
    """rmsmp_conv2d_pair with the arguments marshalled once (see conv2d_launcher)."""
    args = (pa.handle, ctypes.byref(da), ctypes.byref(epa), _dev(Ya), pb.handle, ctypes.byref(db), ctypes.byref(epb),
            _dev(Yb), _dev(X), _stream(stream))
    fn = _lib.rmsmp_conv2d_pair

    def launch():
        rc = fn(*args)
        if rc:
            _check(rc)
    launch.keepalive = (pa, da, epa, Ya, pb, db, epb, Yb, X)
    return launch


def conv2d_launcher(p, X, d, ep, Y, workspace=None, stream=None):
    """rmsmp_conv2d with the arguments marshalled once: returns a zero-argument callable that
    enqueues the same call again (for launch-bound loops and graph capture)."""
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    args = (p.handle, _dev(X), ctypes.byref(d), ctypes.byref(ep), _dev(Y), _dev(workspace),
            ctypes.c_size_t(wbytes), _stream(stream))
    fn = _lib.rmsmp_conv2d

    def launch():
        rc = fn(*args)
        if rc:
            _check(rc)
    launch.keepalive = (p, X, d, ep, Y, workspace)
    return launch


def gemm_launcher(p, X, N, ep, Y, stream=None):
    args = (p.handle, _dev(X), ctypes.c_int64(N), ctypes.byref(ep), _dev(Y), _stream(stream))
    fn = _lib.rmsmp_gemm

    def launch():
        rc = fn(*args)
        if rc:
            _check(rc)
    launch.keepalive = (p, X, ep, Y)
    return launch


def rmsmp_fake_quant_rows(W, scheme, What, alpha=None, alpha_out=None, stream=None):
    """Device tensors: W, What fp32 [M][K]; scheme uint8 [M]; alpha / alpha_out fp32 [M] or None."""
    M, K = W.shape
    _check(_lib.rmsmp_fake_quant_rows(_dev(W), ctypes.c_int64(M), ctypes.c_int64(K), _dev(scheme), _dev(alpha),
                                      _dev(What), _dev(alpha_out), _stream(stream)))


def rmsmp_ste_backward(dWhat, dW, W=None, alpha=None, stream=None):
    """Device tensors fp32 [M][K]; W and alpha [M] only when the forward pass was given an alpha."""
    M, K = dWhat.shape
    _check(_lib.rmsmp_ste_backward(_dev(W), _dev(alpha), _dev(dWhat), ctypes.c_int64(M), ctypes.c_int64(K),
                                   _dev(dW), _stream(stream)))


def rmsmp_debug_set_wave_split(pixel_blocks=0, k_split=0, side_by_side=0, tile_pairs=0):
    _check(_lib.rmsmp_debug_set_wave_split(int(pixel_blocks), int(k_split), int(side_by_side), int(tile_pairs)))


KERNEL_NAMES = ("none", "general", "skinny", "rows", "first_layer", "lds_resident", "lds_resident_pair")


def rmsmp_debug_last_dispatch():
    """(kernel name, (pixel_blocks, k_split, side_by_side, tile_pairs)) of this thread's last launch."""
    out = (ctypes.c_int32 * 5)()
    _check(_lib.rmsmp_debug_last_dispatch(out))
    return KERNEL_NAMES[out[0]], tuple(int(v) for v in out[1:])


def rmsmp_debug_gelu_breakpoints(out_inv_scale, out_zero_point):
    """No GPU needed.  dict(rise[16], fall[16], y_split, fall_base, n_fall) of the GELU epilogue."""
    rise, fall = np.empty(16, np.float32), np.empty(16, np.float32)
    ys, fb, nf = ctypes.c_float(), ctypes.c_int32(), ctypes.c_int32()
    _check(_lib.rmsmp_debug_gelu_breakpoints(ctypes.c_float(out_inv_scale), ctypes.c_int32(out_zero_point), _ptr(rise),
                                             _ptr(fall), ctypes.byref(ys), ctypes.byref(fb), ctypes.byref(nf)))
    return dict(rise=rise, fall=fall, y_split=float(ys.value), fall_base=int(fb.value), n_fall=int(nf.value))


def rmsmp_debug_measure_peaks():
    """(MFMA-only int8 TOP/s, copy GB/s read + written) of the current device."""
    a, b = ctypes.c_double(), ctypes.c_double()
    _check(_lib.rmsmp_debug_measure_peaks(ctypes.byref(a), ctypes.byref(b)))
    return float(a.value), float(b.value)


# ---- storage helpers for callers (nibble packing of activation codes; no arithmetic of the method)

def pack_u4(codes):
    """uint8 codes (..., K) with values 0..15 -> (..., K/2) bytes, even index in the low nibble."""
    c = np.ascontiguousarray(codes, dtype=np.uint8)
    if c.shape[-1] % 2:
        raise ValueError("last dimension must be even")
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


def unpack_u4(b):
    b = np.ascontiguousarray(b, dtype=np.uint8)
    out = np.empty(b.shape[:-1] + (b.shape[-1] * 2,), np.uint8)
    out[..., 0::2] = b & 15
    out[..., 1::2] = b >> 4
    return out
