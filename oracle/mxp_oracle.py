"""ctypes front-end of oracle/mxp_oracle.c.  Conversion, de-conversion and the MX x MX product are computed in the C
file; this module marshals arguments, and `gemm_w4a16` additionally forms its float64 matrix product with numpy (the
plain definition, on operands the C file de-converted)."""
import ctypes as C
import os

import numpy as np

from . import build as _build

MXFP4 = 0
MXFP4P = 1
MXFP4PP = 2

_lib = None


def _L():
    global _lib
    if _lib is None:
        path = _build.build()
        lib = C.CDLL(path)
        u8p, f32p, u16p, f64p, i64p = (C.POINTER(C.c_uint8), C.POINTER(C.c_float), C.POINTER(C.c_uint16),
                                       C.POINTER(C.c_double), C.POINTER(C.c_int64))
        i64 = C.c_int64
        for name, sp in (("mxo_quantize_f32", f32p), ("mxo_quantize_bf16", u16p),
                         ("mxo_quantize_t_f32", f32p), ("mxo_quantize_t_bf16", u16p)):
            fn = getattr(lib, name)
            fn.argtypes = [sp, i64, i64, i64, C.c_int, u8p, u8p, u8p]
            fn.restype = C.c_int
        lib.mxo_dequantize.argtypes = [u8p, u8p, u8p, C.c_int, i64, i64, f64p, i64]
        lib.mxo_dequantize.restype = C.c_int
        lib.mxo_gemm.argtypes = [i64, i64, i64, u8p, u8p, u8p, C.c_int, u8p, u8p, u8p, C.c_int, f64p, f64p]
        lib.mxo_gemm.restype = C.c_int
        lib.mxo_gemm_sampled.argtypes = [i64, i64p, i64p, i64, u8p, u8p, u8p, C.c_int, u8p, u8p, u8p, C.c_int,
                                         f64p, f64p]
        lib.mxo_gemm_sampled.restype = C.c_int
        lib.mxo_encode_block.argtypes = [f32p, C.c_int, u8p, u8p, u8p]
        lib.mxo_encode_block.restype = None
        lib.mxo_decode_block.argtypes = [u8p, C.c_uint8, C.c_uint8, C.c_int, f64p]
        lib.mxo_decode_block.restype = None
        lib.mxo_num_threads.restype = C.c_int
        _lib = lib
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _src(x):
    """fp32 array, or bf16 given as a uint16 array of bit patterns."""
    x = np.asarray(x)
    if x.dtype == np.float32:
        return x, "f32", C.c_float
    if x.dtype == np.uint16:
        return x, "bf16", C.c_uint16
    raise TypeError("oracle input must be float32 or uint16 (bf16 bits), got %s" % x.dtype)


def quantize(x, fmt=MXFP4P):
    """x: [rows, K] (row stride may exceed K).  Returns (elems [rows,K/2] u8, scales [rows,K/32] u8, idx [rows,K/32] u8)."""
    x, kind, ct = _src(x)
    assert x.ndim == 2 and x.strides[1] == x.itemsize
    rows, K = x.shape
    ld = x.strides[0] // x.itemsize if rows > 1 else K
    elems = np.zeros((rows, K // 2), np.uint8)
    scales = np.zeros((rows, K // 32), np.uint8)
    idx = np.zeros((rows, K // 32), np.uint8)
    rc = getattr(_L(), "mxo_quantize_" + kind)(_p(x, ct), rows, K, ld, fmt, _p(elems, C.c_uint8),
                                               _p(scales, C.c_uint8), _p(idx, C.c_uint8))
    if rc:
        raise ValueError("oracle quantize: bad shape rows=%d K=%d" % (rows, K))
    return elems, scales, idx


def quantize_t(xt, fmt=MXFP4P):
    """xt: [K, rows] C-contiguous (the operand stored K-strided).  Same outputs as quantize(xt.T)."""
    xt, kind, ct = _src(xt)
    assert xt.ndim == 2 and xt.flags.c_contiguous
    K, rows = xt.shape
    elems = np.zeros((rows, K // 2), np.uint8)
    scales = np.zeros((rows, K // 32), np.uint8)
    idx = np.zeros((rows, K // 32), np.uint8)
    rc = getattr(_L(), "mxo_quantize_t_" + kind)(_p(xt, ct), rows, K, rows, fmt, _p(elems, C.c_uint8),
                                                 _p(scales, C.c_uint8), _p(idx, C.c_uint8))
    if rc:
        raise ValueError("oracle quantize_t: bad shape rows=%d K=%d" % (rows, K))
    return elems, scales, idx


def _q3(q):
    e, s, i = (np.ascontiguousarray(a, dtype=np.uint8) for a in q)
    return e, s, i


def dequantize(q, fmt=MXFP4P):
    """q = (elems, scales, idx).  Returns float64 [rows, K] (every value is exactly representable in bf16)."""
    e, s, i = _q3(q)
    rows, K = e.shape[0], e.shape[1] * 2
    out = np.zeros((rows, K), np.float64)
    rc = _L().mxo_dequantize(_p(e, C.c_uint8), _p(s, C.c_uint8), _p(i, C.c_uint8), fmt, rows, K,
                             _p(out, C.c_double), K)
    assert rc == 0
    return out


def gemm(qa, fmt_a, qb, fmt_b):
    """D[m,n] = sum_k deq(A)[m,k] deq(B)[n,k] (float64) and S[m,n] = sum_k |a b|.  A: [M,K], B: [N,K]."""
    ae, as_, ai = _q3(qa)
    be, bs, bi = _q3(qb)
    M, K = ae.shape[0], ae.shape[1] * 2
    N = be.shape[0]
    assert be.shape[1] * 2 == K
    D = np.zeros((M, N), np.float64)
    S = np.zeros((M, N), np.float64)
    rc = _L().mxo_gemm(M, N, K, _p(ae, C.c_uint8), _p(as_, C.c_uint8), _p(ai, C.c_uint8), fmt_a,
                       _p(be, C.c_uint8), _p(bs, C.c_uint8), _p(bi, C.c_uint8), fmt_b,
                       _p(D, C.c_double), _p(S, C.c_double))
    assert rc == 0
    return D, S


def gemm_w4a16(a, qw, fmt_w):
    """Conversion-based product (Sec. 5: blocks de-converted to a wider type and multiplied there): the activations are
    taken as they are (bf16 bit patterns as uint16, or float32), the weights are de-converted by Eq. 2, and the product
    is the plain float64 matrix product.  Returns D[M,N] = a @ deq(W)^T and S = |a| @ |deq(W)|^T."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        a = (a.astype(np.uint32) << 16).view(np.float32)
    a64 = a.astype(np.float64)
    w64 = dequantize(qw, fmt_w)
    assert a64.shape[1] == w64.shape[1]
    return a64 @ w64.T, np.abs(a64) @ np.abs(w64).T


def gemm_sampled(qa, fmt_a, qb, fmt_b, rows_m, rows_n):
    """D[t] = <A[rows_m[t]], B[rows_n[t]]> and S[t], for sampled output positions."""
    ae, as_, ai = _q3(qa)
    be, bs, bi = _q3(qb)
    K = ae.shape[1] * 2
    assert be.shape[1] * 2 == K
    rm = np.ascontiguousarray(rows_m, dtype=np.int64)
    rn = np.ascontiguousarray(rows_n, dtype=np.int64)
    assert rm.shape == rn.shape and rm.ndim == 1
    assert rm.size == 0 or (0 <= rm.min() and rm.max() < ae.shape[0] and 0 <= rn.min() and rn.max() < be.shape[0])
    D = np.zeros(rm.size, np.float64)
    S = np.zeros(rm.size, np.float64)
    rc = _L().mxo_gemm_sampled(rm.size, _p(rm, C.c_int64), _p(rn, C.c_int64), K,
                               _p(ae, C.c_uint8), _p(as_, C.c_uint8), _p(ai, C.c_uint8), fmt_a,
                               _p(be, C.c_uint8), _p(bs, C.c_uint8), _p(bi, C.c_uint8), fmt_b,
                               _p(D, C.c_double), _p(S, C.c_double))
    assert rc == 0
    return D, S


def encode_block(x32, fmt=MXFP4P):
    x = np.ascontiguousarray(x32, dtype=np.float32)
    assert x.shape == (32,)
    e = np.zeros(16, np.uint8)
    s = C.c_uint8(0)
    i = C.c_uint8(0)
    _L().mxo_encode_block(_p(x, C.c_float), fmt, _p(e, C.c_uint8), C.byref(s), C.byref(i))
    return e, s.value, i.value


def decode_block(elems16, scale, idx, fmt=MXFP4P):
    e = np.ascontiguousarray(elems16, dtype=np.uint8)
    assert e.shape == (16,)
    out = np.zeros(32, np.float64)
    _L().mxo_decode_block(_p(e, C.c_uint8), int(scale), int(idx), fmt, _p(out, C.c_double))
    return out


def num_threads():
    return int(_L().mxo_num_threads())
