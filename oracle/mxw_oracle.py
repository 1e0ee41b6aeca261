"""ctypes front-end of oracle/mxw_oracle.c: the six- and eight-bit MX / MX+ formats.  Conversion and de-conversion are
computed in the C file; `gemm` forms the float64 matrix product of the de-converted operands with numpy (the plain
definition of the product)."""
import ctypes as C

import numpy as np

from . import build as _build

MXFP6 = 3
MXFP6P = 4
MXFP8 = 5
MXFP8P = 6

_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = C.CDLL(_build.build())
        u8p, f32p, u16p, f64p = (C.POINTER(C.c_uint8), C.POINTER(C.c_float), C.POINTER(C.c_uint16),
                                 C.POINTER(C.c_double))
        i64 = C.c_int64
        lib.mxw_quantize_f32.argtypes = [f32p, i64, i64, i64, C.c_int, u8p, u8p, u8p]
        lib.mxw_quantize_bf16.argtypes = [u16p, i64, i64, i64, C.c_int, u8p, u8p, u8p]
        lib.mxw_dequantize.argtypes = [u8p, u8p, u8p, C.c_int, i64, i64, f64p, i64]
        lib.mxw_encode_block.argtypes = [f32p, C.c_int, u8p, u8p, u8p]
        lib.mxw_decode_block.argtypes = [u8p, C.c_uint8, C.c_uint8, C.c_int, f64p]
        lib.mxw_elem_bytes_per_block.argtypes = [C.c_int]
        for n in ("mxw_quantize_f32", "mxw_quantize_bf16", "mxw_dequantize", "mxw_encode_block", "mxw_decode_block",
                  "mxw_elem_bytes_per_block"):
            getattr(lib, n).restype = C.c_int
        _lib = lib
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def block_bytes(fmt):
    n = _L().mxw_elem_bytes_per_block(fmt)
    if n < 0:
        raise ValueError("not a six- or eight-bit format: %r" % (fmt,))
    return n


def quantize(x, fmt):
    """x: [rows, K] float32 or uint16 (bf16 bits).  Returns (elems [rows, K/32 * block_bytes] u8, scales, idx)."""
    x = np.asarray(x)
    assert x.ndim == 2 and x.strides[1] == x.itemsize
    rows, K = x.shape
    ld = x.strides[0] // x.itemsize if rows > 1 else K
    bb = block_bytes(fmt)
    elems = np.zeros((rows, K // 32 * bb), np.uint8)
    scales = np.zeros((rows, K // 32), np.uint8)
    idx = np.zeros((rows, K // 32), np.uint8)
    if x.dtype == np.float32:
        rc = _L().mxw_quantize_f32(_p(x, C.c_float), rows, K, ld, fmt, _p(elems, C.c_uint8), _p(scales, C.c_uint8),
                                   _p(idx, C.c_uint8))
    elif x.dtype == np.uint16:
        rc = _L().mxw_quantize_bf16(_p(x, C.c_uint16), rows, K, ld, fmt, _p(elems, C.c_uint8), _p(scales, C.c_uint8),
                                    _p(idx, C.c_uint8))
    else:
        raise TypeError("oracle input must be float32 or uint16 (bf16 bits), got %s" % x.dtype)
    if rc:
        raise ValueError("oracle quantize: bad shape or format")
    return elems, scales, idx


def dequantize(q, fmt):
    e, s, i = (np.ascontiguousarray(a, dtype=np.uint8) for a in q)
    rows, nb = s.shape
    assert e.shape == (rows, nb * block_bytes(fmt))
    out = np.zeros((rows, nb * 32), np.float64)
    rc = _L().mxw_dequantize(_p(e, C.c_uint8), _p(s, C.c_uint8), _p(i, C.c_uint8), fmt, rows, nb * 32,
                             _p(out, C.c_double), nb * 32)
    assert rc == 0
    return out


def encode_block(x32, fmt):
    """One block -> (codes[32] unpacked, scale byte, index byte)."""
    x = np.ascontiguousarray(x32, dtype=np.float32)
    assert x.shape == (32,)
    codes = np.zeros(32, np.uint8)
    s = C.c_uint8(0)
    i = C.c_uint8(0)
    rc = _L().mxw_encode_block(_p(x, C.c_float), fmt, _p(codes, C.c_uint8), C.byref(s), C.byref(i))
    assert rc == 0
    return codes, s.value, i.value


def decode_block(codes32, scale, idx, fmt):
    c = np.ascontiguousarray(codes32, dtype=np.uint8)
    assert c.shape == (32,)
    out = np.zeros(32, np.float64)
    rc = _L().mxw_decode_block(_p(c, C.c_uint8), int(scale), int(idx), fmt, _p(out, C.c_double))
    assert rc == 0
    return out


def gemm(qa, fmt_a, qb, fmt_b):
    """The product of two six- or eight-bit operands is the matrix product of their de-converted values (Sec. 5.1,
    with the BM taken at its full precision as Sec. 6.2 defines the result): D = deq(A) deq(B)^T in float64 and
    S = |deq(A)| |deq(B)|^T.  A: [M, K], B: [N, K]."""
    a = dequantize(qa, fmt_a)
    b = dequantize(qb, fmt_b)
    assert a.shape[1] == b.shape[1]
    return a @ b.T, np.abs(a) @ np.abs(b).T
