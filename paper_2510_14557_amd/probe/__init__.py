"""Binding of the bench-only MFMA probe (libmxp_probe.so, probe/mxp_probe.h).  Not part of the product: only bench.py uses it."""
from __future__ import annotations

import ctypes as C
import os

import torch

from .. import mxp

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmxp_probe.so")
FLOP_PER_ITER = 256 * 4 * 16 * 2 * 32 * 32 * 64
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise mxp.MxpError("libmxp_probe.so is not built: run paper_2510_14557_amd/build.py")
        L = C.CDLL(LIB_PATH)
        vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int
        L.mxp_probe_mfma.argtypes = [i32, i32, i32, C.c_uint32, vp, vp]
        L.mxp_probe_mfma.restype = i32
        L.mxp_probe_mfma_images.argtypes = [vp, i32, i64, vp, i32, i64, i64, i32, vp, vp]
        L.mxp_probe_mfma_images.restype = i32
        _lib = L
    return _lib


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def mfma(iters: int, a_kind: int = mxp.IMAGE_E2M3, b_kind: int = mxp.IMAGE_E2M3, seed: int = 1, sink: torch.Tensor | None = None):
    """MFMAs only, on register-resident pseudo-random operands (FLOP_PER_ITER flop per iteration)."""
    if sink is None:
        sink = torch.empty(65536, dtype=torch.float32, device="cuda")
    rc = lib().mxp_probe_mfma(a_kind, b_kind, iters, seed, C.c_void_p(sink.data_ptr()), _stream())
    if rc != 0:
        raise mxp.MxpError("mxp_probe_mfma: status %d" % rc)
    return sink


def mfma_images(iters: int, a_image: torch.Tensor, a_kind: int, rows_a: int, b_image: torch.Tensor, b_kind: int, rows_b: int, K: int,
                sink: torch.Tensor | None = None):
    """The same loop on operand bits loaded once from two real images."""
    if sink is None:
        sink = torch.empty(65536, dtype=torch.float32, device="cuda")
    rc = lib().mxp_probe_mfma_images(C.c_void_p(a_image.data_ptr()), a_kind, rows_a, C.c_void_p(b_image.data_ptr()), b_kind, rows_b, K,
                                     iters, C.c_void_p(sink.data_ptr()), _stream())
    if rc != 0:
        raise mxp.MxpError("mxp_probe_mfma_images: status %d" % rc)
    return sink
