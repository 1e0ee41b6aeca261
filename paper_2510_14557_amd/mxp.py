"""Thin Python binding over the C-ABI HIP library (include/mxp.h): argument marshalling only.

Every function here has the name of the C entry point it calls (minus the `mxp_` prefix).  torch supplies device
memory and the current stream; nothing is computed in Python and there is no fallback path: if libmxp.so is missing
or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

F32, BF16 = 0, 1
MXFP4, MXFP4P, MXFP4PP = 0, 1, 2
MXFP6, MXFP6P, MXFP8, MXFP8P = 3, 4, 5, 6          # conversion and de-conversion only
_CODE_BITS = {MXFP4: 4, MXFP4P: 4, MXFP4PP: 4, MXFP6: 6, MXFP6P: 6, MXFP8: 8, MXFP8P: 8}
IMAGE_E2M3, IMAGE_E2M1, IMAGE_E4M3, IMAGE_E2M1R, IMAGE_E2M1X = 0, 1, 2, 3, 4

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmxp.so")

EXPORTS = ("mxp_quantize", "mxp_quantize_t", "mxp_quantize_gather", "mxp_dequantize", "mxp_image_bytes", "mxp_prepack", "mxp_quantize_image",
           "mxp_image_bytes_e2m1", "mxp_prepack_e2m1", "mxp_image_bytes_e2m1r", "mxp_prepack_e2m1r", "mxp_prepack_e2m1x", "mxp_image_bytes_e4m3", "mxp_prepack_e4m3", "mxp_gemm_workspace_bytes", "mxp_gemm_workspace_bytes_e4m3", "mxp_gemm_workspace_bytes_fmt", "mxp_image_bytes_fp6", "mxp_prepack_fp6", "mxp_quantize_image_fp6", "mxp_prepack_seg", "mxp_prepack_fp8", "mxp_gemm", "mxp_gemm_prepacked", "mxp_gemm_bf16a_workspace_bytes", "mxp_gemm_decode", "mxp_gemm_decode_bf16a",
           "mxp_gemm_bf16a", "mxp_gemm_w4a16", "mxp_convert_operands", "mxp_gemm_workspace_size", "mxp_gemm_static", "mxp_gemm_static_capacity", "mxp_status_string", "mxp_version")

_lib = None


class MxpError(RuntimeError):
    pass


def lib():
    """Load libmxp.so once (after torch, so both share one HIP runtime) and declare the signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise MxpError("libmxp.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                       "or `python paper_2510_14557_amd/build.py` (needs hipcc)")
    L = C.CDLL(LIB_PATH)
    vp, i64, i32, sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
    L.mxp_quantize.argtypes = [vp, i32, i64, i64, i64, i32, vp, vp, vp, vp]
    L.mxp_quantize_t.argtypes = [vp, i32, i64, i64, i64, i32, vp, vp, vp, vp]
    L.mxp_quantize_gather.argtypes = [vp, i32, i64, i64, i64, i64, vp, i32, vp, vp, vp, vp]
    L.mxp_quantize_gather.restype = i32
    L.mxp_dequantize.argtypes = [vp, vp, vp, i32, i64, i64, vp, i32, i64, vp]
    L.mxp_image_bytes.argtypes = [i64, i64]
    L.mxp_image_bytes.restype = sz
    L.mxp_prepack.argtypes = [vp, vp, vp, i32, i64, i64, vp, sz, vp]
    L.mxp_quantize_image.argtypes = [vp, i32, i64, i64, i64, i32, vp, vp, vp, vp, sz, vp]
    L.mxp_gemm_workspace_bytes.argtypes = [i64, i64, i64]
    L.mxp_gemm_workspace_bytes.restype = sz
    L.mxp_gemm_workspace_bytes_e4m3.argtypes = [i64, i64, i64]
    L.mxp_gemm_workspace_bytes_e4m3.restype = sz
    L.mxp_gemm.argtypes = [i64, i64, i64, vp, vp, vp, i32, vp, vp, vp, i32, vp, i32, i64, vp, sz, vp]
    L.mxp_gemm_prepacked.argtypes = [i64, i64, i64, vp, i32, vp, i32, vp, i32, i64, vp]
    L.mxp_gemm_decode.argtypes = [i64, i64, i64, vp, vp, vp, vp, i32, vp, i32, i64, vp]
    L.mxp_gemm_decode_bf16a.argtypes = [i64, i64, i64, vp, i32, i64, i32, vp, vp, vp, i32, vp, i32, i64, vp, sz, vp]
    L.mxp_image_bytes_e2m1.argtypes = [i64, i64]
    L.mxp_image_bytes_e2m1.restype = sz
    L.mxp_prepack_e2m1.argtypes = [vp, vp, i64, i64, vp, sz, vp]
    L.mxp_image_bytes_e2m1r.argtypes = [i64, i64]
    L.mxp_image_bytes_e2m1r.restype = sz
    L.mxp_prepack_e2m1r.argtypes = [vp, vp, vp, i64, i64, vp, sz, vp]
    L.mxp_prepack_e2m1r.restype = i32
    L.mxp_prepack_e2m1x.argtypes = [vp, vp, vp, i32, i64, i64, vp, sz, vp]
    L.mxp_prepack_e2m1x.restype = i32
    L.mxp_image_bytes_e4m3.argtypes = [i64, i64]
    L.mxp_image_bytes_e4m3.restype = sz
    L.mxp_prepack_e4m3.argtypes = [vp, vp, vp, i32, i64, i64, vp, sz, vp]
    L.mxp_gemm_workspace_bytes_fmt.argtypes = [i64, i64, i64, i32, i32]
    L.mxp_gemm_workspace_bytes_fmt.restype = sz
    L.mxp_image_bytes_fp6.argtypes = [i64, i64, i32]
    L.mxp_image_bytes_fp6.restype = sz
    L.mxp_prepack_fp6.argtypes = [vp, vp, vp, i32, i64, i64, i32, C.c_uint, vp, sz, vp]
    L.mxp_prepack_fp6.restype = i32
    L.mxp_quantize_image_fp6.argtypes = [vp, i32, i64, i64, i64, i32, i32, C.c_uint, vp, vp, vp, vp, sz, vp]
    L.mxp_quantize_image_fp6.restype = i32
    L.mxp_prepack_seg.argtypes = [vp, vp, vp, i32, i64, i64, i32, C.c_uint, vp, sz, vp]
    L.mxp_prepack_seg.restype = i32
    L.mxp_prepack_fp8.argtypes = [vp, vp, i64, i64, vp, sz, vp]
    L.mxp_prepack_fp8.restype = i32
    L.mxp_gemm_bf16a_workspace_bytes.argtypes = [i64, i64]
    L.mxp_gemm_bf16a_workspace_bytes.restype = sz
    L.mxp_gemm_bf16a.argtypes = [i64, i64, i64, vp, i32, i64, i32, vp, i32, vp, i32, i64, vp, sz, vp]
    L.mxp_gemm_w4a16.argtypes = [i64, i64, i64, vp, i32, i64, vp, vp, vp, i32, vp, i32, i64, vp]
    L.mxp_gemm_w4a16.restype = i32
    L.mxp_convert_operands.argtypes = [vp, i32, i64, i64, i64, i32, vp, vp, vp, vp, sz, vp, vp, vp, i32, i64, vp, sz, vp]
    L.mxp_convert_operands.restype = i32
    L.mxp_gemm_static.argtypes = [i64, i64, i64, vp, vp, vp, i32, vp, vp, vp, i32, vp, i32, i64, vp]
    L.mxp_gemm_static.restype = i32
    L.mxp_gemm_static_capacity.argtypes = []
    L.mxp_gemm_static_capacity.restype = sz
    L.mxp_gemm_workspace_size.argtypes = [i64, i64, i64, i32, i32]
    L.mxp_gemm_workspace_size.restype = sz
    L.mxp_status_string.argtypes = [i32]
    L.mxp_status_string.restype = C.c_char_p
    L.mxp_version.restype = i32
    for n in ("mxp_quantize", "mxp_quantize_t", "mxp_dequantize", "mxp_prepack", "mxp_quantize_image", "mxp_prepack_e2m1", "mxp_prepack_e4m3", "mxp_gemm", "mxp_gemm_prepacked",
              "mxp_gemm_bf16a", "mxp_gemm_decode", "mxp_gemm_decode_bf16a"):
        getattr(L, n).restype = i32
    _lib = L
    return L


def status_string(rc: int) -> str:
    return lib().mxp_status_string(rc).decode()


def version() -> int:
    return lib().mxp_version()


def _check(rc: int, what: str):
    if rc != 0:
        raise MxpError("%s failed: %s (%d)" % (what, status_string(rc), rc))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("expected float32 or bfloat16, got %s" % t.dtype)


def _dev2d(t: torch.Tensor):
    if not t.is_cuda:
        raise MxpError("tensor must live on the GPU")
    if t.dim() != 2 or t.stride(1) != 1:
        raise MxpError("expected a 2-D tensor with unit inner stride")
    return t


def _p(t):
    return None if t is None else t.data_ptr()


def quantize(x: torch.Tensor, fmt: int = MXFP4P):
    """x [rows, K] fp32/bf16 on the GPU -> (elems [rows, K*bits/8], scales [rows,K/32], bm_idx [rows,K/32]) uint8."""
    _dev2d(x)
    rows, K = x.shape
    ld = x.stride(0) if rows > 1 else max(K, 1)
    elems = torch.empty((rows, K * _CODE_BITS.get(fmt, 4) // 8), dtype=torch.uint8, device=x.device)
    scales = torch.empty((rows, K // 32), dtype=torch.uint8, device=x.device)
    idx = torch.empty((rows, K // 32), dtype=torch.uint8, device=x.device)
    _check(lib().mxp_quantize(_p(x), _dt(x), rows, K, ld, fmt, _p(elems), _p(scales), _p(idx), _stream()), "mxp_quantize")
    return elems, scales, idx


def quantize_into(x, fmt, elems, scales, idx):
    """Same, into caller-provided buffers (no allocation)."""
    rows, K = x.shape
    ld = x.stride(0) if rows > 1 else max(K, 1)
    _check(lib().mxp_quantize(_p(x), _dt(x), rows, K, ld, fmt, _p(elems), _p(scales), _p(idx), _stream()), "mxp_quantize")


def quantize_gather(x: torch.Tensor, perm: torch.Tensor, fmt: int = MXFP4P):
    """Rows of x with their channels reordered: output element k is x[:, perm[k]] (perm int32 on the GPU, length K)."""
    _dev2d(x)
    if perm.dtype != torch.int32 or not perm.is_cuda or perm.dim() != 1 or not perm.is_contiguous():
        raise MxpError("perm must be a contiguous 1-D int32 tensor on the GPU")
    rows, n_src = x.shape
    K = perm.numel()
    ld = x.stride(0) if rows > 1 else max(n_src, 1)
    elems = torch.empty((rows, K // 2), dtype=torch.uint8, device=x.device)
    scales = torch.empty((rows, K // 32), dtype=torch.uint8, device=x.device)
    idx = torch.empty((rows, K // 32), dtype=torch.uint8, device=x.device)
    _check(lib().mxp_quantize_gather(_p(x), _dt(x), rows, K, n_src, ld, _p(perm), fmt, _p(elems), _p(scales), _p(idx), _stream()),
           "mxp_quantize_gather")
    return elems, scales, idx


def quantize_t(xt: torch.Tensor, fmt: int = MXFP4P):
    """xt [K, rows] (the operand stored K-strided).  Same outputs as quantize(xt.T)."""
    _dev2d(xt)
    K, rows = xt.shape
    ld = xt.stride(0) if K > 1 else max(rows, 1)
    elems = torch.empty((rows, K // 2), dtype=torch.uint8, device=xt.device)
    scales = torch.empty((rows, K // 32), dtype=torch.uint8, device=xt.device)
    idx = torch.empty((rows, K // 32), dtype=torch.uint8, device=xt.device)
    _check(lib().mxp_quantize_t(_p(xt), _dt(xt), rows, K, ld, fmt, _p(elems), _p(scales), _p(idx), _stream()),
           "mxp_quantize_t")
    return elems, scales, idx


def dequantize(q, fmt: int = MXFP4P, dtype: torch.dtype = torch.float32, out: torch.Tensor | None = None):
    elems, scales, idx = q
    rows, K = elems.shape[0], elems.shape[1] * 8 // _CODE_BITS.get(fmt, 4)
    if out is None:
        out = torch.empty((rows, K), dtype=dtype, device=elems.device)
    ld = out.stride(0) if rows > 1 else max(K, 1)
    _check(lib().mxp_dequantize(_p(elems), _p(scales), _p(idx), fmt, rows, K, _p(out), _dt(out), ld, _stream()),
           "mxp_dequantize")
    return out


def image_bytes(rows: int, K: int) -> int:
    return int(lib().mxp_image_bytes(rows, K))


def prepack(q, fmt: int = MXFP4P, out: torch.Tensor | None = None):
    elems, scales, idx = q
    rows, K = elems.shape[0], elems.shape[1] * 2
    n = image_bytes(rows, K)
    if out is None:
        out = torch.empty(n, dtype=torch.uint8, device=elems.device)
    _check(lib().mxp_prepack(_p(elems), _p(scales), _p(idx), fmt, rows, K, _p(out), out.numel(), _stream()), "mxp_prepack")
    return out


def quantize_image(x: torch.Tensor, fmt: int = MXFP4P, canonical: bool = False, out=None, q_out=None):
    """x [rows, K] fp32/bf16 -> MFMA-ready image (E4M3 for MXFP4PP, else E2M3); with canonical=True also
    (elems, scales, bm_idx), from the same pass."""
    _dev2d(x)
    rows, K = x.shape
    ld = x.stride(0) if rows > 1 else max(K, 1)
    if out is None:
        nbytes = image_bytes_e4m3(rows, K) if fmt == MXFP4PP else image_bytes(rows, K)
        out = torch.empty(nbytes, dtype=torch.uint8, device=x.device)
    q = (None, None, None)
    if q_out is not None:
        q = q_out
    elif canonical:
        q = (torch.empty((rows, K // 2), dtype=torch.uint8, device=x.device),
             torch.empty((rows, K // 32), dtype=torch.uint8, device=x.device),
             torch.empty((rows, K // 32), dtype=torch.uint8, device=x.device))
    _check(lib().mxp_quantize_image(_p(x), _dt(x), rows, K, ld, fmt, _p(q[0]), _p(q[1]), _p(q[2]), _p(out), out.numel(),
                                    _stream()), "mxp_quantize_image")
    return (out, q) if (canonical or q_out is not None) else out


def convert_operands(a: torch.Tensor, fmt_a: int, q_out, a_image: torch.Tensor, qw, fmt_w: int, w_image: torch.Tensor):
    """One launch: activations -> (canonical arrays q_out, or None) + E2M3 image; canonical weights qw -> E2M3 image."""
    _dev2d(a)
    M, K = a.shape
    ae, as_, ai = q_out if q_out is not None else (None, None, None)
    we, ws, wi = qw
    N = we.shape[0]
    lda = a.stride(0) if M > 1 else max(K, 1)
    _check(lib().mxp_convert_operands(_p(a), _dt(a), M, K, lda, fmt_a, _p(ae), _p(as_), _p(ai), _p(a_image), a_image.numel(),
                                      _p(we), _p(ws), _p(wi), fmt_w, N, _p(w_image), w_image.numel(), _stream()),
           "mxp_convert_operands")
    return a_image, w_image


def image_bytes_e2m1(rows: int, K: int) -> int:
    return int(lib().mxp_image_bytes_e2m1(rows, K))


def image_bytes_e4m3(rows: int, K: int) -> int:
    return int(lib().mxp_image_bytes_e4m3(rows, K))


def prepack_e4m3(q, fmt: int = MXFP4PP, out: torch.Tensor | None = None):
    """Canonical MXFP4 / MXFP4+ / MXFP4++ -> E4M3 image (the kind that carries MXFP4++ operands)."""
    elems, scales, idx = q
    rows, K = elems.shape[0], elems.shape[1] * 2
    if out is None:
        out = torch.empty(image_bytes_e4m3(rows, K), dtype=torch.uint8, device=elems.device)
    _check(lib().mxp_prepack_e4m3(_p(elems), _p(scales), _p(idx), fmt, rows, K, _p(out), out.numel(), _stream()), "mxp_prepack_e4m3")
    return out


def image_bytes_fp6(rows: int, K: int, n_seg: int = 1) -> int:
    return int(lib().mxp_image_bytes_fp6(rows, K, n_seg))


def prepack_fp6(q, fmt: int = MXFP6P, n_seg: int = 1, res_mask: int = 0, out: torch.Tensor | None = None):
    """Canonical MXFP6 / MXFP6+ -> E2M3 image of n_seg K segments (each K rounded up to 128 wide); bit s of res_mask makes
    segment s the BM residual instead of the primary operand."""
    elems, scales, idx = q
    rows, K = elems.shape[0], scales.shape[1] * 32
    if out is None:
        out = torch.empty(image_bytes_fp6(rows, K, n_seg), dtype=torch.uint8, device=elems.device)
    _check(lib().mxp_prepack_fp6(_p(elems), _p(scales), _p(idx), fmt, rows, K, n_seg, res_mask, _p(out), out.numel(), _stream()),
           "mxp_prepack_fp6")
    return out


def quantize_image_fp6(x: torch.Tensor, fmt: int = MXFP6P, n_seg: int = 1, res_mask: int = 0, canonical: bool = False,
                       out: torch.Tensor | None = None):
    """bf16 / fp32 rows -> the K-segment E2M3 image of prepack_fp6 in one pass; with canonical=True also the canonical
    (elems, scales, idx) arrays.  Returns image, or (image, q)."""
    _dev2d(x)
    rows, K = x.shape
    if out is None:
        out = torch.empty(image_bytes_fp6(rows, K, n_seg), dtype=torch.uint8, device=x.device)
    q = None
    if canonical:
        q = (torch.empty((rows, K // 32 * 24), dtype=torch.uint8, device=x.device), torch.empty((rows, K // 32), dtype=torch.uint8, device=x.device),
             torch.zeros((rows, K // 32), dtype=torch.uint8, device=x.device))
    e, s_, i = q if q is not None else (None, None, None)
    ld = x.stride(0) if rows > 1 else max(K, 1)
    _check(lib().mxp_quantize_image_fp6(_p(x), _dt(x), rows, K, ld, fmt, n_seg, res_mask, _p(e), _p(s_), _p(i if fmt == MXFP6P else None),
                                        _p(out), out.numel(), _stream()), "mxp_quantize_image_fp6")
    return (out, q) if canonical else out


def prepack_seg(q, fmt: int, n_seg: int, roles: int, out: torch.Tensor | None = None):
    """Canonical MXFP4 / MXFP4+ / MXFP4++ -> E2M3 image of n_seg K segments; two bits of `roles` per segment: 0 the whole
    operand, 1 all elements but the BM (scale lowered by delta), 2 the BM alone."""
    elems, scales, idx = q
    rows, K = elems.shape[0], scales.shape[1] * 32
    if out is None:
        out = torch.empty(image_bytes_fp6(rows, K, n_seg), dtype=torch.uint8, device=elems.device)
    _check(lib().mxp_prepack_seg(_p(elems), _p(scales), _p(idx), fmt, rows, K, n_seg, roles, _p(out), out.numel(), _stream()),
           "mxp_prepack_seg")
    return out


def prepack_fp8(q, out: torch.Tensor | None = None):
    """Canonical plain MXFP8 -> E4M3 image."""
    elems, scales = q[0], q[1]
    rows, K = elems.shape[0], scales.shape[1] * 32
    if out is None:
        out = torch.empty(image_bytes_e4m3(rows, K), dtype=torch.uint8, device=elems.device)
    _check(lib().mxp_prepack_fp8(_p(elems), _p(scales), rows, K, _p(out), out.numel(), _stream()), "mxp_prepack_fp8")
    return out


def prepack_e2m1(q, out: torch.Tensor | None = None):
    """Plain MXFP4 operand (elems, scales[, ignored]) -> E2M1 image for the B side of the product."""
    elems, scales = q[0], q[1]
    rows, K = elems.shape[0], elems.shape[1] * 2
    if out is None:
        out = torch.empty(image_bytes_e2m1(rows, K), dtype=torch.uint8, device=elems.device)
    _check(lib().mxp_prepack_e2m1(_p(elems), _p(scales), rows, K, _p(out), out.numel(), _stream()), "mxp_prepack_e2m1")
    return out


def image_bytes_e2m1r(rows: int, K: int) -> int:
    return int(lib().mxp_image_bytes_e2m1r(rows, K))


def prepack_e2m1r(q, out: torch.Tensor | None = None):
    """MXFP4+ weights -> 4-bit image with residual bytes (IMAGE_E2M1R): the B side of the few-row product."""
    elems, scales, idx = q
    rows, K = elems.shape[0], elems.shape[1] * 2
    if out is None:
        out = torch.empty(image_bytes_e2m1r(rows, K), dtype=torch.uint8, device=elems.device)
    _check(lib().mxp_prepack_e2m1r(_p(elems), _p(scales), _p(idx), rows, K, _p(out), out.numel(), _stream()), "mxp_prepack_e2m1r")
    return out


def prepack_e2m1x(q, fmt: int = MXFP4PP, out: torch.Tensor | None = None):
    """MXFP4+ / MXFP4++ weights -> 4-bit image with index bytes (IMAGE_E2M1X): the B side of the few-row product."""
    elems, scales, idx = q
    rows, K = elems.shape[0], elems.shape[1] * 2
    if out is None:
        out = torch.empty(image_bytes_e2m1r(rows, K), dtype=torch.uint8, device=elems.device)
    _check(lib().mxp_prepack_e2m1x(_p(elems), _p(scales), _p(idx), fmt, rows, K, _p(out), out.numel(), _stream()), "mxp_prepack_e2m1x")
    return out


def gemm_workspace_bytes(M: int, N: int, K: int, fmt_a: int = MXFP4P, fmt_b: int = MXFP4P) -> int:
    return int(lib().mxp_gemm_workspace_bytes_fmt(M, N, K, fmt_a, fmt_b))


def gemm_workspace_size(M: int, N: int, K: int, fmt_a: int = MXFP4P, fmt_b: int = MXFP4P) -> int:
    return int(lib().mxp_gemm_workspace_size(M, N, K, fmt_a, fmt_b))


def gemm(qa, fmt_a, qb, fmt_b, out_dtype: torch.dtype = torch.float32, out: torch.Tensor | None = None,
         workspace: torch.Tensor | None = None):
    """D[M,N] = deq(A)[M,K] @ deq(B)[N,K]^T from canonical operands."""
    ae, as_, ai = qa
    be, bs, bi = qb
    M, K = ae.shape[0], as_.shape[1] * 32
    N = be.shape[0]
    if bs.shape[1] * 32 != K:
        raise MxpError("K mismatch between operands")
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=ae.device)
    if workspace is None:
        workspace = torch.empty(max(gemm_workspace_bytes(M, N, K, fmt_a, fmt_b), 16), dtype=torch.uint8, device=ae.device)
    ldd = out.stride(0) if M > 1 else max(N, 1)
    _check(lib().mxp_gemm(M, N, K, _p(ae), _p(as_), _p(ai), fmt_a, _p(be), _p(bs), _p(bi), fmt_b, _p(out), _dt(out), ldd,
                          _p(workspace), workspace.numel(), _stream()), "mxp_gemm")
    return out


def gemm_static_capacity() -> int:
    return int(lib().mxp_gemm_static_capacity())


def gemm_static(qa, fmt_a, qb, fmt_b, out: torch.Tensor):
    """mxp_gemm with the operand images in the library's built-in scratch array: nothing is allocated, `out` is the caller's."""
    ae, as_, ai = qa
    be, bs, bi = qb
    M, K = ae.shape[0], as_.shape[1] * 32
    N = be.shape[0]
    if bs.shape[1] * 32 != K:
        raise MxpError("K mismatch between operands")
    ldd = out.stride(0) if M > 1 else max(N, 1)
    _check(lib().mxp_gemm_static(M, N, K, _p(ae), _p(as_), _p(ai), fmt_a, _p(be), _p(bs), _p(bi), fmt_b, _p(out), _dt(out), ldd,
                                 _stream()), "mxp_gemm_static")
    return out


def gemm_prepacked(M, N, K, a_image, b_image, out_dtype: torch.dtype = torch.float32, out: torch.Tensor | None = None,
                   b_kind: int = IMAGE_E2M3, a_kind: int = IMAGE_E2M3):
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=a_image.device)
    ldd = out.stride(0) if M > 1 else max(N, 1)
    _check(lib().mxp_gemm_prepacked(M, N, K, _p(a_image), a_kind, _p(b_image), b_kind, _p(out), _dt(out), ldd, _stream()),
           "mxp_gemm_prepacked")
    return out


def gemm_decode(M, N, K, a_image, qw, fmt_w: int = MXFP4P, out_dtype: torch.dtype = torch.float32, out: torch.Tensor | None = None):
    """Few rows (M <= 64) of prepacked activations x canonical weights, widened inside the kernel."""
    we, ws, wi = qw
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=a_image.device)
    ldd = out.stride(0) if M > 1 else max(N, 1)
    _check(lib().mxp_gemm_decode(M, N, K, _p(a_image), _p(we), _p(ws), _p(wi), fmt_w, _p(out), _dt(out), ldd, _stream()),
           "mxp_gemm_decode")
    return out


def gemm_decode_bf16a(a: torch.Tensor, fmt_a: int, qw, fmt_w: int = MXFP4P, out_dtype: torch.dtype = torch.float32,
                      out: torch.Tensor | None = None, workspace: torch.Tensor | None = None):
    """Un-quantized activations (M <= 64 rows), quantized on the fly, x canonical weights."""
    _dev2d(a)
    we, ws, wi = qw
    M, K = a.shape
    N = we.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=a.device)
    if workspace is None:
        workspace = torch.empty(max(gemm_bf16a_workspace_bytes(M, K), 16), dtype=torch.uint8, device=a.device)
    lda = a.stride(0) if M > 1 else max(K, 1)
    ldd = out.stride(0) if M > 1 else max(N, 1)
    _check(lib().mxp_gemm_decode_bf16a(M, N, K, _p(a), _dt(a), lda, fmt_a, _p(we), _p(ws), _p(wi), fmt_w, _p(out), _dt(out), ldd,
                                       _p(workspace), workspace.numel(), _stream()), "mxp_gemm_decode_bf16a")
    return out


def gemm_w4a16(a: torch.Tensor, qw, fmt_w: int = MXFP4P, out_dtype: torch.dtype = torch.float32, out: torch.Tensor | None = None):
    """Un-quantized bf16 activations x canonical weights of any block format, de-converted inside the kernel (4-bit weights:
    few-row kernel for M <= 64; otherwise 256 x 256 tiles on the bf16 MFMA)."""
    _dev2d(a)
    we, ws, wi = qw
    M, K = a.shape
    N = we.shape[0]
    if ws.shape[1] * 32 != K:
        raise MxpError("K mismatch between operands")
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=a.device)
    lda = a.stride(0) if M > 1 else max(K, 1)
    ldd = out.stride(0) if M > 1 else max(N, 1)
    _check(lib().mxp_gemm_w4a16(M, N, K, _p(a), _dt(a), lda, _p(we), _p(ws), _p(wi), fmt_w, _p(out), _dt(out), ldd, _stream()),
           "mxp_gemm_w4a16")
    return out


def gemm_bf16a_workspace_bytes(M: int, K: int) -> int:
    return int(lib().mxp_gemm_bf16a_workspace_bytes(M, K))


def gemm_bf16a(a: torch.Tensor, fmt_a, b_image, N: int, out_dtype: torch.dtype = torch.float32,
               out: torch.Tensor | None = None, workspace: torch.Tensor | None = None, b_kind: int = IMAGE_E2M3):
    """Activations quantized on the fly, weights given as a prepacked image (fmt_a MXFP4PP: b_kind IMAGE_E4M3)."""
    _dev2d(a)
    M, K = a.shape
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=a.device)
    if workspace is None:
        nbytes = image_bytes_e4m3(M, K) if fmt_a == MXFP4PP else gemm_bf16a_workspace_bytes(M, K)
        workspace = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=a.device)
    lda = a.stride(0) if M > 1 else max(K, 1)
    ldd = out.stride(0) if M > 1 else max(N, 1)
    _check(lib().mxp_gemm_bf16a(M, N, K, _p(a), _dt(a), lda, fmt_a, _p(b_image), b_kind, _p(out), _dt(out), ldd,
                                _p(workspace), workspace.numel(), _stream()), "mxp_gemm_bf16a")
    return out
