"""CPU-side checks of the boundary: the library loads, exports every symbol include/mxp.h declares, and rejects bad
arguments with the documented status codes before touching the GPU.  No kernels are launched here."""
import ctypes as C
import os
import re

import pytest

from paper_2510_14557_amd import mxp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mxp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mxp_[a-z0-9_]+)\s*\(", text)))


def test_library_is_built_and_exports_every_declared_symbol():
    assert os.path.exists(mxp.LIB_PATH), "libmxp.so missing: run __graft_entry__.build()"
    L = mxp.lib()
    names = declared_symbols()
    assert set(names) == set(mxp.EXPORTS)
    for n in names:
        assert hasattr(L, n), n
    assert mxp.version() >= 100
    assert mxp.status_string(0) == "ok"
    for rc in range(-9, 0):
        assert mxp.status_string(rc) not in ("ok", "unknown status")


def test_argument_errors_are_reported_not_launched():
    L = mxp.lib()
    buf = (C.c_uint8 * 4096)()
    addr = (C.addressof(buf) + 15) & ~15
    p = C.c_void_p(addr)
    odd = C.c_void_p(addr + 4)
    # K not a multiple of 32
    assert L.mxp_quantize(p, mxp.BF16, 4, 48, 48, mxp.MXFP4P, p, p, p, None) == -2
    # ld smaller than K
    assert L.mxp_quantize(p, mxp.BF16, 4, 64, 32, mxp.MXFP4P, p, p, p, None) == -2
    # null pointers
    assert L.mxp_quantize(None, mxp.BF16, 4, 64, 64, mxp.MXFP4P, p, p, p, None) == -1
    assert L.mxp_quantize(p, mxp.BF16, 4, 64, 64, mxp.MXFP4P, p, p, None, None) == -1
    # misaligned pointer / leading dimension
    assert L.mxp_quantize(odd, mxp.BF16, 4, 64, 64, mxp.MXFP4P, p, p, p, None) == -3
    assert L.mxp_quantize(p, mxp.BF16, 4, 64, 68, mxp.MXFP4P, p, p, p, None) == -3
    # unknown dtype / format
    assert L.mxp_quantize(p, 7, 4, 64, 64, mxp.MXFP4P, p, p, p, None) == -4
    assert L.mxp_quantize(p, mxp.BF16, 4, 64, 64, 9, p, p, p, None) == -5
    assert L.mxp_dequantize(p, p, p, 9, 4, 64, p, mxp.F32, 64, None) == -5
    assert L.mxp_dequantize(p, p, p, mxp.MXFP4P, 4, 64, p, 5, 64, None) == -4
    assert L.mxp_dequantize(p, p, p, mxp.MXFP4P, 4, 40, p, mxp.F32, 64, None) == -2
    # six- and eight-bit formats: conversion and de-conversion take them (same argument rules; the plain forms need no
    # index array), every other entry point reports them as a format it does not know
    assert L.mxp_quantize(p, mxp.BF16, 4, 48, 48, mxp.MXFP8P, p, p, p, None) == -2
    assert L.mxp_quantize(p, mxp.BF16, 4, 64, 64, mxp.MXFP6P, p, p, None, None) == -1
    assert L.mxp_quantize(p, mxp.BF16, 0, 64, 64, mxp.MXFP6, None, None, None, None) == 0
    assert L.mxp_dequantize(p, p, None, mxp.MXFP8P, 4, 64, p, mxp.F32, 64, None) == -1
    assert L.mxp_dequantize(p, p, None, mxp.MXFP8, 0, 64, p, mxp.F32, 64, None) == 0
    assert L.mxp_quantize_t(p, mxp.BF16, 4, 64, 64, mxp.MXFP6P, p, p, p, None) == -5
    assert L.mxp_prepack(p, p, p, mxp.MXFP8P, 64, 64, p, 1 << 20, None) in (-5, -8)
    # workspace too small
    need = mxp.gemm_workspace_bytes(64, 64, 64)
    assert need > 0
    assert L.mxp_gemm(64, 64, 64, p, p, p, 1, p, p, p, 1, p, mxp.F32, 64, p, need - 1, None) == -6
    assert L.mxp_prepack(p, p, p, 1, 64, 64, p, 16, None) == -6
    assert L.mxp_gemm(64, 64, 48, p, p, p, 1, p, p, p, 1, p, mxp.F32, 64, p, need, None) == -2
    assert L.mxp_gemm(64, 64, 64, p, p, p, 1, p, p, p, 1, p, mxp.F32, 32, p, need, None) == -2
    # the one-pass conversion: image required, canonical arrays all or none, image buffer size checked
    big = mxp.image_bytes(4, 64)
    assert L.mxp_quantize_image(p, mxp.BF16, 4, 64, 64, mxp.MXFP4P, None, None, None, None, big, None) == -1
    assert L.mxp_quantize_image(p, mxp.BF16, 4, 64, 64, mxp.MXFP4P, p, None, None, p, big, None) == -1
    assert L.mxp_quantize_image(p, mxp.BF16, 4, 64, 64, mxp.MXFP4P, p, p, None, p, big, None) == -1
    assert L.mxp_quantize_image(p, mxp.BF16, 4, 64, 64, mxp.MXFP4P, None, None, None, p, big - 1, None) == -6
    assert L.mxp_quantize_image(p, mxp.BF16, 4, 48, 48, mxp.MXFP4P, None, None, None, p, big, None) == -2
    assert L.mxp_quantize_image(p, 3, 4, 64, 64, mxp.MXFP4P, None, None, None, p, big, None) == -4
    assert L.mxp_quantize_image(odd, mxp.BF16, 4, 64, 64, mxp.MXFP4P, None, None, None, p, big, None) == -3
    # image kinds
    assert L.mxp_prepack_e2m1(p, p, 64, 64, p, 16, None) == -6
    assert L.mxp_prepack_e2m1(p, None, 64, 64, p, 1 << 20, None) == -1
    assert L.mxp_gemm_prepacked(64, 64, 64, p, 0, p, 5, p, mxp.F32, 64, None) == -5
    assert L.mxp_gemm_prepacked(65, 64, 64, p, mxp.IMAGE_E2M3, p, mxp.IMAGE_E2M1X, p, mxp.F32, 64, None) == -8
    assert L.mxp_prepack_e2m1x(p, p, p, mxp.MXFP4, 64, 64, p, 1 << 20, None) == -8
    assert L.mxp_prepack_e2m1x(p, p, p, mxp.MXFP6, 64, 64, p, 1 << 20, None) == -5
    assert L.mxp_prepack_e2m1x(p, p, None, mxp.MXFP4PP, 64, 64, p, 1 << 20, None) == -1
    assert L.mxp_prepack_e2m1x(p, p, p, mxp.MXFP4PP, 64, 64, p, 16, None) == -6
    # the 4-bit MXFP4+ weight image with residual bytes: B side of the few-row product only
    assert L.mxp_gemm_prepacked(65, 64, 64, p, mxp.IMAGE_E2M3, p, mxp.IMAGE_E2M1R, p, mxp.F32, 64, None) == -8
    assert L.mxp_gemm_prepacked(8, 64, 64, p, mxp.IMAGE_E2M1, p, mxp.IMAGE_E2M1R, p, mxp.F32, 64, None) == -8
    assert L.mxp_gemm_prepacked(8, 64, 64, p, mxp.IMAGE_E2M1R, p, mxp.IMAGE_E2M3, p, mxp.F32, 64, None) == -5
    assert L.mxp_gemm_bf16a(65, 64, 64, p, mxp.BF16, 64, mxp.MXFP4P, p, mxp.IMAGE_E2M1R, p, mxp.F32, 64, p, 1 << 20, None) == -8
    assert L.mxp_prepack_e2m1r(p, p, None, 64, 64, p, 1 << 20, None) == -1
    assert L.mxp_prepack_e2m1r(p, p, p, 64, 48, p, 1 << 20, None) == -2
    assert L.mxp_prepack_e2m1r(p, p, p, 64, 64, p, mxp.image_bytes_e2m1(64, 64), None) == -6
    assert mxp.image_bytes_e2m1r(4096, 4096) == mxp.image_bytes_e2m1(4096, 4096) + 4096 * 128
    assert L.mxp_gemm_prepacked(64, 64, 64, p, 0, p, 2, p, mxp.F32, 64, None) == -8      # E4M3 images only in pairs
    assert L.mxp_gemm_prepacked(65, 64, 64, p, 2, p, 1, p, mxp.F32, 64, None) == -8      # (few rows: E4M3 activations x 4-bit weights run)
    assert L.mxp_prepack_e4m3(p, p, p, mxp.MXFP4PP, 64, 64, p, 16, None) == -6
    assert L.mxp_prepack_e4m3(p, p, None, mxp.MXFP4PP, 64, 64, p, 1 << 20, None) == -1
    assert L.mxp_prepack_e4m3(p, p, p, mxp.MXFP6P, 64, 64, p, 1 << 20, None) == -5
    assert mxp.image_bytes_e4m3(256, 128) == 8 * 2 * 2048 + 2 * 2 * 256
    assert L.mxp_gemm_prepacked(64, 64, 64, p, 3, p, 0, p, mxp.F32, 64, None) == -5
    assert L.mxp_gemm_prepacked(64, 64, 64, p, mxp.IMAGE_E2M1, p, mxp.IMAGE_E2M3, p, mxp.F32, 64, None) == -8
    assert L.mxp_gemm_prepacked(64, 64, 64, p, 0, None, mxp.IMAGE_E2M1, p, mxp.F32, 64, None) == -1
    assert L.mxp_gemm_bf16a(64, 64, 64, p, mxp.BF16, 64, mxp.MXFP4P, p, 5, p, mxp.F32, 64, p, 1 << 20, None) == -5
    assert L.mxp_gemm_bf16a(64, 64, 64, p, mxp.BF16, 64, mxp.MXFP4P, p, 0, p, mxp.F32, 64, p, 16, None) == -6
    # channel-reordered conversion and the conversion-based product
    assert L.mxp_quantize_gather(p, mxp.BF16, 4, 64, 64, 64, None, mxp.MXFP4P, p, p, p, None) == -1
    assert L.mxp_quantize_gather(p, mxp.BF16, 4, 64, 0, 64, p, mxp.MXFP4P, p, p, p, None) == -2
    assert L.mxp_quantize_gather(p, mxp.BF16, 4, 64, 128, 64, p, mxp.MXFP4P, p, p, p, None) == -2
    assert L.mxp_quantize_gather(p, mxp.BF16, 4, 64, 64, 64, odd, mxp.MXFP4P, p, p, p, None) == -3
    assert L.mxp_quantize_gather(p, mxp.BF16, 4, 40, 64, 64, p, mxp.MXFP4P, p, p, p, None) == -2
    assert L.mxp_gemm_w4a16(8, 64, 64, p, mxp.BF16, 64, p, p, p, 7, p, mxp.F32, 64, None) == -5
    assert L.mxp_gemm_w4a16(8, 64, 64, p, mxp.F32, 64, p, p, p, mxp.MXFP4P, p, mxp.F32, 64, None) == -8
    assert L.mxp_gemm_w4a16(8, 64, 64, p, mxp.BF16, 64, p, p, None, mxp.MXFP4PP, p, mxp.F32, 64, None) == -1
    assert L.mxp_gemm_w4a16(8, 64, 64, p, mxp.BF16, 32, p, p, p, mxp.MXFP4P, p, mxp.F32, 64, None) == -2
    assert L.mxp_gemm_w4a16(8, 64, 64, p, mxp.BF16, 64, p, p, p, mxp.MXFP4P, p, mxp.F32, 32, None) == -2
    # MXFP4++ is a codec: no image, no W4A4 product
    assert L.mxp_prepack(p, p, p, mxp.MXFP4PP, 64, 64, p, 1 << 20, None) == -8
    # an MXFP4++ operand sends both through E4M3 images: a workspace sized for E2M3 images is too small
    assert mxp.gemm_workspace_bytes(64, 64, 64, mxp.MXFP4PP, mxp.MXFP4P) > mxp.gemm_workspace_bytes(64, 64, 64)
    assert L.mxp_gemm(64, 64, 64, p, p, p, mxp.MXFP4PP, p, p, p, 1, p, mxp.F32, 64, p, mxp.gemm_workspace_bytes(64, 64, 64), None) == -6
    assert L.mxp_gemm(64, 64, 64, p, p, None, mxp.MXFP4PP, p, p, p, 1, p, mxp.F32, 64, p, 1 << 20, None) == -1
    # MXFP4++ activations become an E4M3 image (larger than the E2M3 one) and pair with E4M3 weight images only
    assert L.mxp_quantize_image(p, mxp.BF16, 4, 64, 64, mxp.MXFP4PP, None, None, None, p, mxp.image_bytes(4, 64), None) == -6
    assert L.mxp_quantize_image(p, mxp.BF16, 4, 64, 64, mxp.MXFP4PP, p, p, None, p, 1 << 20, None) == -1
    assert L.mxp_gemm_bf16a(4, 64, 64, p, mxp.BF16, 64, mxp.MXFP4PP, p, mxp.IMAGE_E2M3, p, mxp.F32, 64, p, 1 << 20, None) == -8
    assert L.mxp_gemm_bf16a(4, 64, 64, p, mxp.BF16, 64, mxp.MXFP4P, p, mxp.IMAGE_E4M3, p, mxp.F32, 64, p, 1 << 20, None) == -8
    assert L.mxp_gemm_bf16a(4, 64, 64, p, mxp.BF16, 64, mxp.MXFP4PP, p, mxp.IMAGE_E4M3, p, mxp.F32, 64, p,
                            mxp.gemm_bf16a_workspace_bytes(4, 64), None) == -6
    # six-bit operand images: segments 1..4, a residual only for MXFP6+, sized by the segment count
    assert L.mxp_prepack_fp6(p, p, p, mxp.MXFP6P, 64, 64, 5, 0, p, 1 << 24, None) == -2
    assert L.mxp_prepack_fp6(p, p, p, mxp.MXFP6P, 64, 64, 2, 0b100, p, 1 << 24, None) == -2
    assert L.mxp_prepack_fp6(p, p, p, mxp.MXFP6, 64, 64, 2, 0b10, p, 1 << 24, None) == -2
    assert L.mxp_prepack_fp6(p, p, None, mxp.MXFP6P, 64, 64, 2, 0b10, p, 1 << 24, None) == -1
    assert L.mxp_prepack_fp6(p, p, p, mxp.MXFP4P, 64, 64, 1, 0, p, 1 << 24, None) == -5
    assert L.mxp_prepack_fp6(p, p, p, mxp.MXFP6P, 64, 64, 2, 0b10, p, mxp.image_bytes_fp6(64, 64, 1), None) == -6
    # one-pass conversion into the same images
    assert L.mxp_quantize_image_fp6(p, mxp.BF16, 64, 64, 64, mxp.MXFP6P, 5, 0, None, None, None, p, 1 << 24, None) == -2
    assert L.mxp_quantize_image_fp6(p, mxp.BF16, 64, 64, 64, mxp.MXFP6, 2, 0b10, None, None, None, p, 1 << 24, None) == -2
    assert L.mxp_quantize_image_fp6(p, mxp.BF16, 64, 64, 32, mxp.MXFP6P, 1, 0, None, None, None, p, 1 << 24, None) == -2
    assert L.mxp_quantize_image_fp6(p, 7, 64, 64, 64, mxp.MXFP6P, 1, 0, None, None, None, p, 1 << 24, None) == -4
    assert L.mxp_quantize_image_fp6(p, mxp.BF16, 64, 64, 64, mxp.MXFP4P, 1, 0, None, None, None, p, 1 << 24, None) == -5
    assert L.mxp_quantize_image_fp6(None, mxp.BF16, 64, 64, 64, mxp.MXFP6P, 1, 0, None, None, None, p, 1 << 24, None) == -1
    assert L.mxp_quantize_image_fp6(p, mxp.BF16, 64, 64, 64, mxp.MXFP6P, 1, 0, p, p, None, p, 1 << 24, None) == -1
    assert L.mxp_quantize_image_fp6(p, mxp.BF16, 64, 64, 64, mxp.MXFP6P, 2, 0b10, None, None, None, p, mxp.image_bytes_fp6(64, 64, 1), None) == -6
    assert L.mxp_quantize_image_fp6(p, mxp.BF16, 0, 64, 64, mxp.MXFP6P, 1, 0, None, None, None, None, 0, None) == 0
    assert mxp.image_bytes_fp6(64, 64, 2) == mxp.image_bytes(64, 256) and mxp.image_bytes_fp6(64, 64, 0) == 0
    assert L.mxp_prepack_fp8(p, p, 64, 64, p, 16, None) == -6
    assert L.mxp_prepack_fp8(p, None, 64, 64, p, 1 << 24, None) == -1
    # products: MXFP6 / MXFP6+ pair with each other, MXFP8 with MXFP8, MXFP8+ with nothing
    assert mxp.gemm_workspace_bytes(64, 64, 64, mxp.MXFP6P, mxp.MXFP6P) == 2 * mxp.image_bytes_fp6(64, 64, 4)
    assert mxp.gemm_workspace_bytes(64, 64, 64, mxp.MXFP6P, mxp.MXFP4) == 2 * mxp.image_bytes_fp6(64, 64, 2)
    assert mxp.gemm_workspace_bytes(64, 64, 64, mxp.MXFP6P, mxp.MXFP4PP) == 64 * 64 * 2         # route without images: A as bf16 (optional)
    assert mxp.gemm_workspace_bytes(64, 64, 64, mxp.MXFP8, mxp.MXFP4P) == 64 * 64 * 2           # exact route as well
    assert mxp.gemm_workspace_bytes(64, 64, 64, mxp.MXFP8, mxp.MXFP8) == 64 * 64 * 2            # exact route: no images, A as bf16
    assert mxp.gemm_workspace_bytes(64, 64, 64, mxp.MXFP4PP, mxp.MXFP4) == 2 * mxp.image_bytes_fp6(64, 64, 2)
    assert mxp.gemm_workspace_bytes(64, 64, 64, mxp.MXFP4PP, mxp.MXFP4PP) == 2 * mxp.image_bytes_e4m3(64, 64)
    assert L.mxp_gemm(64, 64, 64, p, p, None, mxp.MXFP6P, p, p, p, mxp.MXFP4PP, p, mxp.F32, 64, None, 0, None) == -1   # taken: arguments checked
    assert L.mxp_gemm(64, 64, 64, p, p, p, mxp.MXFP8P, p, p, None, mxp.MXFP6P, p, mxp.F32, 64, None, 0, None) == -1   # mixed widths: taken, arguments checked
    assert L.mxp_gemm(64, 64, 64, p, p, None, mxp.MXFP8P, p, p, p, mxp.MXFP8, p, mxp.F32, 64, None, 0, None) == -1
    assert mxp.gemm_workspace_bytes(64, 64, 64, mxp.MXFP8P, mxp.MXFP8) == 64 * 64 * 2
    assert L.mxp_gemm_w4a16(8, 64, 64, p, mxp.BF16, 64, p, p, None, mxp.MXFP8P, p, mxp.F32, 64, None) == -1
    assert L.mxp_gemm_w4a16(8, 64, 64, p, mxp.BF16, 64, p, p, None, 7, p, mxp.F32, 64, None) == -5
    assert L.mxp_gemm(64, 64, 64, p, p, None, mxp.MXFP6P, p, p, None, mxp.MXFP6, p, mxp.F32, 64, p, 1 << 24, None) == -1
    assert L.mxp_gemm(64, 64, 64, p, p, p, mxp.MXFP6P, p, p, None, mxp.MXFP6, p, mxp.F32, 64, p, 1024, None) == -6
    assert L.mxp_gemm(64, 64, 64, p, p, p, mxp.MXFP4PP, p, p, None, mxp.MXFP4, p, mxp.F32, 64, p, 1024, None) == -6
    assert L.mxp_prepack_seg(p, p, p, mxp.MXFP4PP, 64, 64, 2, 0, p, 1 << 24, None) == -8        # MXFP4++ has no one-scale form
    assert L.mxp_prepack_seg(p, p, None, mxp.MXFP4, 64, 64, 2, 1, p, 1 << 24, None) == -8       # MXFP4 has no BM to split off
    assert L.mxp_prepack_seg(p, p, p, mxp.MXFP4P, 64, 64, 2, 3, p, 1 << 24, None) == -2         # unknown role
    assert L.mxp_prepack_seg(p, p, p, mxp.MXFP4PP, 64, 64, 2, 9, p, 16, None) == -6
    assert L.mxp_gemm(64, 64, 64, p, p, p, 7, p, p, p, mxp.MXFP6, p, mxp.F32, 64, p, 1 << 24, None) == -5
    # the products take K up to 2^21 (prepacked images, which may hold four K segments: 2^23)
    assert L.mxp_gemm(64, 64, (1 << 21) + 32, p, p, p, 1, p, p, p, 1, p, mxp.F32, 64, p, 1 << 24, None) == -8
    assert L.mxp_gemm_prepacked(64, 64, (1 << 23) + 128, p, 0, p, 0, p, mxp.F32, 64, None) == -8
    assert L.mxp_gemm_bf16a(4, 64, (1 << 21) + 32, p, mxp.BF16, 1 << 22, mxp.MXFP4P, p, mxp.IMAGE_E2M3, p, mxp.F32, 64, p, 1 << 20, None) == -8
    assert L.mxp_quantize(None, mxp.BF16, 0, 64, 64, mxp.MXFP4P, None, None, None, None) == 0
    assert L.mxp_gemm(0, 64, 64, None, None, None, 1, None, None, None, 1, None, mxp.F32, 64, None, 0, None) == 0


def test_image_geometry():
    # 24 bytes per 32-element block + 1 scale byte, rows padded to 256 and K to 128
    assert mxp.image_bytes(256, 128) == 256 * 4 * 24 + 256 * 4
    assert mxp.image_bytes(1, 32) == mxp.image_bytes(256, 128)
    assert mxp.image_bytes(4096, 4096) == 4096 * 128 * 25
    assert mxp.gemm_workspace_bytes(4096, 4096, 4096) == 2 * 4096 * 128 * 25
    # a plain MXFP4 operand kept in 4-bit codes: 16 bytes per block + 1 scale byte
    assert mxp.image_bytes_e2m1(256, 128) == 256 * 4 * 16 + 256 * 4
    assert mxp.image_bytes_e2m1(4096, 4096) == 4096 * 128 * 17
    assert mxp.gemm_bf16a_workspace_bytes(4096, 4096) == 4096 * 128 * 25


def test_gemm_static_refuses_oversized_products_before_touching_the_gpu():
    L = mxp.lib()
    buf = (C.c_uint8 * 4096)()
    p = C.c_void_p((C.addressof(buf) + 15) & ~15)
    assert L.mxp_gemm_static_capacity() == 64 << 20
    # the 70B-shaped product needs ~235 MB of images: more than the built-in array holds
    assert L.mxp_gemm_workspace_size(8192, 28672, 8192, mxp.MXFP4P, mxp.MXFP4P) > L.mxp_gemm_static_capacity()
    assert L.mxp_gemm_static(8192, 28672, 8192, p, p, p, mxp.MXFP4P, p, p, p, mxp.MXFP4P, p, mxp.F32, 28672, None) == -9
    assert L.mxp_gemm_static(8, 8, 32, p, p, p, 11, p, p, p, mxp.MXFP4P, p, mxp.F32, 8, None) == -5
    assert L.mxp_gemm_static(-1, 8, 32, p, p, p, mxp.MXFP4P, p, p, p, mxp.MXFP4P, p, mxp.F32, 8, None) == -2
    assert "scratch" in mxp.status_string(-9)


def test_bench_refuses_more_than_one_gpu_and_names_its_kernels():
    """bench.py is a one-GPU program: any other --gpus value ends with a message before anything touches a device; the
    kernel it names in its roofline entry follows the library's routing of the shape."""
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in (r.stdout + r.stderr)
    sys.path.insert(0, root)
    import bench
    assert bench.product_kernel_name(4096, 14336) == "gemm_kernel_dma"
    assert bench.product_kernel_name(2048, 1024) == "gemm_block_kernel"
    assert bench.product_kernel_name(8, 4096) == "gemm_skinny16_kernel"
    assert bench.product_kernel_name(8, 28672) == "gemm_skinny_kernel"


def test_product_path_and_oracle_share_nothing():
    """The package never reaches the oracle and the oracle never reaches the package (only the tests, the smoke check and
    the bench's CPU baseline use the oracle); the only module both sides take inputs from holds no format arithmetic."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg, orc = os.path.join(root, "paper_2510_14557_amd"), os.path.join(root, "oracle")
    uses_oracle = re.compile(r"^\s*(import\s+oracle\b|from\s+oracle\b)|oracle/|libmxp_oracle", re.M)
    for dirpath, _, names in os.walk(pkg):
        for n in names:
            if n.endswith((".py", ".hip", ".h", ".cpp", ".c")):
                text = open(os.path.join(dirpath, n)).read()
                assert not uses_oracle.search(text), "%s refers to the oracle" % n
    uses_pkg = re.compile(r"paper_2510_14557_amd|libmxp\.so|mxp\.h|csrc")
    for n in os.listdir(orc):
        if n.endswith((".py", ".c", ".h")):
            assert not uses_pkg.search(open(os.path.join(orc, n)).read()), "oracle/%s refers to the HIP path" % n
    synth = open(os.path.join(pkg, "synth.py")).read()
    for word in ("quantize", "E2M1", "e2m1", "scale_byte", "shared_exp"):
        assert word not in synth, "synth.py mentions %s" % word


def test_missing_library_is_an_error_not_a_fallback(monkeypatch):
    """Without the built HIP library every call of the binding raises: there is no CPU route behind it."""
    monkeypatch.setattr(mxp, "_lib", None)
    monkeypatch.setattr(mxp, "LIB_PATH", os.path.join(os.path.dirname(mxp.LIB_PATH), "no_such_libmxp.so"))
    with pytest.raises(mxp.MxpError):
        mxp.lib()
    with pytest.raises(mxp.MxpError):
        mxp.version()
    with pytest.raises(mxp.MxpError):
        mxp.image_bytes(64, 64)
