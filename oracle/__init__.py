"""CPU oracle for MXFP4 / MXFP4+ (test infrastructure; see mxp_oracle.c for what it follows) and, as `oracle.wide`,
for the six- and eight-bit MX+ formats (mxw_oracle.c).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
It never imports the product package and the product package never imports it.
"""
from .mxp_oracle import (  # noqa: F401
    MXFP4, MXFP4P, MXFP4PP, quantize, quantize_t, dequantize, gemm, gemm_w4a16, gemm_sampled, encode_block, decode_block, num_threads,
)
from . import mxw_oracle as wide  # noqa: F401,E402
