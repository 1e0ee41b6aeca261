"""MXFP4+ quantization and W4A4 GEMM for AMD MI355X (gfx950), after MX+ (arXiv 2510.14557).

`paper_2510_14557_amd.mxp` is the thin binding over the C-ABI HIP library (include/mxp.h);
`paper_2510_14557_amd.synth` draws the seeded synthetic inputs.  Importing the package loads nothing.
"""
__all__ = ["mxp", "synth"]
