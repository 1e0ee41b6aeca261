/*
 * mxp_probe.h -- measurement aid for bench.py, built as its own library (libmxp_probe.so); NOT part of the product ABI.
 * It serves the roofline: it times nothing but block-scaled MFMAs, so that the rate the chip sustains at its power
 * limit can be put next to the nominal 10.1 PFLOP/s.
 */
#ifndef MXP_PROBE_H_
#define MXP_PROBE_H_
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

/* flop of one iteration of either probe: 256 workgroups x 4 wavefronts x 16 MFMAs of 32x32x64 */
#define MXP_PROBE_FLOP_PER_ITER (256.0 * 4.0 * 16.0 * 2.0 * 32.0 * 32.0 * 64.0)

/* Operands are pseudo-random bit patterns that never leave the registers (seed 0: all-zero operands).  a_kind / b_kind
 * are image kinds of mxp.h (E2M3 / E2M1 in any mix, or both E4M3).  sink: 65536 floats (device).  Returns an mxp status. */
int mxp_probe_mfma(int a_kind, int b_kind, int iters, uint32_t seed, float* sink, void* stream);

/* The same loop on operand bits taken from real images (device pointers; kinds E2M3 / E2M1 in any mix, or both E4M3):
 * wavefront w of workgroup g loads four tiles and their scale dwords of each image once -- tiles spread over the
 * whole image by (g, w) -- and then only multiplies.  rows_a / rows_b / K describe the images as for mxp_image_bytes*.
 * This is the like-for-like ceiling of a product kernel on those operands: the MFMA's power draw, and with it the
 * clock, depends on the operand bits. */
int mxp_probe_mfma_images(const void* a_image, int a_kind, int64_t rows_a, const void* b_image, int b_kind, int64_t rows_b,
                          int64_t K, int iters, float* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif
