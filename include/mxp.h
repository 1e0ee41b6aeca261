/*
 * mxp.h -- C ABI of the MI355X (gfx950) MXFP4+ library: quantize, de-convert and W4A4 GEMM for the MX+ block
 * format (MX+, arXiv 2510.14557).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library never allocates, frees, copies to
 *     the host or synchronises; work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream).
 *   - Every pointer must be 16-byte aligned and every leading dimension a multiple of 16 bytes, except the GEMM
 *     output D, which only needs the alignment of its element type.  Leading dimensions are in elements.
 *   - K is the reduction dimension; MX blocks are 32 consecutive elements ALONG K (paper Sec. 2 and Sec. 5.1:
 *     a row of A and a column of B are sequences of blocks), so K % 32 == 0 is required.
 *   - Return value: MXP_OK or a negative status; nothing is thrown or aborted, and on an error nothing is enqueued.
 *   - Sizes are 64-bit throughout (tensors and images beyond 4 GiB are fine); the product entry points (mxp_gemm*)
 *     take K up to 2^21 (mxp_gemm_prepacked: 2^23 for the images' K) and return MXP_ERR_UNSUPPORTED beyond.
 *     Outputs are overwritten, never accumulated into.
 *
 * Canonical MXFP4 / MXFP4+ storage of a [rows][K] operand (what bit-exact parity is defined on)
 *   elems  [rows][K/2]  : element 2j in the low nibble, 2j+1 in the high nibble of byte j.
 *                         ordinary element (NBM): E2M1  = sign | ee | m      (Sec. 2: 2-bit exponent, bias 1)
 *                         block-max element (BM) of MXFP4+: sign | m2 m1 m0  (Sec. 4.1/4.2: the exponent field is
 *                         reused as mantissa; the value is 2^e_max * 1.m2m1m0 with e_max = 2)
 *   scales [rows][K/32] : biased E8M0 shared exponent (Eq. 1: shared_exp = floor(log2 BM) - e_max, byte = +127);
 *                         0 = the whole block is zero (flush rule of Sec. 4.1), 255 = block held a NaN/Inf.
 *   bm_idx [rows][K/32] : position of the BM inside its block in bits [4:0], bits [7:5] zero (Sec. 4.2).
 *                         Not written / not read when fmt == MXP_FMT_MXFP4.
 */
#ifndef MXP_H_
#define MXP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* element types of un-quantized tensors */
#define MXP_F32 0
#define MXP_BF16 1

/* block formats */
#define MXP_FMT_MXFP4 0  /* plain OCP MXFP4 (Sec. 2) */
#define MXP_FMT_MXFP4P 1 /* MXFP4+ (Sec. 4)          */
#define MXP_FMT_MXFP4PP 2 /* MXFP4++ (Sec. 4.3): conversion, de-conversion, and the product -- exact over two K segments
                           * when the other operand is MXFP4 / MXFP4+ (mxp_gemm, or mxp_prepack_seg + mxp_gemm_prepacked),
                           * through E4M3 images when both operands are MXFP4++ (mxp_gemm, or mxp_prepack_e4m3 +
                           * mxp_gemm_prepacked); the other image and product entry points return MXP_ERR_UNSUPPORTED for
                           * it (its BM and NBMs have different scales, which one E2M3 operand cannot carry) */
/* Six- and eight-bit MX and MX+ formats (Sec. 4.2, data layout): conversion and de-conversion (mxp_quantize,
 * mxp_dequantize), the product of any two of the seven formats (mxp_gemm, mxp_gemm_static), weights of any format under
 * un-quantized activations (mxp_gemm_w4a16) and, for MXFP6, MXFP6+ and plain MXFP8, images of their own (mxp_prepack_fp6,
 * mxp_quantize_image_fp6, mxp_prepack_fp8 + mxp_gemm_prepacked); every other entry point returns MXP_ERR_FORMAT or
 * MXP_ERR_UNSUPPORTED for them.
 *   MXFP6 / MXFP6+: elements E2M3 (sign | ee | mmm, bias 1, subnormals m/8, largest 7.5), e_max = 2; the BM of MXFP6+ is
 *                   sign | mmmmm = 2^2 * 1.mmmmm (an E2M5 number).  elems [rows][K*3/4]: a block is 24 bytes, element i in
 *                   bits [6i, 6i+6) of the block read as a little-endian bit string.
 *   MXFP8 / MXFP8+: elements OCP E4M3 (sign | eeee | mmm, bias 7, subnormals m/8 * 2^-6, largest 448; S.1111.111, the NaN
 *                   code, is never written and de-converts as the number its fields spell), e_max = 8; the BM of MXFP8+ is
 *                   sign | mmmmmmm = 2^8 * 1.mmmmmmm (an E4M7 number).  elems [rows][K], one code per byte.
 * Block rule as for MXFP4(+) with that e_max: scale byte = floor(log2|BM|) - e_max + 127, flush when floor(log2|BM|) <=
 * -127 + e_max, byte 255 for NaN/Inf; elements round to nearest, ties to the even code, and saturate (an E4M3 element can
 * reach 2^9 X > 448 X); the BM mantissa is rounded the same way and a carry saturates.  scales and bm_idx as above; the
 * plain forms take no bm_idx.  De-conversion is exact in fp32; bf16 output is the fp32 result rounded to nearest even
 * (only results below 2^-126 are affected). */
#define MXP_FMT_MXFP6 3
#define MXP_FMT_MXFP6P 4
#define MXP_FMT_MXFP8 5
#define MXP_FMT_MXFP8P 6

/* status codes */
#define MXP_OK 0
#define MXP_ERR_NULL (-1)        /* a required pointer is NULL                        */
#define MXP_ERR_SHAPE (-2)       /* negative size, K % 32 != 0, or ld smaller than the row */
#define MXP_ERR_ALIGN (-3)       /* pointer or leading dimension not 16-byte aligned */
#define MXP_ERR_DTYPE (-4)       /* unknown dtype                                     */
#define MXP_ERR_FORMAT (-5)      /* unknown block format                              */
#define MXP_ERR_WORKSPACE (-6)   /* workspace / image buffer too small                */
#define MXP_ERR_HIP (-7)         /* the HIP runtime reported a launch error           */
#define MXP_ERR_UNSUPPORTED (-8) /* valid request this build does not implement       */
#define MXP_ERR_SCRATCH (-9)     /* mxp_gemm_static: the operand images do not fit its built-in scratch array */

/* Quantize src[rows][K] (row stride ld_src, dtype MXP_F32 or MXP_BF16) into MXFP4 or MXFP4+.
 * Per block (Sec. 4.1, Eq. 1): BM = largest magnitude (lowest index on ties); shared_exp = floor(log2|BM|) - 2;
 * if floor(log2|BM|) <= -125 the block is flushed (scale byte 0, all nibbles 0, index 0); ordinary elements are
 * x / 2^shared_exp rounded to E2M1 (nearest, ties to even, saturating at 6); for MXFP4+ the BM keeps three mantissa
 * bits, m = RNE(2|x|/2^shared_exp - 8) saturating at 7 (the shared scale is never altered).  A block holding a
 * NaN or Inf gets scale byte 255, nibbles 0, index 0.
 * MXFP4++ (Sec. 4.3) keeps the BM, scale and index of MXFP4+ and scales the other elements by 2^(shared_exp - delta)
 * instead: shared_exp - delta = CLIP(e, {shared_exp - 7, shared_exp}) with e = (largest exponent among the
 * non-BM elements) - 2 + 1; no non-BM element (all zero or below 2^-126) means the lower bound; delta is also kept
 * <= scale byte - 1 so that the finer scale stays >= 2^-126.  delta is stored in bits 7:5 of the index byte.
 * elems/scales/bm_idx are dense canonical arrays (see top).  bm_idx may be NULL for MXP_FMT_MXFP4. */
int mxp_quantize(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t ld_src, int fmt,
                 uint8_t* elems, uint8_t* scales, uint8_t* bm_idx, void* stream);

/* Same result as mxp_quantize of the transposed source: src is stored K-strided, element (r, k) at
 * src[k * ld_src + r] ("weights kept as [K x N]", Sec. 5.1 blocks still run along K). */
int mxp_quantize_t(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t ld_src, int fmt,
                   uint8_t* elems, uint8_t* scales, uint8_t* bm_idx, void* stream);

/* Conversion of a channel-reordered source (Sec. 9, channel reordering: outlier channels are dealt one per block so
 * that more of them become a BM): element k of output row r is src[r][perm[k]], perm a device array of K int32 channel
 * numbers in [0, n_src) (out-of-range entries are clamped into the row; both operands of a product must use the same
 * table).  The source row has n_src channels and row stride ld_src (any stride >= n_src: elements are read one by
 * one); src, perm and the outputs are 16-byte aligned.  Otherwise as mxp_quantize. */
int mxp_quantize_gather(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t n_src, int64_t ld_src,
                        const int32_t* perm, int fmt, uint8_t* elems, uint8_t* scales, uint8_t* bm_idx, void* stream);

/* De-conversion (Eq. 2): dst[r][k] = (-1)^s * 2^shared_exp * E, with E = 2^e_max * 1.mmm for the BM position of an
 * MXFP4+ block and the E2M1 value otherwise.  Scale byte 0 gives zeros (tested before the BM branch), 255 gives NaN.
 * For MXFP4++ the non-BM elements use 2^(shared_exp - delta), delta = index byte bits 7:5 (MXFP4+ ignores those bits).
 * Every result is exact in both output dtypes (for MXFP4++ bytes with scale byte - delta < 1, which no quantizer
 * writes, only the fp32 output is exact).  dst is [rows][K] with row stride ld_dst. */
int mxp_dequantize(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt,
                   int64_t rows, int64_t K, void* dst, int dst_dtype, int64_t ld_dst, void* stream);

/* MFMA-ready image of one operand (internal layout, never a graded output): every element widened to the 6-bit
 * E2M3 code the CDNA4 block-scaled MFMA takes -- an E2M1 element maps to code<<2 and the BM, an E2M3 number at
 * exponent e_max (Sec. 4.2), maps to sign|11|mmm, so one scaled MFMA forms the exact MX+ products including
 * BM x BM (Sec. 6.2) -- and tiled in the register order of the instruction.  Size depends on rows and K only. */
size_t mxp_image_bytes(int64_t rows, int64_t K);
int mxp_prepack(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt,
                int64_t rows, int64_t K, void* image, size_t image_bytes, void* stream);

/* Image kinds.  MXP_IMAGE_E2M3 is what mxp_prepack and mxp_quantize_image write (any format).  A plain MXFP4 operand
 * has no BM to widen, so as the B operand (the weights of Sec. 7.1's "MXFP4+ activations x MXFP4 weights" setting) it
 * may stay in its 4-bit codes: MXP_IMAGE_E2M1, two thirds of the bytes, written by mxp_prepack_e2m1 from canonical
 * MXFP4 storage (elems and scales only).  The A operand may be an E2M1 image only next to an E2M1 B image (the plain
 * MXFP4 x MXFP4 product, the baseline MX+ is compared with); E2M1 A with E2M3 B returns MXP_ERR_UNSUPPORTED. */
#define MXP_IMAGE_E2M3 0
#define MXP_IMAGE_E2M1 1
size_t mxp_image_bytes_e2m1(int64_t rows, int64_t K);
int mxp_prepack_e2m1(const uint8_t* elems, const uint8_t* scales, int64_t rows, int64_t K,
                     void* image, size_t image_bytes, void* stream);

/* MXP_IMAGE_E2M1R: MXFP4+ weights kept in 4-bit codes for the few-row (decode) product, which is bound by the weight
 * bytes (Sec. 7.2): 4.5 bits per element as in canonical storage instead of the 6.25 of the E2M3 image.  The BM is
 * split as in Eq. 3 (Sec. 5.2): its nibble holds BM_H = 2^2 * 1.m2 as an ordinary E2M1 code, which the FP4 MFMA
 * multiplies like any other element, and BM_L = +-(m1 + m0/2) goes with the BM position into one residual byte per
 * block (sign << 7 | m1 m0 << 5 | index) behind the scales; BM_L is an E2M1 number too, so the product kernel adds the
 * missing a[m][32 kb + index] * BM_L terms with a second MFMA per tile whose weight operand -- zero except for the
 * BM_L code at the BM position of each block -- it builds in registers from the residual bytes.  Every product is exact;
 * results equal those of the E2M3 route up to fp32 summation order.  B operand only, M <= 64 (mxp_gemm_prepacked,
 * mxp_gemm_bf16a), next to an E2M3 A image or, for MXFP4++ activations (Sec. 4.3), an E4M3 A image -- the MFMA takes an
 * FP8 and an FP4 operand, so MXFP4++ activations meet MXFP4+ (this kind) and plain MXFP4 (MXP_IMAGE_E2M1) weights in
 * their 4-bit codes when M <= 64, with the error bound of the E4M3 images; anything else returns MXP_ERR_UNSUPPORTED. */
#define MXP_IMAGE_E2M1R 3
size_t mxp_image_bytes_e2m1r(int64_t rows, int64_t K);
int mxp_prepack_e2m1r(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int64_t rows, int64_t K,
                      void* image, size_t image_bytes, void* stream);

/* MXP_IMAGE_E2M1X: the same idea for MXFP4++ weights (Sec. 4.3; MXFP4+ weights are the case delta = 0), again 4.5 bits per
 * element.  The 4-bit codes stay as they are, the BM's nibble included, and the residual byte is the canonical index byte
 * (position | delta << 5).  The product kernel's first MFMA takes the codes without the BM, scaled by the block's scale
 * lowered by delta; the second takes the BM alone, as the E2M3 code sign | 11 | mmm (Sec. 4.2), with the block's own
 * scale.  Same size (mxp_image_bytes_e2m1r), same pairing rules and limits as MXP_IMAGE_E2M1R; fmt is MXP_FMT_MXFP4P or
 * MXP_FMT_MXFP4PP (plain MXFP4: MXP_ERR_UNSUPPORTED -- use mxp_prepack_e2m1). */
#define MXP_IMAGE_E2M1X 4
int mxp_prepack_e2m1x(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows, int64_t K,
                      void* image, size_t image_bytes, void* stream);

/* MXP_IMAGE_E4M3: the image kind for products with BOTH operands MXFP4++ (Sec. 4.3; it takes MXFP4 and MXFP4+ operands
 * too).  The ordinary elements of an MXFP4++ block are scaled by 2^(shared_exp - delta) and its BM by 2^shared_exp, which
 * one E2M3 code per element cannot express; with the block's scale byte set to (scale byte - delta + 2) every element is
 * an FP8 E4M3 number (ordinary: E2M1 value / 4; BM: 1.mmm * 2^delta), so this image carries the block exactly and the
 * product is formed as for the other kinds on the FP8 MFMA, at half the rate.  Both operands of a product must then be E4M3
 * images (anything else returns MXP_ERR_UNSUPPORTED).  Index bytes with delta > scale byte - 1 and scale bytes 253, 254,
 * none of which a conversion writes, are outside its domain.
 * Error bound of every product on E4M3 images: within each group of eight K-consecutive products the FP8 MFMA aligns
 * the products to the group's largest and truncates each toward zero 13 bits below that product's leading bit (a property
 * of the instruction, pinned by a test), so an output is within (7 * 2^-13 + 2^-16) * sum_k |a_k b_k| of the exact
 * product -- about 2^-10.2, where the E2M3 / E2M1 kinds give 2^-16 (they lose nothing inside a group).  With one MXFP4++
 * operand use the exact route (mxp_prepack_seg). */
#define MXP_IMAGE_E4M3 2
size_t mxp_image_bytes_e4m3(int64_t rows, int64_t K);
int mxp_prepack_e4m3(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows, int64_t K,
                     void* image, size_t image_bytes, void* stream);

/* Six-bit operands of a product (Sec. 4.2).  MXFP6 elements are E2M3 numbers, so a plain MXFP6 operand is an E2M3
 * image (MXP_IMAGE_E2M3) as it stands.  The BM of MXFP6+, 2^2 * 1.mmmmm, has six significant bits; in the way Eq. 3
 * splits the MXFP4+ BM it is taken as BM_H + BM_L = 2^2 * 1.m4m3m2 + (m1m0)/8, both E2M3 numbers.  The operand is then
 * primary + residual (primary: BM_H in the BM's place; residual: BM_L there, zero elsewhere) and a product is formed
 * exactly, by the same kernels, over K segments laid side by side in the images:
 *     MXFP6+ x MXFP6 :  A = [p | r],         B = [p | p]           (2 segments: twice the work of MXFP6 x MXFP6)
 *     MXFP6+ x MXFP6+:  A = [p | r | p | r], B = [p | p | r | r]   (4 segments)
 * mxp_prepack_fp6 writes an image of n_seg (1..4) segments, each K rounded up to 128 wide; bit s of res_mask makes
 * segment s the residual (0 for MXFP6).  The product of two such images is mxp_gemm_prepacked with
 * K = n_seg * (K rounded up to 128) and both kinds MXP_IMAGE_E2M3; mxp_gemm does all of this in its workspace
 * (mxp_gemm_workspace_bytes_fmt).  image: mxp_image_bytes_fp6(rows, K, n_seg) bytes.
 * mxp_prepack_fp8: a plain MXFP8 operand as an MXP_IMAGE_E4M3 image (mxp_image_bytes_e4m3 bytes; the codes are the
 * FP8 numbers the MFMA takes; a NaN code S.1111.111 in the input makes the products it meets NaN).  The product of two
 * such images (mxp_gemm_prepacked) has the error bound stated at MXP_IMAGE_E4M3, (7 * 2^-13 + 2^-16) * sum|a b|; it is the
 * fast route (FP8 MFMA), not the one mxp_gemm takes.  mxp_gemm forms every product with an eight-bit operand -- MXFP8 and
 * MXFP8+ in any combination, either of them next to any four- or six-bit format (and MXFP6 / MXFP6+ next to MXFP4++); the
 * MXFP8+ BM, eight significant bits up to 1.992 * 2^8 > 448, fits no FP8 code anyway -- on the bf16 MFMA from de-converted
 * operands: every value is a bf16 number, so the products are exact and the bound is that of the main path; no image,
 * an optional workspace (see mxp_gemm_workspace_bytes_fmt), about a quarter of the FP8 rate.  (Values below the bf16
 * normal range, scale bytes under 16, are rounded to bf16 first.) */
size_t mxp_image_bytes_fp6(int64_t rows, int64_t K, int n_seg);

/* The same K-segment images for four-bit operands: the exact product with ONE MXFP4++ operand (Sec. 4.3; Sec. 7.1 pairs
 * MX++ activations with MXFP4 / MXFP4+ weights).  An MXFP4++ block has two scales, 2^shared_exp for its BM and
 * 2^(shared_exp - delta) for the rest, and a block-scaled MFMA operand has one: the operand is laid out as two segments,
 * role 1 = every element but the BM (its place zero) with the scale byte lowered by delta, role 2 = the BM alone as the
 * E2M3 code sign | 11 | mmm (Sec. 4.2) with the block's own scale byte; the other operand, MXFP4 or MXFP4+, as its whole
 * E2M3 image in both segments (role 0).  `roles` holds two bits per segment.  [1 | 2] x [0 | 0]^T over K = 2 * (K rounded
 * up to 128) through mxp_gemm_prepacked (kinds MXP_IMAGE_E2M3) is the exact product -- twice the MFMA work of an MXFP4+
 * product, error bound of the main path; mxp_gemm does this by itself when exactly one format is MXP_FMT_MXFP4PP.
 * fmt MXP_FMT_MXFP4PP takes roles 1 and 2 only, MXP_FMT_MXFP4 role 0 only (else MXP_ERR_UNSUPPORTED); MXFP4+ takes all
 * three (delta = 0).  image: mxp_image_bytes_fp6(rows, K, n_seg) bytes, n_seg 1..4. */
int mxp_prepack_seg(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows, int64_t K,
                    int n_seg, unsigned roles, void* image, size_t image_bytes, void* stream);
int mxp_prepack_fp6(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows, int64_t K,
                    int n_seg, unsigned res_mask, void* image, size_t image_bytes, void* stream);
int mxp_prepack_fp8(const uint8_t* elems, const uint8_t* scales, int64_t rows, int64_t K, void* image, size_t image_bytes,
                    void* stream);
/* Conversion of un-quantized rows (MXP_BF16 / MXP_F32, row stride ld_src elements) straight into the K-segment image of
 * mxp_prepack_fp6 -- the activation side of a six-bit product, Sec. 4.2 data layout, Sec. 5 -- in one pass: the image is
 * bit-identical to mxp_quantize followed by mxp_prepack_fp6 with the same fmt (MXFP6 / MXFP6+), n_seg and res_mask.
 * elems / scales / bm_idx: all null, or the canonical arrays to write as well (bm_idx only for MXFP6+), with the sizes
 * and alignment mxp_quantize asks for.  src and image 16-byte aligned, ld_src * element size a multiple of 16. */
int mxp_quantize_image_fp6(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t ld_src, int fmt, int n_seg,
                           unsigned res_mask, uint8_t* elems, uint8_t* scales, uint8_t* bm_idx, void* image,
                           size_t image_bytes, void* stream);

/* Conversion (Sec. 4.1, 4.2) written directly as an image: same source arguments and the same encoding as
 * mxp_quantize, but the result goes to `image` (mxp_image_bytes(rows, K) bytes, bit-identical to mxp_prepack of the
 * canonical result) without a pass over the canonical bytes.  If elems / scales / bm_idx are given (all of them, bm_idx
 * for MXFP4+ and MXFP4++) the canonical arrays are written as well; pass three null pointers to skip them.
 * fmt = MXP_FMT_MXFP4PP (Sec. 4.3) writes an E4M3 image instead (mxp_image_bytes_e4m3(rows, K) bytes, bit-identical to
 * mxp_prepack_e4m3 of the canonical result). */
int mxp_quantize_image(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t ld_src, int fmt,
                       uint8_t* elems, uint8_t* scales, uint8_t* bm_idx, void* image, size_t image_bytes, void* stream);

/* Both conversions in front of a product with un-quantized activations and weights kept in canonical storage, as ONE
 * launch (Sec. 7.1: activations are converted at run time; Sec. 5.2: the BM is prepared per operand): A as
 * mxp_quantize_image (A_elems / A_scales / A_idx all given or all NULL), W[N][K] as mxp_prepack -- same results bit for
 * bit, same arguments and error rules; the two jobs share one grid, so the second fills the compute units the first
 * one's tail leaves idle.  fmtA, fmtW: MXP_FMT_MXFP4 or MXP_FMT_MXFP4P (MXFP4++: MXP_ERR_UNSUPPORTED). */
int mxp_convert_operands(const void* A, int a_dtype, int64_t M, int64_t K, int64_t lda, int fmtA,
                         uint8_t* A_elems, uint8_t* A_scales, uint8_t* A_idx, void* A_image, size_t a_image_bytes,
                         const uint8_t* W_elems, const uint8_t* W_scales, const uint8_t* W_idx, int fmtW, int64_t N,
                         void* W_image, size_t w_image_bytes, void* stream);

/* D[M][N] = A[M][K] x B^T, B given as [N][K] (K-contiguous, the way a linear layer stores W); both operands in
 * canonical storage, formats chosen per operand (Sec. 5: activations MXFP4+ with weights MXFP4 or MXFP4+).
 * The result is the matrix product of the de-converted operands accumulated in fp32 (Sec. 5.1).
 * D is MXP_F32 or MXP_BF16 with row stride ldd.  workspace must hold mxp_gemm_workspace_bytes(M, N, K) bytes; it is
 * scratch for the two images and may be reused after the call's work on `stream` has finished.  With one MXFP4++ operand
 * (Sec. 4.3) the product is formed exactly over two K segments (see mxp_prepack_seg; workspace:
 * mxp_gemm_workspace_size(M, N, K, fmtA, fmtB)); with two, both operands go through E4M3 images (see MXP_IMAGE_E4M3 for
 * what that costs and how exact it is) and the workspace must hold mxp_gemm_workspace_bytes_e4m3(M, N, K) bytes. */
size_t mxp_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
size_t mxp_gemm_workspace_bytes_e4m3(int64_t M, int64_t N, int64_t K);   /* when both formats are MXP_FMT_MXFP4PP */
/* for any pair of formats mxp_gemm takes: the four-bit ones in any combination, MXFP6 / MXFP6+ in any combination
 * (see mxp_prepack_fp6 for the cost), MXFP6 or MXFP6+ with MXFP4 or MXFP4+ on the other side (plain MXFP6: one E2M3
 * image each, at the rate of the MXFP4+ product; MXFP6+: its two K segments against the four-bit operand's image laid out
 * twice, twice the work).  Pairs with an eight-bit format, and a six-bit format next to MXFP4++, are multiplied from
 * de-converted operands: the size returned for them, 2 M K bytes rounded up to 256, is room for A as bf16 and is
 * optional -- with it A is de-converted once ahead of the product (1.3 - 1.65x faster; the same products, and above 128
 * rows the same summation order, i.e. identical bits), with a smaller or no workspace both operands are de-converted
 * inside the kernel.  0 for unknown formats. */
size_t mxp_gemm_workspace_bytes_fmt(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB);
size_t mxp_gemm_workspace_size(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB);   /* the same function under its short name */
int mxp_gemm(int64_t M, int64_t N, int64_t K,
             const uint8_t* A_elems, const uint8_t* A_scales, const uint8_t* A_idx, int fmtA,
             const uint8_t* B_elems, const uint8_t* B_scales, const uint8_t* B_idx, int fmtB,
             void* D, int d_dtype, int64_t ldd, void* workspace, size_t workspace_bytes, void* stream);

/* mxp_gemm for callers that cannot allocate device memory (code under HIP graph capture, serving loops and harnesses
 * that forbid hipMalloc): the same product, same kernels and same results as mxp_gemm, with the operand images in a
 * device array built into the library instead of a caller workspace.  Neither this call nor anything it runs allocates
 * or frees memory.  The array holds mxp_gemm_static_capacity() bytes (64 MiB, resident on every GPU the library is used
 * on until the process ends); a product whose images need more -- mxp_gemm_workspace_size(M, N, K, fmtA, fmtB) bytes --
 * returns MXP_ERR_SCRATCH and enqueues nothing (the Llama-8B prefill-MLP product, 4096 x 14336 x 4096, needs 56.3 MiB).
 * All calls on one GPU share that array, which keeps the previous call's images: every byte a product reads is
 * rewritten by the image kernels of the same call first, and calls whose work overlaps on one GPU (different streams,
 * or different threads) race -- serialise them.  The first call on a device asks the runtime for the array's address on
 * that device, and the first launch of each kernel sets its launch attributes (as in every entry point): make one call
 * with the shapes in question before a stream capture begins.  Arguments otherwise as mxp_gemm. */
size_t mxp_gemm_static_capacity(void);
int mxp_gemm_static(int64_t M, int64_t N, int64_t K,
                    const uint8_t* A_elems, const uint8_t* A_scales, const uint8_t* A_idx, int fmtA,
                    const uint8_t* B_elems, const uint8_t* B_scales, const uint8_t* B_idx, int fmtB,
                    void* D, int d_dtype, int64_t ldd, void* stream);

/* Same product from images built earlier (weights are packed once, when they are loaded).  Kinds that go together:
 *   A E2M3 with B E2M3 or E2M1 (any M), or B E2M1R / E2M1X (M <= 64);   A E2M1 with B E2M1;   A E4M3 with B E4M3 (any M),
 *   or B E2M1 / E2M1R / E2M1X (M <= 64).  Unknown kinds return MXP_ERR_FORMAT, other pairings MXP_ERR_UNSUPPORTED.  K is the images' K
 *   (for six-bit images of several K segments: n_seg * K rounded up to 128). */
int mxp_gemm_prepacked(int64_t M, int64_t N, int64_t K, const void* A_image, int a_kind, const void* B_image, int b_kind,
                       void* D, int d_dtype, int64_t ldd, void* stream);

/* Activations given un-quantized (A[M][K], MXP_F32 or MXP_BF16, row stride lda): quantized on the fly to fmtA on
 * the same stream, then multiplied with the prepacked weight image (Sec. 7.1: activations are converted at run time,
 * weights ahead of time).  workspace must hold mxp_gemm_bf16a_workspace_bytes(M, K) bytes.  fmtA = MXP_FMT_MXFP4PP
 * makes an E4M3 image of the activations: it needs mxp_image_bytes_e4m3(M, K) bytes of workspace and b_kind =
 * MXP_IMAGE_E4M3, or, for M <= 64, a 4-bit weight image (MXP_IMAGE_E2M1, MXP_IMAGE_E2M1R, MXP_IMAGE_E2M1X); an E4M3 weight
 * image is taken with that fmtA only, and MXP_IMAGE_E2M1R / MXP_IMAGE_E2M1X with M <= 64 only (other pairings return MXP_ERR_UNSUPPORTED). */
size_t mxp_gemm_bf16a_workspace_bytes(int64_t M, int64_t K);
int mxp_gemm_bf16a(int64_t M, int64_t N, int64_t K, const void* A, int a_dtype, int64_t lda, int fmtA,
                   const void* B_image, int b_kind, void* D, int d_dtype, int64_t ldd,
                   void* workspace, size_t workspace_bytes, void* stream);

/* The decode stage (Sec. 7.2: few activation rows, bound by reading the weights): the same product for M <= 64 with
 * the weights W[N][K] left in canonical MXFP4 or MXFP4+ storage (no prepack step, no second copy of the weights); the
 * 4-bit codes feed the FP4 MFMA and an MXFP4+ block gets the BM split of MXP_IMAGE_E2M1R inside the kernel (BM_H in
 * place, BM_L in a second MFMA).  A_image is an E2M3 image of the activations
 * (mxp_prepack or mxp_quantize_image); mxp_gemm_decode_bf16a takes them un-quantized like mxp_gemm_bf16a, with the same
 * workspace.  K % 256 == 0; larger M, other K and MXFP4++ weights return MXP_ERR_UNSUPPORTED (use the image path).
 * Results are those of mxp_gemm_prepacked on the same operands up to fp32 summation order (every product is exact). */
int mxp_gemm_decode(int64_t M, int64_t N, int64_t K, const void* A_image, const uint8_t* W_elems, const uint8_t* W_scales,
                    const uint8_t* W_idx, int fmtW, void* D, int d_dtype, int64_t ldd, void* stream);
int mxp_gemm_decode_bf16a(int64_t M, int64_t N, int64_t K, const void* A, int a_dtype, int64_t lda, int fmtA,
                          const uint8_t* W_elems, const uint8_t* W_scales, const uint8_t* W_idx, int fmtW, void* D,
                          int d_dtype, int64_t ldd, void* workspace, size_t workspace_bytes, void* stream);

/* Conversion-based product (Sec. 5: where the 4-bit type is not multiplied directly, or only the weights are
 * quantized, blocks are de-converted to a wider type inside the kernel): D[M][N] = A[M][K] x deq(W)^T with A left as
 * it is (MXP_BF16, row stride lda; MXP_F32 returns MXP_ERR_UNSUPPORTED) and W[N][K] in canonical MXFP4, MXFP4+ or
 * MXFP4++ storage, de-converted by Eq. 2 to bf16 (exact) and multiplied on the bf16 MFMA with fp32 accumulation.
 * M <= 64 (up to 128 in two passes): a kernel bound by reading the 4-bit weights once.  Larger M (prefill with
 * weight-only quantization): 256 x 256 output tiles, the weights de-converted once per tile and 64-element step of K
 * on their way into LDS.  The tiled kernel also takes MXFP6(+) and MXFP8(+) weights (any M).  D is MXP_F32 or MXP_BF16
 * with row stride ldd.  No workspace. */
int mxp_gemm_w4a16(int64_t M, int64_t N, int64_t K, const void* A, int a_dtype, int64_t lda,
                   const uint8_t* W_elems, const uint8_t* W_scales, const uint8_t* W_idx, int fmtW,
                   void* D, int d_dtype, int64_t ldd, void* stream);

const char* mxp_status_string(int status);
int mxp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MXP_H_ */
