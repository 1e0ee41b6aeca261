/*
 * mxp_oracle.c -- slow, plain CPU reference for MXFP4 / MXFP4+ (MX+, arXiv 2510.14557).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke check and
 * the benchmark's "cpu_baseline" leg may build or call it.  It shares no code, header, table
 * or constant generator with the HIP library; both sides only ever see the same input bits.
 *
 * What it follows (paper sections / equations):
 *   - MX block: 32 elements + one 8-bit shared scale X = 2^shared_exp        (Sec. 2, "Microscaling Formats")
 *   - shared_exp = max floor(log2|x|) - e_max, e_max = 2 for E2M1             (Eq. 1)
 *   - MX+ block-max (BM) element: exponent field reused as mantissa, the BM is an E2M3 number
 *     whose exponent is always e_max; the shared scale is unchanged           (Sec. 4.1, 4.2)
 *   - flush: floor(log2 BM) <= -127 + e_max  => whole block zero, biased scale 0 reserved for it (Sec. 4.1)
 *   - +8 bits per block: 5-bit BM index, 3 reserved                            (Sec. 4.2)
 *   - de-conversion                                                            (Eq. 2)
 *   - BM = BM_H + BM_L split into two E2M1 numbers                             (Eq. 3)
 *   - D = A x B with K-blocked operands, BM x BM products kept at full width   (Sec. 5.1, Sec. 6.2 BCU)
 *
 * Readings where the paper is silent:
 *   - element rounding: round to nearest, ties to the even code; |v| > 6 saturates to 6 (Sec. 4.3 shows
 *     7.92 saturating to 6.0)
 *   - BM mantissa carry (scaled BM >= 7.75): saturates to 7.5 because the shared scale is never altered
 *   - arg-max tie: lowest index is the BM, other equal magnitudes are ordinary elements
 *   - sign bit of the input is kept even when the magnitude code is 0; a flushed block is all +0
 *   - any NaN/Inf in a block: scale byte 255 (the E8M0 NaN code), all nibbles 0, index 0
 *   - nibble order: element 2j in the low nibble, 2j+1 in the high nibble of byte j
 *   - BM nibble = sign | m2 m1 m0 (m2 m1 sit in the former exponent bits)
 *
 * MX++ (Sec. 4.3): the NBMs get their own, smaller-or-equal shared exponent
 *     e = max2 floor(log2|x|) - e_max + 1,   shared_exp_new = CLIP(e, {shared_exp - 7, shared_exp}),
 * and delta = shared_exp - shared_exp_new goes into the 3 reserved bits of the index byte.  Readings:
 *   - max2 ("second-largest exponent") = the largest exponent among the NBMs, i.e. all elements but the BM index;
 *     it equals the BM's exponent when another element shares it, which is the case the upper clip bound is for
 *   - NBMs all zero or below the fp32 normal range: no exponent to take, the lower clip bound applies
 *   - delta is also limited to (scale byte - 1), so that the NBM scale stays an E8M0 number >= 2^-126
 *   - NBM rounding and saturation as in MXFP4 (saturation can only happen when delta = 0)
 *   - index byte = index | delta << 5; BM, flush and NaN rules as for MXFP4+
 *
 * All arithmetic that decides a code is done on exact values (scaling by a power of two is exact in
 * double), so no rounding happens before the one rounding step that defines the format.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#include <stdlib.h>

#define MXO_BLOCK 32
#define MXO_EMAX 2          /* E2M1: exponent field 11b, bias 1  (Sec. 2) */
#define MXO_FMT_MXFP4 0
#define MXO_FMT_MXFP4P 1
#define MXO_FMT_MXFP4PP 2

static float bf16_to_f32(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* floor(log2(a)) for finite a > 0, exact (frexp returns a = m * 2^e with m in [0.5,1)). */
static int floor_log2(double a) {
  int e;
  (void)frexp(a, &e);
  return e - 1;
}

/* Round-half-to-even of a non-negative double to an integer (exact: q is a small dyadic number). */
static long rne(double q) {
  double f = floor(q);
  double r = q - f;
  long n = (long)f;
  if (r > 0.5) return n + 1;
  if (r < 0.5) return n;
  return (n & 1) ? n + 1 : n;
}

/* E2M1 magnitude code (3 bits: ee m) of a >= 0 already divided by X.
 * An E2M1 number is  2^(ee-1) * (1 + m/2) for ee>0  and  0.5*m for ee=0 (subnormal), max 6.
 * Rounding = pick the binade, round the significand to one fraction bit (ties to even), carry into
 * the next binade if needed, saturate above the largest number. */
static unsigned e2m1_code(double a) {
  if (a <= 0.0) return 0;
  int e = floor_log2(a);
  if (e < 0) e = 0;                 /* subnormal range shares the spacing of the first binade: 0.5 */
  double step = ldexp(1.0, e - 1);  /* spacing of representable numbers in this binade */
  long q = rne(a / step);           /* value = q * step */
  double v = (double)q * step;
  if (v > 6.0) v = 6.0;             /* saturate (Sec. 4.3 example) */
  /* translate the representable value back into its bit pattern */
  if (v == 0.0) return 0;
  if (v == 0.5) return 1;
  int ev = floor_log2(v);           /* 0,1,2 */
  unsigned m = (v / ldexp(1.0, ev) == 1.5) ? 1u : 0u;
  return ((unsigned)(ev + 1) << 1) | m;
}

/* BM magnitude code: a in [4,8) after scaling; E2M3 at exponent e_max: a ~ 4*(1+m/8), m=0..7. */
static unsigned bm_code(double a) {
  long m = rne((a - 4.0) / 0.5);
  if (m > 7) m = 7;                 /* no carry into the scale: MX+ never alters it (Sec. 4.1) */
  if (m < 0) m = 0;
  return (unsigned)m;
}

/* Encode one block.  x: 32 finite-or-not floats.  elems: 16 bytes.  Returns nothing; writes outputs. */
void mxo_encode_block(const float *x, int fmt, uint8_t *elems, uint8_t *scale, uint8_t *bmidx) {
  memset(elems, 0, MXO_BLOCK / 2);
  *bmidx = 0;
  for (int i = 0; i < MXO_BLOCK; ++i) {
    if (isnan(x[i]) || isinf(x[i])) { *scale = 255; return; }
  }
  /* BM = element of largest magnitude, lowest index on ties (Sec. 3.2 defines BM / NBM). */
  int idx = 0;
  double amax = fabs((double)x[0]);
  for (int i = 1; i < MXO_BLOCK; ++i) {
    double a = fabs((double)x[i]);
    if (a > amax) { amax = a; idx = i; }
  }
  /* Flush rule (Sec. 4.1). amax == 0 has no logarithm and is flushed too. */
  if (amax == 0.0) { *scale = 0; return; }
  int e = floor_log2(amax);
  if (e <= -127 + MXO_EMAX) { *scale = 0; return; }
  int shared_exp = e - MXO_EMAX;                        /* Eq. 1 */
  *scale = (uint8_t)(shared_exp + 127);                 /* E8M0, bias 127 */
  int delta = 0;
  if (fmt == MXO_FMT_MXFP4PP) {                         /* Sec. 4.3: shared exponent of the NBMs */
    double a2 = 0.0;                                    /* largest NBM magnitude */
    for (int i = 0; i < MXO_BLOCK; ++i)
      if (i != idx && fabs((double)x[i]) > a2) a2 = fabs((double)x[i]);
    int lo = shared_exp - 7, enew = lo;
    if (a2 > 0.0 && floor_log2(a2) >= -126) {
      enew = floor_log2(a2) - MXO_EMAX + 1;
      if (enew < lo) enew = lo;
      if (enew > shared_exp) enew = shared_exp;
    }
    delta = shared_exp - enew;
    if (delta > (int)*scale - 1) delta = (int)*scale - 1;
  }
  const int plus = (fmt == MXO_FMT_MXFP4P || fmt == MXO_FMT_MXFP4PP);
  for (int i = 0; i < MXO_BLOCK; ++i) {
    unsigned s = signbit(x[i]) ? 8u : 0u;
    unsigned code;
    if (plus && i == idx) code = bm_code(fabs(ldexp((double)x[i], -shared_exp)));          /* BM / X, exact */
    else code = e2m1_code(fabs(ldexp((double)x[i], -(shared_exp - delta))));               /* NBM / X_new */
    unsigned nib = s | code;
    elems[i >> 1] |= (uint8_t)((i & 1) ? (nib << 4) : nib);
  }
  if (plus) *bmidx = (uint8_t)(idx | (delta << 5));     /* bits [4:0] index; bits [7:5] delta (0 for MXFP4+) */
}

/* Decode one block to doubles (Eq. 2). */
void mxo_decode_block(const uint8_t *elems, uint8_t scale, uint8_t bmidx, int fmt, double *out) {
  if (scale == 0) {                                     /* reserved all-zero code (Sec. 4.1) */
    for (int i = 0; i < MXO_BLOCK; ++i) out[i] = 0.0;
    return;
  }
  if (scale == 255) {
    for (int i = 0; i < MXO_BLOCK; ++i) out[i] = NAN;
    return;
  }
  int shared_exp = (int)scale - 127;
  int bm = (fmt == MXO_FMT_MXFP4P || fmt == MXO_FMT_MXFP4PP) ? (bmidx & 31) : -1;
  int delta = (fmt == MXO_FMT_MXFP4PP) ? (bmidx >> 5) : 0;        /* MXFP4+ ignores the reserved bits */
  for (int i = 0; i < MXO_BLOCK; ++i) {
    unsigned nib = (i & 1) ? (elems[i >> 1] >> 4) : (elems[i >> 1] & 15u);
    double sgn = (nib & 8u) ? -1.0 : 1.0;
    double E;
    if (i == bm) {
      unsigned m = nib & 7u;
      E = ldexp(1.0, MXO_EMAX) * (1.0 + (double)m / 8.0);             /* 2^e_max * m_i, 3 fraction bits */
    } else {
      unsigned ee = (nib >> 1) & 3u, m = nib & 1u;
      if (ee == 0) E = 0.5 * (double)m;                               /* subnormal */
      else E = ldexp(1.0, (int)ee - 1) * (1.0 + (double)m / 2.0);     /* 2^(e_i - b) * m_i, b = 1 */
    }
    out[i] = sgn * ldexp(E, i == bm ? shared_exp : shared_exp - delta);
  }
}

/* ---- tensor-level wrappers: rows x K, K-contiguous, blocks along K ------------------------------- */

static int check_shape(int64_t rows, int64_t K) { return (rows >= 0 && K >= 0 && K % MXO_BLOCK == 0) ? 0 : -1; }

int mxo_quantize_f32(const float *src, int64_t rows, int64_t K, int64_t ld, int fmt,
                     uint8_t *elems, uint8_t *scales, uint8_t *bmidx) {
  if (check_shape(rows, K)) return -1;
  int64_t nb = K / MXO_BLOCK;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t b = 0; b < nb; ++b) {
      uint8_t ib;
      mxo_encode_block(src + r * ld + b * MXO_BLOCK, fmt, elems + (r * nb + b) * 16, scales + r * nb + b, &ib);
      if (bmidx) bmidx[r * nb + b] = ib;
    }
  return 0;
}

int mxo_quantize_bf16(const uint16_t *src, int64_t rows, int64_t K, int64_t ld, int fmt,
                      uint8_t *elems, uint8_t *scales, uint8_t *bmidx) {
  if (check_shape(rows, K)) return -1;
  int64_t nb = K / MXO_BLOCK;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t b = 0; b < nb; ++b) {
      float x[MXO_BLOCK];
      for (int i = 0; i < MXO_BLOCK; ++i) x[i] = bf16_to_f32(src[r * ld + b * MXO_BLOCK + i]);
      uint8_t ib;
      mxo_encode_block(x, fmt, elems + (r * nb + b) * 16, scales + r * nb + b, &ib);
      if (bmidx) bmidx[r * nb + b] = ib;
    }
  return 0;
}

/* Source given K-strided: element (r, k) lives at src[k * ld + r]  ("weights stored as [K x N]"). */
int mxo_quantize_t_f32(const float *src, int64_t rows, int64_t K, int64_t ld, int fmt,
                       uint8_t *elems, uint8_t *scales, uint8_t *bmidx) {
  if (check_shape(rows, K)) return -1;
  int64_t nb = K / MXO_BLOCK;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t b = 0; b < nb; ++b) {
      float x[MXO_BLOCK];
      for (int i = 0; i < MXO_BLOCK; ++i) x[i] = src[(b * MXO_BLOCK + i) * ld + r];
      uint8_t ib;
      mxo_encode_block(x, fmt, elems + (r * nb + b) * 16, scales + r * nb + b, &ib);
      if (bmidx) bmidx[r * nb + b] = ib;
    }
  return 0;
}

int mxo_quantize_t_bf16(const uint16_t *src, int64_t rows, int64_t K, int64_t ld, int fmt,
                        uint8_t *elems, uint8_t *scales, uint8_t *bmidx) {
  if (check_shape(rows, K)) return -1;
  int64_t nb = K / MXO_BLOCK;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t b = 0; b < nb; ++b) {
      float x[MXO_BLOCK];
      for (int i = 0; i < MXO_BLOCK; ++i) x[i] = bf16_to_f32(src[(b * MXO_BLOCK + i) * ld + r]);
      uint8_t ib;
      mxo_encode_block(x, fmt, elems + (r * nb + b) * 16, scales + r * nb + b, &ib);
      if (bmidx) bmidx[r * nb + b] = ib;
    }
  return 0;
}

/* Decode a whole tensor to double, row stride ld_dst (elements). */
int mxo_dequantize(const uint8_t *elems, const uint8_t *scales, const uint8_t *bmidx, int fmt,
                   int64_t rows, int64_t K, double *dst, int64_t ld_dst) {
  if (check_shape(rows, K)) return -1;
  int64_t nb = K / MXO_BLOCK;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t b = 0; b < nb; ++b)
      mxo_decode_block(elems + (r * nb + b) * 16, scales[r * nb + b], bmidx ? bmidx[r * nb + b] : 0, fmt,
                       dst + r * ld_dst + b * MXO_BLOCK);
  return 0;
}

/* D[m][n] = sum_k deq(A)[m][k] * deq(B)[n][k]  in double, and S[m][n] = sum_k |a*b|  (plain definition of
 * the matmul of Sec. 5.1 on the decoded operands; the BM x BM term of Sec. 6.2 is just one of the products).
 * A is [M][K], B is [N][K]; both K-contiguous with blocks along K.  D and S are [M][N] doubles (S may be 0). */
int mxo_gemm(int64_t M, int64_t N, int64_t K,
             const uint8_t *Ae, const uint8_t *As, const uint8_t *Ai, int fmtA,
             const uint8_t *Be, const uint8_t *Bs, const uint8_t *Bi, int fmtB,
             double *D, double *S) {
  if (check_shape(M, K) || check_shape(N, K)) return -1;
  double *a = (double *)malloc(sizeof(double) * (size_t)(M * K + 1));
  double *b = (double *)malloc(sizeof(double) * (size_t)(N * K + 1));
  if (!a || !b) { free(a); free(b); return -2; }
  mxo_dequantize(Ae, As, Ai, fmtA, M, K, a, K);
  mxo_dequantize(Be, Bs, Bi, fmtB, N, K, b, K);
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      double acc = 0.0, sab = 0.0;
      for (int64_t k = 0; k < K; ++k) {
        double p = a[m * K + k] * b[n * K + k];
        acc += p;
        sab += fabs(p);
      }
      D[m * N + n] = acc;
      if (S) S[m * N + n] = sab;
    }
  free(a);
  free(b);
  return 0;
}

/* Sampled outputs: D[t] = <A row rows_m[t], B row rows_n[t]> for t < T (used at sizes where the full
 * product is too slow for a test). */
int mxo_gemm_sampled(int64_t T, const int64_t *rows_m, const int64_t *rows_n, int64_t K,
                     const uint8_t *Ae, const uint8_t *As, const uint8_t *Ai, int fmtA,
                     const uint8_t *Be, const uint8_t *Bs, const uint8_t *Bi, int fmtB,
                     double *D, double *S) {
  if (K % MXO_BLOCK) return -1;
  int64_t nb = K / MXO_BLOCK;
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < T; ++t) {
    int64_t m = rows_m[t], n = rows_n[t];
    double acc = 0.0, sab = 0.0;
    for (int64_t kb = 0; kb < nb; ++kb) {
      double a[MXO_BLOCK], b[MXO_BLOCK];
      mxo_decode_block(Ae + (m * nb + kb) * 16, As[m * nb + kb], Ai ? Ai[m * nb + kb] : 0, fmtA, a);
      mxo_decode_block(Be + (n * nb + kb) * 16, Bs[n * nb + kb], Bi ? Bi[n * nb + kb] : 0, fmtB, b);
      for (int i = 0; i < MXO_BLOCK; ++i) {
        double p = a[i] * b[i];
        acc += p;
        sab += fabs(p);
      }
    }
    D[t] = acc;
    if (S) S[t] = sab;
  }
  return 0;
}

int mxo_num_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
