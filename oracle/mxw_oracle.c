/*
 * mxw_oracle.c -- slow, plain CPU reference for the six- and eight-bit MX+ formats: MXFP6 (E2M3), MXFP6+, MXFP8 (E4M3)
 * and MXFP8+ (MX+, arXiv 2510.14557, Sec. 4.2 "Data Layout").
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT (same rules as mxp_oracle.c: only the test-suite, the smoke check and the
 * benchmark's CPU leg may build or call it; it shares nothing with the HIP library).
 *
 * What it follows:
 *   - MX block: 32 elements + one E8M0 scale X = 2^shared_exp, shared_exp = floor(log2 max|x|) - e_max     (Sec. 2, Eq. 1)
 *     e_max = 2 for E2M3 and 8 for E4M3 (Sec. 4.2 names both)
 *   - MX+: the block-max element (BM) keeps no exponent field; its exponent is e_max, so all of its non-sign bits are
 *     mantissa: E0M5 in a six-bit slot (an E2M5 number), E0M7 in an eight-bit slot (an E4M7 number)          (Sec. 4.2)
 *   - one extra byte per block: BM index in bits 4:0, bits 7:5 zero                                           (Sec. 4.2)
 *   - flush: floor(log2 BM) <= -127 + e_max => block of zeros with scale byte 0                                (Sec. 4.1)
 *   - de-conversion: (-1)^s * X * 2^e_max * 1.m for the BM, (-1)^s * X * 2^(e-b) * m otherwise               (Eq. 2)
 *
 * Element types (OCP MX specification, which Sec. 2 builds on):
 *   E2M3: sign | ee | mmm, bias 1; ee = 0 is subnormal (m/8); largest 7.5; no Inf/NaN codes.
 *   E4M3: sign | eeee | mmm, bias 7; eeee = 0 is subnormal (m/8 * 2^-6); largest 448 (S.1111.110);
 *         S.1111.111 is NaN and is never written.
 *
 * Readings where the paper is silent (the same ones as for MXFP4+):
 *   - rounding: nearest, ties to the even code; magnitudes above the largest number saturate to it (for E4M3 a scaled
 *     element can reach 2^9 > 448, so saturation is an ordinary case there)
 *   - BM mantissa: RNE of the scaled BM at exponent e_max; a carry saturates to all-ones (the scale is never altered)
 *   - arg-max tie: lowest index; the sign of an element is kept even when its magnitude code is 0
 *   - NaN/Inf in a block: scale byte 255, all codes 0, index 0
 *
 * Storage written by the tensor wrappers:
 *   eight-bit formats: elems[rows][K], one code per byte
 *   six-bit formats:   elems[rows][K*3/4]; a block is 24 bytes, element i sits in bits [6i, 6i+6) of the block read as a
 *                      little-endian bit string (bit j of the string = bit j%8 of byte j/8)
 *
 * All arithmetic that decides a code is exact (doubles, scaling by powers of two).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

#define MXW_BLOCK 32
#define MXW_FMT_MXFP6 3
#define MXW_FMT_MXFP6P 4
#define MXW_FMT_MXFP8 5
#define MXW_FMT_MXFP8P 6

typedef struct {
  int bits;      /* code width */
  int ebits;     /* exponent field width of an ordinary element */
  int mbits;     /* mantissa field width of an ordinary element */
  int bias;
  int emax;      /* exponent of the largest binade (Eq. 1) */
  double maxval; /* largest ordinary element */
  int plus;
} mxw_format;

static int mxw_get(int fmt, mxw_format *f) {
  switch (fmt) {
    case MXW_FMT_MXFP6:  *f = (mxw_format){6, 2, 3, 1, 2, 7.5, 0}; return 0;
    case MXW_FMT_MXFP6P: *f = (mxw_format){6, 2, 3, 1, 2, 7.5, 1}; return 0;
    case MXW_FMT_MXFP8:  *f = (mxw_format){8, 4, 3, 7, 8, 448.0, 0}; return 0;
    case MXW_FMT_MXFP8P: *f = (mxw_format){8, 4, 3, 7, 8, 448.0, 1}; return 0;
  }
  return -1;
}

static float mxw_bf16_to_f32(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

static int mxw_floor_log2(double a) {
  int e;
  (void)frexp(a, &e);
  return e - 1;
}

static long mxw_rne(double q) {
  double f = floor(q);
  double r = q - f;
  long n = (long)f;
  if (r > 0.5) return n + 1;
  if (r < 0.5) return n;
  return (n & 1) ? n + 1 : n;
}

/* Value of a magnitude code (exponent and mantissa fields, no sign) of an ordinary element. */
static double mxw_elem_value(const mxw_format *f, unsigned code) {
  unsigned e = code >> f->mbits, m = code & ((1u << f->mbits) - 1u);
  double frac = (double)m / (double)(1u << f->mbits);
  if (e == 0) return ldexp(frac, 1 - f->bias);               /* subnormal: 0.m * 2^(1-bias) */
  return ldexp(1.0 + frac, (int)e - f->bias);                /* 2^(e-b) * 1.m */
}

/* Magnitude code of a >= 0 (already divided by X): nearest representable number, ties to the even code. */
static unsigned mxw_elem_code(const mxw_format *f, double a) {
  if (a <= 0.0) return 0;
  int e = mxw_floor_log2(a);
  int emin = 1 - f->bias;                                    /* exponent of the first normal binade */
  if (e < emin) e = emin;                                    /* subnormals share its spacing */
  double step = ldexp(1.0, e - f->mbits);
  double v = (double)mxw_rne(a / step) * step;               /* may have carried into the next binade */
  if (v > f->maxval) v = f->maxval;
  if (v == 0.0) return 0;
  if (v < ldexp(1.0, emin)) return (unsigned)(v / ldexp(1.0, emin - f->mbits));
  int ev = mxw_floor_log2(v);
  unsigned m = (unsigned)((v / ldexp(1.0, ev) - 1.0) * (double)(1u << f->mbits));
  return ((unsigned)(ev + f->bias) << f->mbits) | m;
}

/* BM mantissa: a in [2^emax, 2^(emax+1)) after scaling; all bits-1 non-sign bits are fraction bits. */
static unsigned mxw_bm_code(const mxw_format *f, double a) {
  int fb = f->bits - 1;
  double unit = ldexp(1.0, f->emax - fb);                    /* weight of the last fraction bit */
  long m = mxw_rne((a - ldexp(1.0, f->emax)) / unit);
  long top = (1L << fb) - 1;
  if (m > top) m = top;                                      /* no carry into the scale (Sec. 4.1) */
  if (m < 0) m = 0;
  return (unsigned)m;
}

/* codes: one code per element, unpacked (low `bits` bits of each byte). */
int mxw_encode_block(const float *x, int fmt, uint8_t *codes, uint8_t *scale, uint8_t *bmidx) {
  mxw_format f;
  if (mxw_get(fmt, &f)) return -1;
  memset(codes, 0, MXW_BLOCK);
  *bmidx = 0;
  for (int i = 0; i < MXW_BLOCK; ++i)
    if (isnan(x[i]) || isinf(x[i])) { *scale = 255; return 0; }
  int idx = 0;
  double amax = fabs((double)x[0]);
  for (int i = 1; i < MXW_BLOCK; ++i) {
    double a = fabs((double)x[i]);
    if (a > amax) { amax = a; idx = i; }
  }
  if (amax == 0.0) { *scale = 0; return 0; }
  int e = mxw_floor_log2(amax);
  if (e <= -127 + f.emax) { *scale = 0; return 0; }          /* flush (Sec. 4.1) */
  int shared_exp = e - f.emax;                               /* Eq. 1 */
  *scale = (uint8_t)(shared_exp + 127);
  unsigned signbit_ = 1u << (f.bits - 1);
  for (int i = 0; i < MXW_BLOCK; ++i) {
    double a = fabs(ldexp((double)x[i], -shared_exp));       /* exact */
    unsigned code = (f.plus && i == idx) ? mxw_bm_code(&f, a) : mxw_elem_code(&f, a);
    codes[i] = (uint8_t)((signbit(x[i]) ? signbit_ : 0u) | code);
  }
  if (f.plus) *bmidx = (uint8_t)idx;
  return 0;
}

int mxw_decode_block(const uint8_t *codes, uint8_t scale, uint8_t bmidx, int fmt, double *out) {
  mxw_format f;
  if (mxw_get(fmt, &f)) return -1;
  if (scale == 0) {
    for (int i = 0; i < MXW_BLOCK; ++i) out[i] = 0.0;
    return 0;
  }
  if (scale == 255) {
    for (int i = 0; i < MXW_BLOCK; ++i) out[i] = NAN;
    return 0;
  }
  int shared_exp = (int)scale - 127;
  int bm = f.plus ? (bmidx & 31) : -1;
  unsigned signbit_ = 1u << (f.bits - 1);
  for (int i = 0; i < MXW_BLOCK; ++i) {
    unsigned c = codes[i] & ((1u << f.bits) - 1u);
    double sgn = (c & signbit_) ? -1.0 : 1.0;
    unsigned mag = c & (signbit_ - 1u);
    double E;
    if (i == bm) E = ldexp(1.0 + (double)mag / (double)signbit_, f.emax);   /* 2^e_max * 1.m  (Eq. 2, first case) */
    else E = mxw_elem_value(&f, mag);                                         /* Eq. 2, second case */
    out[i] = sgn * ldexp(E, shared_exp);
  }
  return 0;
}

/* ---- packing ------------------------------------------------------------------------------------------------- */
static int64_t mxw_block_bytes(int bits) { return MXW_BLOCK * bits / 8; }

static void mxw_pack(const uint8_t *codes, int bits, uint8_t *dst) {
  memset(dst, 0, (size_t)mxw_block_bytes(bits));
  for (int i = 0; i < MXW_BLOCK; ++i)
    for (int b = 0; b < bits; ++b)
      if ((codes[i] >> b) & 1u) {
        int j = i * bits + b;                                /* position in the block's bit string */
        dst[j >> 3] |= (uint8_t)(1u << (j & 7));
      }
}

static void mxw_unpack(const uint8_t *src, int bits, uint8_t *codes) {
  for (int i = 0; i < MXW_BLOCK; ++i) {
    unsigned c = 0;
    for (int b = 0; b < bits; ++b) {
      int j = i * bits + b;
      if ((src[j >> 3] >> (j & 7)) & 1u) c |= 1u << b;
    }
    codes[i] = (uint8_t)c;
  }
}

/* ---- tensor wrappers: rows x K, K-contiguous, blocks along K -------------------------------------------------- */
int mxw_elem_bytes_per_block(int fmt) {
  mxw_format f;
  if (mxw_get(fmt, &f)) return -1;
  return (int)mxw_block_bytes(f.bits);
}

static int mxw_quantize_any(const float *s32, const uint16_t *s16, int64_t rows, int64_t K, int64_t ld, int fmt,
                            uint8_t *elems, uint8_t *scales, uint8_t *bmidx) {
  mxw_format f;
  if (mxw_get(fmt, &f) || rows < 0 || K < 0 || K % MXW_BLOCK) return -1;
  int64_t nb = K / MXW_BLOCK, bb = mxw_block_bytes(f.bits);
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t b = 0; b < nb; ++b) {
      float x[MXW_BLOCK];
      for (int i = 0; i < MXW_BLOCK; ++i)
        x[i] = s32 ? s32[r * ld + b * MXW_BLOCK + i] : mxw_bf16_to_f32(s16[r * ld + b * MXW_BLOCK + i]);
      uint8_t codes[MXW_BLOCK], ib;
      mxw_encode_block(x, fmt, codes, scales + r * nb + b, &ib);
      mxw_pack(codes, f.bits, elems + (r * nb + b) * bb);
      if (bmidx) bmidx[r * nb + b] = ib;
    }
  return 0;
}

int mxw_quantize_f32(const float *src, int64_t rows, int64_t K, int64_t ld, int fmt, uint8_t *elems, uint8_t *scales,
                     uint8_t *bmidx) {
  return mxw_quantize_any(src, 0, rows, K, ld, fmt, elems, scales, bmidx);
}

int mxw_quantize_bf16(const uint16_t *src, int64_t rows, int64_t K, int64_t ld, int fmt, uint8_t *elems,
                      uint8_t *scales, uint8_t *bmidx) {
  return mxw_quantize_any(0, src, rows, K, ld, fmt, elems, scales, bmidx);
}

int mxw_dequantize(const uint8_t *elems, const uint8_t *scales, const uint8_t *bmidx, int fmt, int64_t rows, int64_t K,
                   double *dst, int64_t ld_dst) {
  mxw_format f;
  if (mxw_get(fmt, &f) || rows < 0 || K < 0 || K % MXW_BLOCK) return -1;
  int64_t nb = K / MXW_BLOCK, bb = mxw_block_bytes(f.bits);
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t b = 0; b < nb; ++b) {
      uint8_t codes[MXW_BLOCK];
      mxw_unpack(elems + (r * nb + b) * bb, f.bits, codes);
      mxw_decode_block(codes, scales[r * nb + b], bmidx ? bmidx[r * nb + b] : 0, fmt, dst + r * ld_dst + b * MXW_BLOCK);
    }
  return 0;
}
