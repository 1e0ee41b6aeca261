// De-conversion of one dword of codes (Eq. 2), shared by the de-conversion kernels and the product that takes
// un-quantized activations with 4-bit weights.  Device code only.
#pragma once
#include "mxp_common.h"

namespace mxp {

// Magnitude of an E2M1 code in units of X/2: {0, .5, 1, 1.5, 2, 3, 4, 6} * 2  -> one nibble each.
constexpr uint32_t kE2M1TimesTwo = 0xC8643210u;

// fp32 bit pattern of  (-1)^sign * M * 2^(sbyte - 128)  for 1 <= M <= 15, -6 <= sbyte <= 254, built from integer
// fields so that subnormal results (M = 1, sbyte = 1 -> 2^-127; lower still for MXFP4++ bytes no quantizer writes) do
// not depend on the float mode: below the normal range the pattern is the value in units of 2^-149.
__device__ __forceinline__ uint32_t make_f32(uint32_t sign, uint32_t M, int sbyte) {
  const int p = 31 - __builtin_clz(M);
  const int biased = sbyte - 1 + p;
  const uint32_t frac = (M << (23 - p)) & 0x7FFFFFu;
  uint32_t bits = biased <= 0 ? (M << (sbyte + 21)) : (((uint32_t)biased << 23) | frac);
  if (biased >= 255) bits = 0x7F800000u;                 // only reachable with scale bytes a quantizer never writes
  return (sign << 31) | bits;
}

typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef float v2f __attribute__((ext_vector_type(2)));

// Eight elements (one dword of nibbles) per lane.  Common case: the E2M1 elements go through the CDNA4 unpack-convert
// instruction with X = 2^shared_exp as the scale (exact: at most 2 significant bits times a power of two), and the lane
// that holds the BM overwrites that one element with 2^e_max * 1.mmm * X (Eq. 2, first case).  Blocks whose results
// can be subnormal or special (scale byte 0, 1, 255) take the integer path, which does not depend on the float mode.
// out: fp32 patterns, or (OUT_BF16) 4 packed pairs in out[0..3].
// `bm` = index byte & 31 (64 for plain MXFP4); `delta` = bits 7:5 of the index byte for MXFP4++ (Sec. 4.3: the NBMs
// are scaled by 2^(shared_exp - delta), the BM by 2^shared_exp), else 0.
template <bool PLUS, bool OUT_BF16>
__device__ __forceinline__ void decode_group(uint32_t dw, uint32_t sbyte, uint32_t bm, uint32_t part, uint32_t (&out)[8],
                                             uint32_t delta = 0) {
  const bool mine = PLUS && (bm >> 3) == part;       // this lane holds the BM
  const uint32_t pos = bm & 7u;
  if (sbyte >= 2u + delta && sbyte != 255u) {
    const float X = __uint_as_float((sbyte - delta) << 23);          // NBM scale
    const float XB = __uint_as_float(sbyte << 23);                   // BM scale
    const uint32_t nib = (dw >> (4u * pos)) & 15u;
    const float bmv = __uint_as_float(((nib & 8u) << 28) | __float_as_uint((float)(8u + (nib & 7u)) * (XB * 0.5f)));
    if (OUT_BF16) {
      union { v2bf v; uint32_t u; } c0, c1, c2, c3;
      c0.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(dw, X, 0);
      c1.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(dw, X, 1);
      c2.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(dw, X, 2);
      c3.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(dw, X, 3);
      out[0] = c0.u; out[1] = c1.u; out[2] = c2.u; out[3] = c3.u;
      if (mine) {
        const uint32_t h = __float_as_uint(bmv) >> 16;               // exact: 4 significant bits
        const uint32_t sh = (pos & 1u) * 16u;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if ((pos >> 1) == (uint32_t)j) out[j] = (out[j] & ~(0xFFFFu << sh)) | (h << sh);
      }
    } else {
      const v2f f0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(dw, X, 0), f1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(dw, X, 1);
      const v2f f2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(dw, X, 2), f3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(dw, X, 3);
      out[0] = __float_as_uint(f0[0]); out[1] = __float_as_uint(f0[1]); out[2] = __float_as_uint(f1[0]); out[3] = __float_as_uint(f1[1]);
      out[4] = __float_as_uint(f2[0]); out[5] = __float_as_uint(f2[1]); out[6] = __float_as_uint(f3[0]); out[7] = __float_as_uint(f3[1]);
      if (mine) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (pos == (uint32_t)i) out[i] = __float_as_uint(bmv);
      }
    }
  } else {
    uint32_t f[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t nib = (dw >> (4 * i)) & 15u;
      const uint32_t code = nib & 7u;
      uint32_t M = (kE2M1TimesTwo >> (4u * code)) & 15u;           // ordinary element: 2^(e-b) * m   (Eq. 2, second case)
      int sb = (int)sbyte - (int)delta;
      if (mine && pos == (uint32_t)i) { M = 8u + code; sb = (int)sbyte; }   // BM: 2^e_max * 1.mmm   (Eq. 2, first case)
      uint32_t bits = (nib >> 3) << 31;
      if (M != 0u) bits = make_f32(nib >> 3, M, sb);
      if (sbyte == 0u) bits = 0u;                                  // reserved all-zero code, tested before anything else
      if (sbyte == 255u) bits = 0x7FC00000u;
      f[i] = bits;
    }
    if (OUT_BF16) {
#pragma unroll
      for (int j = 0; j < 4; ++j) out[j] = (f[2 * j] >> 16) | (f[2 * j + 1] & 0xFFFF0000u);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) out[i] = f[i];
    }
  }
}

// ---- six- and eight-bit blocks (Sec. 4.2 formats) -> 32 bf16, one lane per block ----------------------------------
// raw: the block's element bytes as dwords (6 for the six-bit string, 8 for eight-bit codes).  Elements are E2M3
// (bias 1, e_max 2) or OCP E4M3 (bias 7, e_max 8); the BM of a + format is sign | all-mantissa at exponent e_max.
// Every value has at most 8 significant bits, so it is a bf16 number unless it falls below the bf16 normal range; there
// (scale bytes below 16) it is rounded to nearest even, as mxp_dequantize does for bf16 output.
// Common case (scale byte 16 .. 240, no E4M3 NaN code; or the reserved scale bytes 0 / 255): the CDNA4 unpack-convert
// instructions with X = 2^shared_exp, the BM written over its element from integer fields.  Anything else takes the
// integer path; the choice is made per wavefront (`general` must be wavefront-uniform).
typedef uint32_t v6u_dec __attribute__((ext_vector_type(6)));
typedef __bf16 v32bf_dec __attribute__((ext_vector_type(32)));

__device__ __forceinline__ uint32_t wide_f32_bits(uint32_t sign, uint32_t M, int p) {   // (-1)^sign * M * 2^p
  if (M == 0u) return sign << 31;
  const int h = 31 - __builtin_clz(M);
  const int biased = p + h + 127;
  uint32_t bits;
  if (biased >= 255) bits = 0x7F800000u;
  else if (biased >= 1) bits = ((uint32_t)biased << 23) | ((M << (23 - h)) & 0x7FFFFFu);
  else {
    const int sh = p + 149;
    bits = sh >= 0 ? (M << sh) : (M >> (-sh > 31 ? 31 : -sh));
  }
  return (sign << 31) | bits;
}
__device__ __forceinline__ uint32_t wide_bf16_rne(uint32_t f32_bits) {
  return (f32_bits + 0x7FFFu + ((f32_bits >> 16) & 1u)) >> 16;
}

template <int BITS>
__device__ __forceinline__ uint32_t wide_code_at(const uint32_t (&raw)[8], uint32_t i) {   // element i, dynamic index
  if (BITS == 8) {
    uint32_t d = raw[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) d = (i >> 2) == (uint32_t)j ? raw[j] : d;
    return (d >> (8u * (i & 3u))) & 0xFFu;
  }
  const uint32_t bit = 6u * i, w = bit >> 5, sh = bit & 31u;
  uint32_t lo = 0, hi = 0;
#pragma unroll
  for (int j = 0; j < 6; ++j) {
    lo = w == (uint32_t)j ? raw[j] : lo;
    hi = w + 1u == (uint32_t)j ? raw[j] : hi;
  }
  return (uint32_t)((((uint64_t)hi << 32) | lo) >> sh) & 0x3Fu;
}

// true when the block can take the unpack-convert path; bm = position of the BM (its byte is all mantissa and is
// written over afterwards, so S.1111.111 there is no NaN code) or >= 32
template <int BITS>
__device__ __forceinline__ bool wide_block_is_plain(const uint32_t (&raw)[8], uint32_t sbyte, uint32_t bm) {
  if (sbyte == 0u || sbyte == 255u) return true;
  if (sbyte < 16u || sbyte > 240u) return false;
  if (BITS == 8) {
    uint32_t nanlike = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      uint32_t n = ((raw[j] & 0x7F7F7F7Fu) + 0x01010101u) & 0x80808080u;
      if ((bm >> 2) == (uint32_t)j) n &= ~(0x80u << (8u * (bm & 3u)));
      nanlike |= n;
    }
    return nanlike == 0u;
  }
  return true;
}

template <int BITS>
__device__ __forceinline__ void decode_wide_block_bf16(const uint32_t (&raw)[8], uint32_t sbyte, uint32_t ib, bool plus,
                                                       bool general, uint32_t (&w)[16]) {
  constexpr int MB = 3, BIAS = BITS == 6 ? 1 : 7, EMAX = BITS == 6 ? 2 : 8;
  const uint32_t bm = plus ? (ib & 31u) : 64u;
  if (!general) {
    const float X = __uint_as_float((sbyte == 0u || sbyte == 255u ? 127u : sbyte) << 23);
    if (BITS == 6) {
      const v6u_dec str = {raw[0], raw[1], raw[2], raw[3], raw[4], raw[5]};
      union { v32bf_dec v; uint32_t u[16]; } c;
      c.v = __builtin_amdgcn_cvt_scalef32_pk32_bf16_fp6(str, X);
#pragma unroll
      for (int j = 0; j < 16; ++j) w[j] = c.u[j];
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        union { v2bf v; uint32_t u; } c0, c1;
        c0.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[j], X, false);
        c1.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[j], X, true);
        w[2 * j] = c0.u;
        w[2 * j + 1] = c1.u;
      }
    }
    if (bm < 32u) {
      // 2^e_max * 1.m * X: sign | exponent field sbyte + e_max | the code's BITS - 1 mantissa bits, left-aligned in 7
      const uint32_t code = wide_code_at<BITS>(raw, bm);
      const uint32_t mant = code & ((1u << (BITS - 1)) - 1u);
      const uint32_t h = ((code >> (BITS - 1)) << 15) | ((sbyte + (uint32_t)EMAX) << 7) | (mant << (8 - BITS));
      const uint32_t sh = (bm & 1u) * 16u;
#pragma unroll
      for (int j = 0; j < 16; ++j) w[j] = (bm >> 1) == (uint32_t)j ? (w[j] & ~(0xFFFFu << sh)) | (h << sh) : w[j];
    }
  } else {
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      uint32_t c;
      if (BITS == 8) c = (raw[i >> 2] >> (8 * (i & 3))) & 0xFFu;
      else {
        const int bit = 6 * i, wd = bit >> 5, sh = bit & 31;
        c = raw[wd] >> sh;
        if (sh > 26) c |= raw[wd + 1] << (32 - sh);
        c &= 0x3Fu;
      }
      const uint32_t sign = c >> (BITS - 1), mag = c & ((1u << (BITS - 1)) - 1u);
      uint32_t bits;
      if (bm == (uint32_t)i) {
        bits = wide_f32_bits(sign, (1u << (BITS - 1)) | mag, EMAX - (BITS - 1) + (int)sbyte - 127);
      } else {
        const uint32_t e = mag >> MB, m = mag & ((1u << MB) - 1u);
        const uint32_t M = e ? ((1u << MB) | m) : m;
        bits = wide_f32_bits(sign, M, (int)(e ? e : 1u) - BIAS - MB + (int)sbyte - 127);
      }
      const uint32_t hb = wide_bf16_rne(bits);
      if (i & 1) w[i >> 1] |= hb << 16;
      else w[i >> 1] = hb;
    }
  }
  if (sbyte == 0u || sbyte == 255u) {                       // reserved codes: an all-zero block, a block that held NaN / Inf
    const uint32_t v = sbyte == 0u ? 0u : 0x7FC07FC0u;
#pragma unroll
    for (int j = 0; j < 16; ++j) w[j] = v;
  }
}

}  // namespace mxp
