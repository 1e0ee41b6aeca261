// Six- and eight-bit MX / MX+ formats (Sec. 4.2, data layout): MXFP6 (E2M3), MXFP6+, MXFP8 (E4M3), MXFP8+.
// The kernels behind mxp_quantize / mxp_dequantize for these format codes, and the kernels that lay MXFP6(+) and plain
// MXFP8 operands out as MFMA-ready images (mxp_prepack_fp6, mxp_prepack_fp8).
//
// Block rule as for MXFP4+ (Eq. 1, Sec. 4.1) with e_max = 2 (E2M3) or 8 (E4M3): scale byte = exponent field of the BM
// - e_max, flush when that field is <= e_max, byte 255 for a block with NaN/Inf.  An ordinary element is x / X rounded
// to the element type (nearest, ties to the even code, saturating at 7.5 / 448); the BM of a + format keeps e_max as
// its exponent and spends all non-sign bits on mantissa (E0M5 / E0M7 in the slot; RNE, a carry saturates).
//
// Storage: eight-bit codes one per byte; six-bit codes as a little-endian bit string, element i of a block in bits
// [6i, 6i+6) of its 24 bytes.  Four lanes share a block, a lane holds 8 consecutive elements (48 or 64 code bits).
// Ordinary elements go through the CDNA4 pack-convert / unpack-convert instructions; the BM, and every block whose
// results could leave the fp32 normal range, through integer code on the fields of the fp32 pattern (nothing there
// depends on the float mode).
#include "mxp_common.h"

namespace {

using namespace mxp;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef short v2s __attribute__((ext_vector_type(2)));
#ifndef MXP_WIDE_HW_FP8
#define MXP_WIDE_HW_FP8 1
#endif

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
constexpr int kQuadSwap1 = 0xB1;   // quad_perm [1,0,3,2]
constexpr int kQuadSwap2 = 0x4E;   // quad_perm [2,3,0,1]
constexpr int kQuadFromEven = 0xA0;  // quad_perm [0,0,2,2]: odd lanes read their left neighbour

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }

template <int BITS>
struct Elem;
template <>
struct Elem<6> {   // E2M3
  static constexpr int MB = 3, BIAS = 1, EMAX = 2;
  static constexpr uint32_t MAXCODE = 0x1Fu;   // 7.5
};
template <>
struct Elem<8> {   // E4M3 (OCP): S.1111.111 is NaN, the largest number is S.1111.110 = 448
  static constexpr int MB = 3, BIAS = 7, EMAX = 8;
  static constexpr uint32_t MAXCODE = 0x7Eu;
};

// Round-to-nearest-even of sig >> shift, 1 <= shift <= 31.
__device__ __forceinline__ uint32_t rne_shift(uint32_t sig, uint32_t shift) {
  const uint32_t t = sig >> shift, rem = sig & ((1u << shift) - 1u), half = 1u << (shift - 1u);
  return t + ((rem > half || (rem == half && (t & 1u))) ? 1u : 0u);
}

// Magnitude code of an ordinary element: a = fp32 magnitude bits of x, the block scale is 2^(sbyte - 127).
// exponent/mantissa fields are produced as one integer, so a mantissa carry moves into the exponent by itself and
// the subnormal range (field 0) needs no case of its own beyond its larger shift.
template <int BITS>
__device__ __forceinline__ uint32_t elem_code(uint32_t a, int sbyte) {
  using F = Elem<BITS>;
  if (a == 0u) return 0u;
  int ea = (int)(a >> 23);
  uint32_t sig = a & 0x7FFFFFu;
  if (ea == 0) {                       // fp32 subnormal input: normalise so that bit 23 is the leading one
    const int lz = __builtin_clz(sig) - 8;
    sig <<= lz;
    ea = 1 - lz;
  } else {
    sig |= 0x800000u;
  }
  const int t = ea - sbyte + F::BIAS;  // exponent field the scaled value would have as a normal number
  const int eff = t > 1 ? t : 1;
  int shift = (23 - F::MB) + (eff - t);
  shift = shift > 31 ? 31 : shift;     // sig < 2^24: everything beyond 25 rounds to zero anyway
  const uint32_t code = ((uint32_t)(eff - 1) << F::MB) + rne_shift(sig, (uint32_t)shift);
  return umin(code, F::MAXCODE);
}

// BM mantissa of a + format: FB = BITS - 1 fraction bits at exponent e_max; a carry out of the field saturates (the
// shared scale is never altered, Sec. 4.1).  The BM of a block that is not flushed is a normal fp32 number.
template <int BITS>
__device__ __forceinline__ uint32_t bm_code(uint32_t a) {
  constexpr int FB = BITS - 1;
  return umin(rne_shift(a & 0x7FFFFFu, 23 - FB), (1u << FB) - 1u);
}

// fp32 pattern of (-1)^sign * M * 2^p for M < 2^24, built from integer fields (exact whenever p >= -149; results
// below the normal range are the value in units of 2^-149).
__device__ __forceinline__ uint32_t make_f32(uint32_t sign, uint32_t M, int p) {
  if (M == 0u) return sign << 31;
  const int h = 31 - __builtin_clz(M);
  const int biased = p + h + 127;
  uint32_t bits;
  if (biased >= 255) bits = 0x7F800000u;
  else if (biased >= 1) bits = ((uint32_t)biased << 23) | ((M << (23 - h)) & 0x7FFFFFu);
  else {
    const int sh = p + 149;            // value = M * 2^(p + 149) units of 2^-149
    bits = sh >= 0 ? (M << sh) : (M >> (-sh > 31 ? 31 : -sh));
  }
  return (sign << 31) | bits;
}

__device__ __forceinline__ uint32_t f32_to_bf16_rne(uint32_t bits) {
  return (bits + 0x7FFFu + ((bits >> 16) & 1u)) >> 16;
}

// ---- quantize -------------------------------------------------------------------------------------------------
// nq = number of 8-element groups (4 per block); a quad of lanes is one block, so a quad is inside or outside as a whole.
template <bool BF16, int BITS, bool PLUS>
__global__ void __launch_bounds__(256) quantize_wide_kernel(const void* __restrict__ src, int64_t nbk, int64_t ld, int64_t nq,
                                                            uint8_t* __restrict__ elems, uint8_t* __restrict__ scales,
                                                            uint8_t* __restrict__ bm_idx) {
  using F = Elem<BITS>;
  const uint32_t part = threadIdx.x & 3u;
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; (q & ~(int64_t)3) < nq; q += stride) {
    const int64_t g = q >> 2;                       // block
    const int64_t row = g / nbk;
    const int64_t off = row * ld + (g - row * nbk) * 32 + part * 8;
    uint32_t a[8], sg[8], raw[8];
    if (BF16) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(src) + off);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
      raw[0] = v.x; raw[1] = v.y; raw[2] = v.z; raw[3] = v.w;
      raw[4] = raw[5] = raw[6] = raw[7] = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        a[2 * j] = (w[j] << 16) & 0x7FFF0000u;
        sg[2 * j] = (w[j] >> 15) & 1u;
        a[2 * j + 1] = w[j] & 0x7FFF0000u;
        sg[2 * j + 1] = w[j] >> 31;
      }
    } else {
      const u32x4* p = reinterpret_cast<const u32x4*>(static_cast<const float*>(src) + off);
      const u32x4 v0 = p[0], v1 = p[1];
      const uint32_t w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        raw[i] = w[i];
        a[i] = w[i] & 0x7FFFFFFFu;
        sg[i] = w[i] >> 31;
      }
    }
    uint32_t mx = a[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) mx = umax(mx, a[i]);
    mx = umax(mx, dpp_mov<kQuadSwap1>(mx));
    mx = umax(mx, dpp_mov<kQuadSwap2>(mx));
    uint32_t pos = 32u;                             // lowest position holding the maximum
#pragma unroll
    for (int i = 7; i >= 0; --i) pos = (a[i] == mx) ? part * 8u + (uint32_t)i : pos;
    pos = umin(pos, dpp_mov<kQuadSwap1>(pos));
    pos = umin(pos, dpp_mov<kQuadSwap2>(pos));
    const uint32_t E = mx >> 23;
    const bool flush = E <= (uint32_t)F::EMAX, nonfinite = E == 255u;
    const int sbyte = (int)E - F::EMAX;             // Eq. 1
    uint32_t lo = 0, hi = 0;                        // this lane's code bits: 48 (lo, hi[15:0]) or 64
    if (BITS == 8 && MXP_WIDE_HW_FP8) {
      // E4M3 elements: the CDNA4 pack-convert (x / X, round to nearest even, sign kept), two per instruction; the BM
      // byte of a + format is replaced afterwards
      const float X = __uint_as_float((uint32_t)(sbyte > 0 ? sbyte : 1) << 23);
      v2s plo = {0, 0}, phi = {0, 0};
      if (BF16) {
        union { uint32_t u; v2bf v; } c0, c1, c2, c3;
        c0.u = raw[0]; c1.u = raw[1]; c2.u = raw[2]; c3.u = raw[3];
        plo = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(plo, c0.v, X, false);
        plo = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(plo, c1.v, X, true);
        phi = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(phi, c2.v, X, false);
        phi = __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(phi, c3.v, X, true);
      } else {
        plo = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(plo, __uint_as_float(raw[0]), __uint_as_float(raw[1]), X, false);
        plo = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(plo, __uint_as_float(raw[2]), __uint_as_float(raw[3]), X, true);
        phi = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(phi, __uint_as_float(raw[4]), __uint_as_float(raw[5]), X, false);
        phi = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(phi, __uint_as_float(raw[6]), __uint_as_float(raw[7]), X, true);
      }
      union { v2s v; uint32_t u; } ul, uh;
      ul.v = plo;
      uh.v = phi;
      // the instruction answers magnitudes that round above 448 with the NaN code S.1111.111; the format saturates:
      // clear bit 0 of every byte whose low seven bits are all ones
      lo = ul.u & ~((((ul.u & 0x7F7F7F7Fu) + 0x01010101u) & 0x80808080u) >> 7);
      hi = uh.u & ~((((uh.u & 0x7F7F7F7Fu) + 0x01010101u) & 0x80808080u) >> 7);
      if (PLUS && (pos >> 3) == part) {
        const uint32_t i = pos & 7u, sh = (i & 3u) * 8u;
        uint32_t ai = 0, si = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          ai = i == (uint32_t)k ? a[k] : ai;
          si = i == (uint32_t)k ? sg[k] : si;
        }
        const uint32_t code = bm_code<8>(ai) | (si << 7);
        if (i < 4u) lo = (lo & ~(0xFFu << sh)) | (code << sh);
        else hi = (hi & ~(0xFFu << sh)) | (code << sh);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        uint32_t c = (PLUS && pos == part * 8u + (uint32_t)i) ? bm_code<BITS>(a[i]) : elem_code<BITS>(a[i], sbyte);
        c |= sg[i] << (BITS - 1);
        const int b = i * BITS;                     // bit position inside the lane's string
        if (b < 32) lo |= c << b;
        if (b + BITS > 32) hi |= (b >= 32) ? (c << (b - 32)) : (c >> (32 - b));
      }
    }
    uint32_t sb = (uint32_t)sbyte, idx = pos;
    if (flush || nonfinite) {
      lo = hi = 0;
      idx = 0;
      sb = nonfinite ? 255u : 0u;
    }
    if (BITS == 8) {
      if (q < nq) *reinterpret_cast<u32x2*>(elems + g * 32 + part * 8) = u32x2{lo, hi};
    } else {
      // 24 bytes = 6 dwords per block: lane 0 -> d0; lane 1 -> d1, d2; lane 2 -> d3; lane 3 -> d4, d5
      const uint32_t left_hi = dpp_mov<kQuadFromEven>(hi);
      uint32_t* out = reinterpret_cast<uint32_t*>(elems + g * 24);
      if (q < nq) {
        if (part & 1u) {
          out[part == 1u ? 1 : 4] = (left_hi & 0xFFFFu) | (lo << 16);
          out[part == 1u ? 2 : 5] = (lo >> 16) | (hi << 16);
        } else {
          out[part == 0u ? 0 : 3] = lo;
        }
      }
    }
    if (part == 0u && q < nq) {
      scales[g] = (uint8_t)sb;
      if (PLUS) bm_idx[g] = (uint8_t)idx;
    }
  }
}

// ---- MXFP6 / MXFP6+ through the 32-element pack-convert ---------------------------------------------------------
// The CDNA4 instruction converts 32 values of ONE lane to 32 E2M3 codes (x / X, round to nearest even, saturating, sign
// kept; code i in bits [6i, 6i+6) of its six result dwords).  The block maximum is still found by the quad; then every
// lane of the quad collects the whole block with quad broadcasts, all four convert it, and lanes 0..2 store 8 of the 24
// bytes each.  The E0M5 BM of MXFP6+ is written over its slot inside each lane's 64-bit share.
typedef __bf16 v32bf __attribute__((ext_vector_type(32)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t v6u __attribute__((ext_vector_type(6)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef float v32f __attribute__((ext_vector_type(32)));
constexpr int kQuadLane0 = 0x00, kQuadLane1 = 0x55, kQuadLane2 = 0xAA, kQuadLane3 = 0xFF;   // quad_perm broadcasts

template <bool BF16, bool PLUS>
__global__ void __launch_bounds__(256) quantize_fp6_kernel(const void* __restrict__ src, int64_t nbk, int64_t ld, int64_t nq,
                                                           uint8_t* __restrict__ elems, uint8_t* __restrict__ scales,
                                                           uint8_t* __restrict__ bm_idx) {
  using F = Elem<6>;
  constexpr int NW = BF16 ? 4 : 8;                  // dwords a lane loads
  const uint32_t part = threadIdx.x & 3u;
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; (q & ~(int64_t)3) < nq; q += stride) {
    const int64_t g = q >> 2;
    const int64_t row = g / nbk;
    const int64_t off = row * ld + (g - row * nbk) * 32 + part * 8;
    uint32_t w[NW], a[8], sg[8];
    if (BF16) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(src) + off);
      w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        a[2 * j] = (w[j] << 16) & 0x7FFF0000u;
        sg[2 * j] = (w[j] >> 15) & 1u;
        a[2 * j + 1] = w[j] & 0x7FFF0000u;
        sg[2 * j + 1] = w[j] >> 31;
      }
    } else {
      const u32x4* p = reinterpret_cast<const u32x4*>(static_cast<const float*>(src) + off);
      const u32x4 v0 = p[0], v1 = p[1];
      const uint32_t t[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        w[i] = t[i];
        a[i] = t[i] & 0x7FFFFFFFu;
        sg[i] = t[i] >> 31;
      }
    }
    uint32_t mx = a[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) mx = umax(mx, a[i]);
    mx = umax(mx, dpp_mov<kQuadSwap1>(mx));
    mx = umax(mx, dpp_mov<kQuadSwap2>(mx));
    uint32_t pos = 32u, bm_sign = 0;
#pragma unroll
    for (int i = 7; i >= 0; --i) {
      const bool hit = a[i] == mx;
      pos = hit ? part * 8u + (uint32_t)i : pos;
      bm_sign = hit ? sg[i] : bm_sign;                // sign at this lane's lowest hit
    }
    // lowest position over the quad, and the sign that goes with it
    uint32_t key = (pos << 1) | bm_sign;
    key = umin(key, dpp_mov<kQuadSwap1>(key));
    key = umin(key, dpp_mov<kQuadSwap2>(key));
    pos = key >> 1;
    bm_sign = key & 1u;
    const uint32_t E = mx >> 23;
    const bool flush = E <= (uint32_t)F::EMAX, nonfinite = E == 255u;
    const int sbyte = (int)E - F::EMAX;
    const float X = __uint_as_float((uint32_t)(sbyte > 0 ? sbyte : 1) << 23);
    // the whole block in every lane of the quad
    uint32_t all[4 * NW];
#pragma unroll
    for (int j = 0; j < NW; ++j) {
      all[0 * NW + j] = dpp_mov<kQuadLane0>(w[j]);
      all[1 * NW + j] = dpp_mov<kQuadLane1>(w[j]);
      all[2 * NW + j] = dpp_mov<kQuadLane2>(w[j]);
      all[3 * NW + j] = dpp_mov<kQuadLane3>(w[j]);
    }
    v6u r;
    if (BF16) {
      union { uint32_t u[16]; v32bf v; } c;
#pragma unroll
      for (int i = 0; i < 16; ++i) c.u[i] = all[i];
      r = __builtin_amdgcn_cvt_scalef32_pk32_fp6_bf16(c.v, X);
    } else {
      v16f lo16, hi16;
#pragma unroll
      for (int i = 0; i < 16; ++i) {                   // the two sources are interleaved: code 2i from the first, 2i + 1 from the second
        lo16[i] = __uint_as_float(all[2 * i]);
        hi16[i] = __uint_as_float(all[2 * i + 1]);
      }
      r = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(lo16, hi16, X);
    }
    // this lane's share: dwords 2 part, 2 part + 1 (lane 3 stores nothing)
    uint32_t s0 = part == 0u ? r[0] : (part == 1u ? r[2] : r[4]);
    uint32_t s1 = part == 0u ? r[1] : (part == 1u ? r[3] : r[5]);
    if (PLUS) {
      // BM code sign | mmmmm at bit 6 pos of the block's string = bit rel of this share (may hang over either edge)
      const uint32_t code = (bm_sign << 5) | bm_code<6>(mx);
      const int rel = (int)(6u * pos) - 64 * (int)part;
      uint64_t share = ((uint64_t)s1 << 32) | s0;
      if (rel > -6 && rel < 64) {
        const uint64_t m = rel >= 0 ? ((uint64_t)0x3Fu << rel) : ((uint64_t)0x3Fu >> (-rel));
        const uint64_t c = rel >= 0 ? ((uint64_t)code << rel) : ((uint64_t)code >> (-rel));
        share = (share & ~m) | c;
      }
      s0 = (uint32_t)share;
      s1 = (uint32_t)(share >> 32);
    }
    uint32_t sb = (uint32_t)sbyte, idx = pos;
    if (flush || nonfinite) {
      s0 = s1 = 0;
      idx = 0;
      sb = nonfinite ? 255u : 0u;
    }
    if (q < nq && part < 3u) *reinterpret_cast<u32x2*>(elems + g * 24 + part * 8) = u32x2{s0, s1};
    if (part == 0u && q < nq) {
      scales[g] = (uint8_t)sb;
      if (PLUS) bm_idx[g] = (uint8_t)idx;
    }
  }
}

// ---- de-conversion (Eq. 2) ------------------------------------------------------------------------------------
template <int BITS, bool PLUS, bool OUT_BF16>
__global__ void __launch_bounds__(256) dequantize_wide_kernel(const uint8_t* __restrict__ elems, const uint8_t* __restrict__ scales,
                                                              const uint8_t* __restrict__ bm_idx, int64_t nbk, int64_t ld,
                                                              int64_t nq, void* __restrict__ dst) {
  using F = Elem<BITS>;
  const uint32_t part = threadIdx.x & 3u;
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < nq; q += stride) {
    const int64_t g = q >> 2;
    const int64_t row = g / nbk;
    const int64_t off = row * ld + (g - row * nbk) * 32 + part * 8;
    // Common case (no result below the normal range, no overflow, no E4M3 NaN code): the CDNA4 unpack-convert
    // instructions, value * X exact in both output types; the lane that holds the BM then writes it over its element.
    {
      const uint32_t sb = scales[g];
      if (sb >= 16u && sb <= 240u) {
        const float X = __uint_as_float(sb << 23);
        const uint32_t bmq = PLUS ? (bm_idx[g] & 31u) : 64u;
        const bool mine = PLUS && (bmq >> 3) == part;
        const uint32_t pi = bmq & 7u;
        uint32_t f[8], hb[4];
        bool done = true;
        if (BITS == 8) {
          const u32x2 v = *reinterpret_cast<const u32x2*>(elems + g * 32 + part * 8);
          // bytes whose low seven bits are all ones (S.1111.111) take the general path below
          const uint32_t nanlike = (((v.x & 0x7F7F7F7Fu) + 0x01010101u) | ((v.y & 0x7F7F7F7Fu) + 0x01010101u)) & 0x80808080u;
          done = nanlike == 0u;
          if (done) {
            const uint32_t code = ((pi < 4u ? v.x : v.y) >> (8u * (pi & 3u))) & 0xFFu;
            const uint32_t bmbits = make_f32(code >> 7, 128u | (code & 127u), F::EMAX - 7 + (int)sb - 127);
            if (OUT_BF16) {
              union { v2bf v; uint32_t u; } c0, c1, c2, c3;
              c0.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(v.x, X, false);
              c1.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(v.x, X, true);
              c2.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(v.y, X, false);
              c3.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(v.y, X, true);
              hb[0] = c0.u; hb[1] = c1.u; hb[2] = c2.u; hb[3] = c3.u;
            } else {
              const v2f f0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(v.x, X, false), f1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(v.x, X, true);
              const v2f f2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(v.y, X, false), f3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(v.y, X, true);
              f[0] = __float_as_uint(f0[0]); f[1] = __float_as_uint(f0[1]); f[2] = __float_as_uint(f1[0]); f[3] = __float_as_uint(f1[1]);
              f[4] = __float_as_uint(f2[0]); f[5] = __float_as_uint(f2[1]); f[6] = __float_as_uint(f3[0]); f[7] = __float_as_uint(f3[1]);
            }
            if (mine) {
              if (OUT_BF16) {
                const uint32_t sh = (pi & 1u) * 16u;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                  if ((pi >> 1) == (uint32_t)j) hb[j] = (hb[j] & ~(0xFFFFu << sh)) | ((bmbits >> 16) << sh);
              } else {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                  if (pi == (uint32_t)i) f[i] = bmbits;
              }
            }
          }
        } else {
          const u32x2* in = reinterpret_cast<const u32x2*>(elems + g * 24);
          const u32x2 d0 = in[0], d1 = in[1], d2 = in[2];
          const v6u str = {d0.x, d0.y, d1.x, d1.y, d2.x, d2.y};
          // the BM's code, from this lane's own 48 bits
          const uint32_t first = (part >> 1) * 3u + (part & 1u);
          const uint32_t w0 = first == 0u ? d0.x : (first == 1u ? d0.y : (first == 3u ? d1.y : d2.x));
          const uint32_t w1 = first == 0u ? d0.y : (first == 1u ? d1.x : (first == 3u ? d2.x : d2.y));
          const uint64_t mine48 = (part & 1u) ? (((uint64_t)w1 << 16) | (w0 >> 16)) : (((uint64_t)(w1 & 0xFFFFu) << 32) | w0);
          const uint32_t code = (uint32_t)(mine48 >> (6u * pi)) & 0x3Fu;
          const uint32_t bmbits = make_f32(code >> 5, 32u | (code & 31u), F::EMAX - 5 + (int)sb - 127);
          if (OUT_BF16) {
            union { v32bf v; uint32_t u[16]; } c;
            c.v = __builtin_amdgcn_cvt_scalef32_pk32_bf16_fp6(str, X);
#pragma unroll
            for (int j = 0; j < 4; ++j)
              hb[j] = part == 0u ? c.u[j] : (part == 1u ? c.u[4 + j] : (part == 2u ? c.u[8 + j] : c.u[12 + j]));
            if (mine) {
              const uint32_t sh = (pi & 1u) * 16u;
#pragma unroll
              for (int j = 0; j < 4; ++j)
                if ((pi >> 1) == (uint32_t)j) hb[j] = (hb[j] & ~(0xFFFFu << sh)) | ((bmbits >> 16) << sh);
            }
          } else {
            union { v32f v; uint32_t u[32]; } c;
            c.v = __builtin_amdgcn_cvt_scalef32_pk32_f32_fp6(str, X);
#pragma unroll
            for (int i = 0; i < 8; ++i)
              f[i] = part == 0u ? c.u[i] : (part == 1u ? c.u[8 + i] : (part == 2u ? c.u[16 + i] : c.u[24 + i]));
            if (mine) {
#pragma unroll
              for (int i = 0; i < 8; ++i)
                if (pi == (uint32_t)i) f[i] = bmbits;
            }
          }
        }
        if (done) {
          if (OUT_BF16) {
            *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(dst) + off) = u32x4{hb[0], hb[1], hb[2], hb[3]};
          } else {
            u32x4* o = reinterpret_cast<u32x4*>(static_cast<float*>(dst) + off);
            o[0] = u32x4{f[0], f[1], f[2], f[3]};
            o[1] = u32x4{f[4], f[5], f[6], f[7]};
          }
          continue;
        }
      }
    }
    uint32_t lo, hi;
    if (BITS == 8) {
      const u32x2 v = *reinterpret_cast<const u32x2*>(elems + g * 32 + part * 8);
      lo = v.x;
      hi = v.y;
    } else {
      const uint32_t* in = reinterpret_cast<const uint32_t*>(elems + g * 24);
      const uint32_t first = (part >> 1) * 3u + (part & 1u);       // dwords 0,1 / 1,2 / 3,4 / 4,5
      const uint32_t w0 = in[first], w1 = in[first + 1];
      if (part & 1u) {
        lo = (w0 >> 16) | (w1 << 16);
        hi = w1 >> 16;
      } else {
        lo = w0;
        hi = w1 & 0xFFFFu;
      }
    }
    const uint32_t sbyte = scales[g];
    const uint32_t bm = PLUS ? (bm_idx[g] & 31u) : 64u;
    uint32_t f[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int b = i * BITS;
      uint32_t c = b < 32 ? (lo >> b) : (hi >> (b - 32));
      if (b < 32 && b + BITS > 32) c |= hi << (32 - b);
      c &= (1u << BITS) - 1u;
      const uint32_t sign = c >> (BITS - 1), mag = c & ((1u << (BITS - 1)) - 1u);
      uint32_t bits;
      if (PLUS && bm == part * 8u + (uint32_t)i) {
        // BM: 2^e_max * 1.m with BITS - 1 fraction bits
        bits = make_f32(sign, (1u << (BITS - 1)) | mag, F::EMAX - (BITS - 1) + (int)sbyte - 127);
      } else {
        const uint32_t e = mag >> F::MB, m = mag & ((1u << F::MB) - 1u);
        const uint32_t M = e ? ((1u << F::MB) | m) : m;            // subnormal: 0.m at the first binade's exponent
        bits = make_f32(sign, M, (int)(e ? e : 1u) - F::BIAS - F::MB + (int)sbyte - 127);
      }
      if (sbyte == 0u) bits = 0u;                                  // reserved all-zero code, tested before anything else
      if (sbyte == 255u) bits = 0x7FC00000u;
      f[i] = bits;
    }
    if (OUT_BF16) {
      uint32_t h[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) h[i] = sbyte == 255u ? 0x7FC0u : f32_to_bf16_rne(f[i]);
      *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(dst) + off) =
          u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
    } else {
      u32x4* o = reinterpret_cast<u32x4*>(static_cast<float*>(dst) + off);
      o[0] = u32x4{f[0], f[1], f[2], f[3]};
      o[1] = u32x4{f[4], f[5], f[6], f[7]};
    }
  }
}

dim3 grid_for(int64_t nq) {
  const int64_t want = (nq + 255) / 256, cap = (int64_t)kNumCU * 32;
  return dim3((unsigned)(want < cap ? want : cap));
}

// ---- operands of a product (MFMA-ready images) -----------------------------------------------------------------
// MXFP6 elements are E2M3 numbers and a block's 24 bytes are already the six-bit operand string of one MFMA lane, so a
// plain MXFP6 operand becomes an E2M3 image by moving bytes.  The BM of MXFP6+, 2^2 * 1.mmmmm = 4 + m/8, has six
// significant bits; as Eq. 3 does for MXFP4+ it is taken as the sum of two numbers of the element type,
// BM_H = 2^2 * 1.m4m3m2 (code s 11 m4m3m2) and BM_L = (m1m0) / 8 (the subnormal code s 00 0m1m0).  An operand is then
// primary + residual, where the primary has BM_H in the BM's place and the residual is BM_L there and zero elsewhere,
// and the product of two operands is one product over concatenated K segments:
//   A+ x B  :  [A_p | A_r] x [B | B]^T           A+ x B+ :  [A_p | A_r | A_p | A_r] x [B_p | B_p | B_r | B_r]^T
// The image written here has n_seg segments of K_p = K rounded up to 128 each; bit s of res_mask says that segment s
// holds the residual.  A workgroup takes 32 rows x 8 K-blocks (4 k-tiles) like the four-bit prepack kernel, one thread
// per block, and writes the 4 tiles of every segment in turn.
// A block's 24 bytes d[0..5] (zeros for a flushed or padding block), its scale byte and its BM position (64: none) -> the
// block's place in the four staging tiles, once per K segment: the primary (BM_H in the BM's place) or the residual (BM_L
// there, zero elsewhere), and out to the image.  Called by all 256 threads of a workgroup that owns row tile rt, k-tiles
// kt0 .. kt0 + 3 of every segment.
template <bool PLUS>
__device__ __forceinline__ void fp6_segments_out(const uint32_t (&d)[6], uint32_t sbyte, uint32_t bm, uint8_t* tiles,
                                                 uint8_t* tile_scales, int64_t rt, int64_t kt0, int64_t kts, int n_seg,
                                                 uint32_t res_mask, uint8_t* __restrict__ img_elems,
                                                 uint8_t* __restrict__ img_scales) {
  const uint32_t t = threadIdx.x, r_in = t >> 3, kb_in = t & 7u;
  const uint32_t slot = (kb_in & 1u) * 32u + r_in;
  const int64_t k_tiles = kts * n_seg;                         // k-tiles of the whole image
  // the BM's six bits: element i sits in 24-bit piece i / 4 (bytes 3 (i/4) .. +2) at bit 6 (i % 4)
  uint32_t pr[6] = {d[0], d[1], d[2], d[3], d[4], d[5]}, rs[6] = {0, 0, 0, 0, 0, 0};
  if (PLUS && bm < 32u) {
    const uint32_t bit = 6u * bm, w = bit >> 5, sh = bit & 31u;            // first dword and shift; may straddle two
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int j = 0; j < 6; ++j) {
      lo = w == (uint32_t)j ? d[j] : lo;
      hi = w + 1u == (uint32_t)j ? d[j] : hi;
    }
    const uint64_t both = ((uint64_t)hi << 32) | lo;
    const uint32_t c = (uint32_t)(both >> sh) & 0x3Fu;                    // s mmmmm
    const uint32_t code_h = (c & 0x20u) | 0x18u | ((c >> 2) & 7u);        // s 11 m4m3m2
    const uint32_t code_l = (c & 0x20u) | (c & 3u);                       // s 00 0m1m0
    const uint64_t clear = ~((uint64_t)0x3Fu << sh);
    const uint64_t ph = (both & clear) | ((uint64_t)code_h << sh), rl = (uint64_t)code_l << sh;
#pragma unroll
    for (int j = 0; j < 6; ++j) {
      if (w == (uint32_t)j) { pr[j] = (uint32_t)ph; rs[j] = (uint32_t)rl; }
      if (w + 1u == (uint32_t)j) { pr[j] = (uint32_t)(ph >> 32); rs[j] = (uint32_t)(rl >> 32); }
    }
  }
  uint8_t* tile = tiles + (kb_in >> 1) * kTileBytes;
  const int64_t nt = kts - kt0 < 4 ? kts - kt0 : 4;            // tiles of this workgroup that exist (per segment)
  const uint32_t nbytes = (uint32_t)nt * kTileBytes;
  for (int sg = 0; sg < n_seg; ++sg) {
    const bool res = (res_mask >> sg) & 1u;
    if (sg > 0) __syncthreads();                                // the previous segment has left LDS
    *reinterpret_cast<u32x4*>(tile + slot * 16u) = res ? u32x4{rs[0], rs[1], rs[2], rs[3]} : u32x4{pr[0], pr[1], pr[2], pr[3]};
    *reinterpret_cast<u32x2*>(tile + 1024u + slot * 8u) = res ? u32x2{rs[4], rs[5]} : u32x2{pr[4], pr[5]};
    tile_scales[(kb_in >> 1) * 64u + slot] = (uint8_t)sbyte;
    __syncthreads();
    const int64_t kt_img = sg * kts + kt0;
    uint8_t* out = img_elems + (rt * k_tiles + kt_img) * (int64_t)kTileBytes;
    for (uint32_t o = t * 16u; o < nbytes; o += 256u * 16u)
      MXP_IMAGE_STORE(*reinterpret_cast<const u32x4*>(tiles + o), reinterpret_cast<u32x4*>(out + o));
    if ((int64_t)(t >> 6) < nt) img_scales[(((rt >> 2) * k_tiles + kt_img + (t >> 6)) * 64 + (t & 63u)) * 4 + (rt & 3)] = tile_scales[t];
  }
}

template <bool PLUS>
__global__ void __launch_bounds__(256) prepack_fp6_kernel(const uint8_t* __restrict__ elems, const uint8_t* __restrict__ scales,
                                                          const uint8_t* __restrict__ bm_idx, int64_t rows, int64_t nbk,
                                                          int64_t kts, int n_seg, uint32_t res_mask,
                                                          uint8_t* __restrict__ img_elems, uint8_t* __restrict__ img_scales) {
  __shared__ __attribute__((aligned(16))) uint8_t tiles[4 * kTileBytes];
  __shared__ uint8_t tile_scales[4 * 64];
  const uint32_t t = threadIdx.x;
  const uint32_t r_in = t >> 3, kb_in = t & 7u;
  const PatchMap pm = patch_of_workgroup(blockIdx.x, (uint32_t)((kts + 3) / 4), (uint32_t)(((rows + kRowPad - 1) / kRowPad) * 2));
  if (!pm.valid) return;
  const int64_t kt0 = pm.kg * 4, rt = pm.rt;
  const int64_t row = rt * kTileRows + r_in, kb = kt0 * 2 + kb_in;
  uint32_t d[6] = {0, 0, 0, 0, 0, 0};
  uint32_t sbyte = 127u, bm = 64u;
  if (row < rows && kb < nbk) {
    const int64_t b = row * nbk + kb;
    const u32x2* src = reinterpret_cast<const u32x2*>(elems + b * 24);
    const u32x2 v0 = __builtin_nontemporal_load(src), v1 = __builtin_nontemporal_load(src + 1), v2 = __builtin_nontemporal_load(src + 2);
    sbyte = scales[b];
    if (sbyte != 0u) { d[0] = v0.x; d[1] = v0.y; d[2] = v1.x; d[3] = v1.y; d[4] = v2.x; d[5] = v2.y; }   // flushed: zeros
    if (PLUS && sbyte != 0u && sbyte != 255u) bm = bm_idx[b] & 31u;
  }
  fp6_segments_out<PLUS>(d, sbyte, bm, tiles, tile_scales, rt, kt0, kts, n_seg, res_mask, img_elems, img_scales);
}

// Conversion straight into such an image (optionally also the canonical arrays): what quantize_fp6_kernel and
// prepack_fp6_kernel do one after the other, without the canonical bytes making a round trip through memory.  One thread
// per block: it loads the block's 32 values (the eight threads of a row read 512 or 1024 contiguous bytes), finds the BM
// (lowest position on ties) and the scale (Eq. 1, flush and NaN rules as in quantize_fp6_kernel), converts the whole block
// with one hardware conversion, writes the MXFP6+ BM's five-bit mantissa over its slot, and hands the 24 bytes to
// fp6_segments_out.
template <bool BF16, bool PLUS>
__global__ void __launch_bounds__(256) quantize_image_fp6_kernel(const void* __restrict__ src, int64_t rows, int64_t nbk, int64_t ld,
                                                                 int64_t kts, int n_seg, uint32_t res_mask,
                                                                 uint8_t* __restrict__ elems, uint8_t* __restrict__ scales,
                                                                 uint8_t* __restrict__ bm_idx, uint8_t* __restrict__ img_elems,
                                                                 uint8_t* __restrict__ img_scales) {
  using F = Elem<6>;
  __shared__ __attribute__((aligned(16))) uint8_t tiles[4 * kTileBytes];
  __shared__ uint8_t tile_scales[4 * 64];
  const uint32_t t = threadIdx.x;
  const uint32_t r_in = t >> 3, kb_in = t & 7u;
  const PatchMap pm = patch_of_workgroup(blockIdx.x, (uint32_t)((kts + 3) / 4), (uint32_t)(((rows + kRowPad - 1) / kRowPad) * 2));
  if (!pm.valid) return;
  const int64_t kt0 = pm.kg * 4, rt = pm.rt;
  const int64_t row = rt * kTileRows + r_in, kb = kt0 * 2 + kb_in;
  uint32_t d[6] = {0, 0, 0, 0, 0, 0};
  uint32_t sbyte = 127u, bm = 64u;                             // a padding block: zero elements, unit scale
  if (row < rows && kb < nbk) {
    const int64_t off = row * ld + kb * 32;
    constexpr int NW = BF16 ? 16 : 32;
    uint32_t w[NW];
    if (BF16) {
      const u32x4* p = reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(src) + off);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const u32x4 v = __builtin_nontemporal_load(p + j);
        w[4 * j] = v.x; w[4 * j + 1] = v.y; w[4 * j + 2] = v.z; w[4 * j + 3] = v.w;
      }
    } else {
      const u32x4* p = reinterpret_cast<const u32x4*>(static_cast<const float*>(src) + off);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const u32x4 v = __builtin_nontemporal_load(p + j);
        w[4 * j] = v.x; w[4 * j + 1] = v.y; w[4 * j + 2] = v.z; w[4 * j + 3] = v.w;
      }
    }
    // block maximum over the magnitudes (fp32 bit patterns), then the lowest position that holds it and its sign
    uint32_t mx = 0;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      const uint32_t a = BF16 ? ((i & 1) ? (w[i >> 1] & 0x7FFF0000u) : ((w[i >> 1] << 16) & 0x7FFF0000u)) : (w[i] & 0x7FFFFFFFu);
      mx = umax(mx, a);
    }
    uint32_t pos = 32u, bm_sign = 0;
#pragma unroll
    for (int i = 31; i >= 0; --i) {
      const uint32_t a = BF16 ? ((i & 1) ? (w[i >> 1] & 0x7FFF0000u) : ((w[i >> 1] << 16) & 0x7FFF0000u)) : (w[i] & 0x7FFFFFFFu);
      const uint32_t sg = BF16 ? ((i & 1) ? (w[i >> 1] >> 31) : ((w[i >> 1] >> 15) & 1u)) : (w[i] >> 31);
      const bool hit = a == mx;
      pos = hit ? (uint32_t)i : pos;                           // ends at the lowest hit
      bm_sign = hit ? sg : bm_sign;
    }
    const uint32_t E = mx >> 23;
    const bool flush = E <= (uint32_t)F::EMAX, nonfinite = E == 255u;
    const int sb = (int)E - F::EMAX;
    const float X = __uint_as_float((uint32_t)(sb > 0 ? sb : 1) << 23);
    v6u r;
    if (BF16) {
      union { uint32_t u[16]; v32bf v; } c;
#pragma unroll
      for (int i = 0; i < 16; ++i) c.u[i] = w[i];
      r = __builtin_amdgcn_cvt_scalef32_pk32_fp6_bf16(c.v, X);
    } else {
      v16f lo16, hi16;
#pragma unroll
      for (int i = 0; i < 16; ++i) {                           // the two sources are interleaved: code 2i from the first, 2i + 1 from the second
        lo16[i] = __uint_as_float(w[2 * i]);
        hi16[i] = __uint_as_float(w[2 * i + 1]);
      }
      r = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(lo16, hi16, X);
    }
    uint32_t c6[6] = {r[0], r[1], r[2], r[3], r[4], r[5]};
    if (PLUS) {
      // BM code sign | mmmmm at bit 6 pos of the block's 192-bit string (may straddle two dwords)
      const uint32_t code = (bm_sign << 5) | bm_code<6>(mx);
      const uint32_t bit = 6u * pos, wd = bit >> 5, sh = bit & 31u;
      const uint64_t m = (uint64_t)0x3Fu << sh, cc = (uint64_t)code << sh;
#pragma unroll
      for (int j = 0; j < 6; ++j) {
        if (wd == (uint32_t)j) c6[j] = (c6[j] & ~(uint32_t)m) | (uint32_t)cc;
        if (wd + 1u == (uint32_t)j) c6[j] = (c6[j] & ~(uint32_t)(m >> 32)) | (uint32_t)(cc >> 32);
      }
    }
    uint32_t idx = pos;
    sbyte = (uint32_t)sb;
    if (flush || nonfinite) {
#pragma unroll
      for (int j = 0; j < 6; ++j) c6[j] = 0;
      idx = 0;
      sbyte = nonfinite ? 255u : 0u;
    }
    if (elems) {
      const int64_t b = row * nbk + kb;
      u32x2* e = reinterpret_cast<u32x2*>(elems + b * 24);
      e[0] = u32x2{c6[0], c6[1]};
      e[1] = u32x2{c6[2], c6[3]};
      e[2] = u32x2{c6[4], c6[5]};
      scales[b] = (uint8_t)sbyte;
      if (PLUS) bm_idx[b] = (uint8_t)idx;
    }
#pragma unroll
    for (int j = 0; j < 6; ++j) d[j] = c6[j];
    if (PLUS && sbyte != 0u && sbyte != 255u) bm = idx;
  }
  fp6_segments_out<PLUS>(d, sbyte, bm, tiles, tile_scales, rt, kt0, kts, n_seg, res_mask, img_elems, img_scales);
}

// Plain MXFP8 operand -> E4M3 image: the elements are the FP8 codes the MFMA takes and the scale byte is the block's
// (e_max only enters the conversion).  Register layout of the FP8 operand: codes 0..15 of block (kb % 2) in register
// half (kb % 2) of lane r, codes 16..31 in the same half of lane r + 32.
__global__ void __launch_bounds__(256) prepack_fp8_kernel(const uint8_t* __restrict__ elems, const uint8_t* __restrict__ scales,
                                                          int64_t rows, int64_t nbk, int64_t k_tiles,
                                                          uint8_t* __restrict__ img_elems, uint8_t* __restrict__ img_scales) {
  __shared__ __attribute__((aligned(16))) uint8_t tiles[4 * kTileBytesE4M3];
  __shared__ uint8_t tile_scales[4 * 64];
  const uint32_t t = threadIdx.x;
  const uint32_t r_in = t >> 3, kb_in = t & 7u;
  const PatchMap pm = patch_of_workgroup(blockIdx.x, (uint32_t)((k_tiles + 3) / 4), (uint32_t)(((rows + kRowPad - 1) / kRowPad) * 2));
  if (!pm.valid) return;
  const int64_t kt0 = pm.kg * 4, rt = pm.rt;
  const int64_t row = rt * kTileRows + r_in, kb = kt0 * 2 + kb_in;
  u32x4 c0 = {0, 0, 0, 0}, c1 = {0, 0, 0, 0};
  uint32_t sbyte = 127u;
  if (row < rows && kb < nbk) {
    const int64_t b = row * nbk + kb;
    const u32x4* src = reinterpret_cast<const u32x4*>(elems + b * 32);
    sbyte = scales[b];
    if (sbyte != 0u) { c0 = __builtin_nontemporal_load(src); c1 = __builtin_nontemporal_load(src + 1); }
    else sbyte = 127u;                                        // flushed: zeros with a unit scale
  }
  uint8_t* tile = tiles + (kb_in >> 1) * kTileBytesE4M3 + (kb_in & 1u) * 1024u;
  *reinterpret_cast<u32x4*>(tile + r_in * 16u) = c0;
  *reinterpret_cast<u32x4*>(tile + (32u + r_in) * 16u) = c1;
  tile_scales[(kb_in >> 1) * 64u + (kb_in & 1u) * 32u + r_in] = (uint8_t)sbyte;
  __syncthreads();
  const int64_t nt = k_tiles - kt0 < 4 ? k_tiles - kt0 : 4;
  uint8_t* out = img_elems + (rt * k_tiles + kt0) * (int64_t)kTileBytesE4M3;
  const uint32_t nbytes = (uint32_t)nt * kTileBytesE4M3;
  for (uint32_t o = t * 16u; o < nbytes; o += 256u * 16u)
    MXP_IMAGE_STORE(*reinterpret_cast<const u32x4*>(tiles + o), reinterpret_cast<u32x4*>(out + o));
  if ((int64_t)(t >> 6) < nt) img_scales[(((rt >> 2) * k_tiles + kt0 + (t >> 6)) * 64 + (t & 63u)) * 4 + (rt & 3)] = tile_scales[t];
}

}  // namespace

namespace mxp {

bool is_wide_format(int fmt) { return fmt >= MXP_FMT_MXFP6 && fmt <= MXP_FMT_MXFP8P; }

int wide_quantize_launch(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t ld_src, int fmt, uint8_t* elems,
                         uint8_t* scales, uint8_t* bm_idx, hipStream_t s) {
  const int64_t nbk = K / kBlock, nq = rows * nbk * 4;
  const dim3 grid = grid_for(nq);
  const bool bf = src_dtype == MXP_BF16;
#define MXP_LAUNCH_QW(B, BT, P) hipLaunchKernelGGL((quantize_wide_kernel<B, BT, P>), grid, dim3(256), 0, s, src, nbk, ld_src, nq, elems, scales, bm_idx)
  switch (fmt) {
#define MXP_LAUNCH_Q6(B, P) hipLaunchKernelGGL((quantize_fp6_kernel<B, P>), grid, dim3(256), 0, s, src, nbk, ld_src, nq, elems, scales, bm_idx)
    case MXP_FMT_MXFP6: if (bf) MXP_LAUNCH_Q6(true, false); else MXP_LAUNCH_Q6(false, false); break;
    case MXP_FMT_MXFP6P: if (bf) MXP_LAUNCH_Q6(true, true); else MXP_LAUNCH_Q6(false, true); break;
#undef MXP_LAUNCH_Q6
    case MXP_FMT_MXFP8: if (bf) MXP_LAUNCH_QW(true, 8, false); else MXP_LAUNCH_QW(false, 8, false); break;
    case MXP_FMT_MXFP8P: if (bf) MXP_LAUNCH_QW(true, 8, true); else MXP_LAUNCH_QW(false, 8, true); break;
    default: return MXP_ERR_FORMAT;
  }
#undef MXP_LAUNCH_QW
  return launch_status();
}

int wide_dequantize_launch(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows,
                           int64_t K, void* dst, int dst_dtype, int64_t ld_dst, hipStream_t s) {
  const int64_t nbk = K / kBlock, nq = rows * nbk * 4;
  const dim3 grid = grid_for(nq);
  const bool bf = dst_dtype == MXP_BF16;
#define MXP_LAUNCH_DW(BT, P, O) hipLaunchKernelGGL((dequantize_wide_kernel<BT, P, O>), grid, dim3(256), 0, s, elems, scales, bm_idx, nbk, ld_dst, nq, dst)
  switch (fmt) {
    case MXP_FMT_MXFP6: if (bf) MXP_LAUNCH_DW(6, false, true); else MXP_LAUNCH_DW(6, false, false); break;
    case MXP_FMT_MXFP6P: if (bf) MXP_LAUNCH_DW(6, true, true); else MXP_LAUNCH_DW(6, true, false); break;
    case MXP_FMT_MXFP8: if (bf) MXP_LAUNCH_DW(8, false, true); else MXP_LAUNCH_DW(8, false, false); break;
    case MXP_FMT_MXFP8P: if (bf) MXP_LAUNCH_DW(8, true, true); else MXP_LAUNCH_DW(8, true, false); break;
    default: return MXP_ERR_FORMAT;
  }
#undef MXP_LAUNCH_DW
  return launch_status();
}

int prepack_fp6_launch(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows, int64_t K,
                       int n_seg, uint32_t res_mask, void* image, hipStream_t stream) {
  const ImageGeom seg = image_geom(rows, K), g = image_geom(rows, seg.K_p * n_seg);
  uint8_t* ie = static_cast<uint8_t*>(image);
  uint8_t* is = ie + g.elem_bytes;
  const int64_t n_wg = patch_grid((seg.k_tiles + 3) / 4, seg.row_tiles / 4);
  if (n_wg > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  dim3 grid((unsigned)n_wg);
  if (fmt == MXP_FMT_MXFP6P)
    hipLaunchKernelGGL((prepack_fp6_kernel<true>), grid, dim3(256), 0, stream, elems, scales, bm_idx, rows, K / kBlock, seg.k_tiles,
                       n_seg, res_mask, ie, is);
  else
    hipLaunchKernelGGL((prepack_fp6_kernel<false>), grid, dim3(256), 0, stream, elems, scales, bm_idx, rows, K / kBlock, seg.k_tiles,
                       n_seg, 0u, ie, is);
  return launch_status();
}

int quantize_image_fp6_launch(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t ld, int fmt, int n_seg, uint32_t res_mask,
                              uint8_t* elems, uint8_t* scales, uint8_t* bm_idx, void* image, hipStream_t stream) {
  const ImageGeom seg = image_geom(rows, K), g = image_geom(rows, seg.K_p * n_seg);
  uint8_t* ie = static_cast<uint8_t*>(image);
  uint8_t* is = ie + g.elem_bytes;
  const int64_t n_wg = patch_grid((seg.k_tiles + 3) / 4, seg.row_tiles / 4);
  if (n_wg > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)n_wg);
  const bool bf = src_dtype == MXP_BF16, plus = fmt == MXP_FMT_MXFP6P;
#define MXP_QI6(B, P) hipLaunchKernelGGL((quantize_image_fp6_kernel<B, P>), grid, dim3(256), 0, stream, src, rows, K / kBlock, ld, seg.k_tiles, \
                                         n_seg, plus ? res_mask : 0u, elems, scales, bm_idx, ie, is)
  if (bf) { if (plus) MXP_QI6(true, true); else MXP_QI6(true, false); }
  else    { if (plus) MXP_QI6(false, true); else MXP_QI6(false, false); }
#undef MXP_QI6
  return launch_status();
}

int prepack_fp8_launch(const uint8_t* elems, const uint8_t* scales, int64_t rows, int64_t K, void* image, hipStream_t stream) {
  const ImageGeom g = image_geom(rows, K, kTileBytesE4M3);
  uint8_t* ie = static_cast<uint8_t*>(image);
  const int64_t n_wg = patch_grid((g.k_tiles + 3) / 4, g.row_tiles / 4);
  if (n_wg > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(prepack_fp8_kernel, dim3((unsigned)n_wg), dim3(256), 0, stream, elems, scales, rows, K / kBlock, g.k_tiles, ie,
                     ie + g.elem_bytes);
  return launch_status();
}

}  // namespace mxp

extern "C" size_t mxp_image_bytes_fp6(int64_t rows, int64_t K, int n_seg) {
  if (rows < 0 || K < 0 || n_seg < 1 || n_seg > 4) return 0;
  return (size_t)mxp::image_geom(rows, mxp::image_geom(rows, K).K_p * n_seg).total();
}

extern "C" int mxp_prepack_fp6(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows,
                               int64_t K, int n_seg, unsigned res_mask, void* image, size_t image_bytes, void* stream) {
  using namespace mxp;
  if (fmt != MXP_FMT_MXFP6 && fmt != MXP_FMT_MXFP6P) return MXP_ERR_FORMAT;
  if (rows < 0 || K < 0 || K % kBlock != 0 || n_seg < 1 || n_seg > 4 || (res_mask >> n_seg) != 0u) return MXP_ERR_SHAPE;
  if (fmt == MXP_FMT_MXFP6 && res_mask != 0u) return MXP_ERR_SHAPE;     // a plain operand has no residual
  if (rows == 0 || K == 0) return MXP_OK;
  if (!elems || !scales || !image || (fmt == MXP_FMT_MXFP6P && !bm_idx)) return MXP_ERR_NULL;
  if (!aligned16(elems) || !aligned16(scales) || !aligned16(image) || (bm_idx && !aligned16(bm_idx))) return MXP_ERR_ALIGN;
  if (image_bytes < mxp_image_bytes_fp6(rows, K, n_seg)) return MXP_ERR_WORKSPACE;
  return prepack_fp6_launch(elems, scales, bm_idx, fmt, rows, K, n_seg, res_mask, image, static_cast<hipStream_t>(stream));
}

extern "C" int mxp_quantize_image_fp6(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t ld_src, int fmt, int n_seg,
                                      unsigned res_mask, uint8_t* elems, uint8_t* scales, uint8_t* bm_idx, void* image,
                                      size_t image_bytes, void* stream) {
  using namespace mxp;
  if (fmt != MXP_FMT_MXFP6 && fmt != MXP_FMT_MXFP6P) return MXP_ERR_FORMAT;
  if (src_dtype != MXP_F32 && src_dtype != MXP_BF16) return MXP_ERR_DTYPE;
  if (rows < 0 || K < 0 || K % kBlock != 0 || n_seg < 1 || n_seg > 4 || (res_mask >> n_seg) != 0u) return MXP_ERR_SHAPE;
  if (fmt == MXP_FMT_MXFP6 && res_mask != 0u) return MXP_ERR_SHAPE;     // a plain operand has no residual
  if (rows == 0 || K == 0) return MXP_OK;
  if (!src || !image) return MXP_ERR_NULL;
  const bool canon = elems || scales || bm_idx;
  if (canon && (!elems || !scales || (fmt == MXP_FMT_MXFP6P && !bm_idx))) return MXP_ERR_NULL;
  if (ld_src < K) return MXP_ERR_SHAPE;
  const int64_t esz = src_dtype == MXP_BF16 ? 2 : 4;
  if (!aligned16(src) || (ld_src * esz) % 16 != 0 || !aligned16(image)) return MXP_ERR_ALIGN;
  if (canon && (!aligned16(elems) || !aligned16(scales) || (bm_idx && !aligned16(bm_idx)))) return MXP_ERR_ALIGN;
  if (image_bytes < mxp_image_bytes_fp6(rows, K, n_seg)) return MXP_ERR_WORKSPACE;
  return quantize_image_fp6_launch(src, src_dtype, rows, K, ld_src, fmt, n_seg, res_mask, elems, scales, bm_idx, image,
                                   static_cast<hipStream_t>(stream));
}

extern "C" int mxp_prepack_fp8(const uint8_t* elems, const uint8_t* scales, int64_t rows, int64_t K, void* image,
                               size_t image_bytes, void* stream) {
  using namespace mxp;
  if (rows < 0 || K < 0 || K % kBlock != 0) return MXP_ERR_SHAPE;
  if (rows == 0 || K == 0) return MXP_OK;
  if (!elems || !scales || !image) return MXP_ERR_NULL;
  if (!aligned16(elems) || !aligned16(scales) || !aligned16(image)) return MXP_ERR_ALIGN;
  if (image_bytes < (size_t)image_geom(rows, K, kTileBytesE4M3).total()) return MXP_ERR_WORKSPACE;
  return prepack_fp8_launch(elems, scales, rows, K, image, static_cast<hipStream_t>(stream));
}
