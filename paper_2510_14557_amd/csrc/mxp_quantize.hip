// mxp_quantize / mxp_quantize_t : fp32 or bf16  ->  canonical MXFP4 / MXFP4+  (Sec. 4.1, 4.2, Eq. 1).
//
// HBM-bound streaming kernel.  Four lanes share one 32-element block: a lane loads 8 consecutive elements with
// 16-byte loads (a wavefront reads 1 KiB of bf16 contiguously), the block maximum and its position are found with
// two DPP quad exchanges, the eight elements are rounded by the CDNA4 pack-convert instruction (round to nearest
// even, saturating, sign kept -- the element rounding the format fixes), the lane owning the BM overwrites that
// nibble with the 3-bit extended mantissa, and each lane stores one dword of nibbles.  Scale and index bytes of
// four neighbouring blocks are gathered into one lane and stored as dwords.
#include "mxp_common.h"
#include "mxp_prepack_body.h"
#include <type_traits>

namespace {

using namespace mxp;

typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
constexpr int kQuadSwap1 = 0xB1;  // quad_perm [1,0,3,2]
constexpr int kQuadSwap2 = 0x4E;  // quad_perm [2,3,0,1]
constexpr int kRowShr4 = 0x114;
constexpr int kRowShr8 = 0x118;

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }

// 3-bit BM mantissa from the 23-bit fraction of the block maximum: round to nearest even on bit 20, and a carry
// out of the field saturates (the shared scale is never altered, Sec. 4.1).
__device__ __forceinline__ uint32_t bm_mantissa(uint32_t frac23) {
  uint32_t m = (frac23 + 0x7FFFFu + ((frac23 >> 20) & 1u)) >> 20;
  return umin(m, 7u);
}

// One group = 8 consecutive elements of one block, held by one lane.  `part` = which quarter of the block.
// Returns the packed dword of 8 nibbles; scale byte and index byte are returned in all four lanes of the quad.
// MODE: 0 = MXFP4, 1 = MXFP4+, 2 = MXFP4++ (Sec. 4.3: the NBMs are scaled by 2^(shared_exp - delta), where
// shared_exp - delta = CLIP(largest NBM exponent - e_max + 1, {shared_exp - 7, shared_exp}), and delta goes into bits
// 7:5 of the index byte; delta is also kept <= scale byte - 1 so that the NBM scale stays an E8M0 number).
template <bool BF16, int MODE>
__device__ __forceinline__ uint32_t encode_group(const uint32_t (&w)[8], int part, uint32_t& sbyte, uint32_t& idx) {
  constexpr bool PLUS = MODE >= 1, PP = MODE == 2;
  uint32_t amax32;  // magnitude bits of the block maximum, as an fp32 pattern
  uint32_t a2 = 0;  // (PP) magnitude bits of the largest element other than the BM
  if (BF16) {
    // key = magnitude(15 bit) << 16 | (31 - position): one unsigned max gives the maximum and, among equal
    // magnitudes, the lowest position.
    uint32_t k = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint32_t m = w[j] & 0x7FFF7FFFu;
      uint32_t klo = (m << 16) | (uint32_t)(7 - 2 * j);
      uint32_t khi = (m & 0xFFFF0000u) | (uint32_t)(6 - 2 * j);
      k = umax(k, umax(klo, khi));
    }
    k += (uint32_t)(3 - part) * 8u;
    k = umax(k, dpp_mov<kQuadSwap1>(k));
    k = umax(k, dpp_mov<kQuadSwap2>(k));
    amax32 = k & 0xFFFF0000u;
    idx = 31u - (k & 31u);
    if (PP) {
      // keys are unique (the position is part of them): the lane whose best key won leaves that element out
      uint32_t k2 = 0;
      const uint32_t off = (uint32_t)(3 - part) * 8u;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t m = w[j] & 0x7FFF7FFFu;
        const uint32_t klo = ((m << 16) | (uint32_t)(7 - 2 * j)) + off;
        const uint32_t khi = ((m & 0xFFFF0000u) | (uint32_t)(6 - 2 * j)) + off;
        k2 = umax(k2, klo == k ? 0u : klo);
        k2 = umax(k2, khi == k ? 0u : khi);
      }
      k2 = umax(k2, dpp_mov<kQuadSwap1>(k2));
      k2 = umax(k2, dpp_mov<kQuadSwap2>(k2));
      a2 = k2 & 0xFFFF0000u;
    }
  } else {
    uint32_t a[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = w[i] & 0x7FFFFFFFu;
    uint32_t mx = a[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) mx = umax(mx, a[i]);
    mx = umax(mx, dpp_mov<kQuadSwap1>(mx));
    mx = umax(mx, dpp_mov<kQuadSwap2>(mx));
    uint32_t p = 32u;
#pragma unroll
    for (int i = 7; i >= 0; --i) p = (a[i] == mx) ? (uint32_t)(part * 8 + i) : p;
    p = umin(p, dpp_mov<kQuadSwap1>(p));
    p = umin(p, dpp_mov<kQuadSwap2>(p));
    amax32 = mx;
    idx = p;
    if (PP) {
      uint32_t m2 = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) m2 = umax(m2, (uint32_t)(part * 8 + i) == p ? 0u : a[i]);
      m2 = umax(m2, dpp_mov<kQuadSwap1>(m2));
      m2 = umax(m2, dpp_mov<kQuadSwap2>(m2));
      a2 = m2;
    }
  }
  const uint32_t E = amax32 >> 23;                     // biased exponent of the BM = floor(log2) + 127
  const bool flush = E <= 2u;                          // floor(log2 BM) <= -127 + e_max      (Sec. 4.1)
  const bool nonfinite = E == 255u;
  uint32_t delta = 0;
  if (PP) {
    const uint32_t sb = E - 2u, E2 = a2 >> 23;                       // biased: BM scale; exponent of the largest NBM
    const uint32_t lo = sb > 7u ? sb - 7u : 0u;                      // (flushed blocks are reset below)
    uint32_t nb = E2 == 0u ? lo : umin(umax(E2 - 1u, lo), sb);       // biased shared_exp_new = E2 - 127 - e_max + 1 + 127
    nb = umax(nb, 1u);
    delta = sb - nb;
  }
  // X = 2^shared_exp, shared_exp = floor(log2 BM) - e_max (Eq. 1); the NBMs of MXFP4++ use 2^(shared_exp - delta)
  const float scale = __uint_as_float((E - 2u - delta) << 23);
  uint32_t packed = 0;
  if (BF16) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      union { uint32_t u; v2bf v; } c;
      c.u = w[j];
      if (j == 0) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(packed, c.v, scale, 0);
      if (j == 1) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(packed, c.v, scale, 1);
      if (j == 2) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(packed, c.v, scale, 2);
      if (j == 3) packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(packed, c.v, scale, 3);
    }
  } else {
    packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, __uint_as_float(w[0]), __uint_as_float(w[1]), scale, 0);
    packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, __uint_as_float(w[2]), __uint_as_float(w[3]), scale, 1);
    packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, __uint_as_float(w[4]), __uint_as_float(w[5]), scale, 2);
    packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, __uint_as_float(w[6]), __uint_as_float(w[7]), scale, 3);
  }
  if (PLUS) {
    // BM nibble = sign | m2 m1 m0 ; the sign is already in the converted nibble.
    const uint32_t m3 = bm_mantissa(amax32 & 0x7FFFFFu);
    const uint32_t sh = (idx & 7u) * 4u;
    const uint32_t nib = ((packed >> sh) & 8u) | m3;
    const uint32_t repl = (packed & ~(0xFu << sh)) | (nib << sh);
    packed = ((idx >> 3) == (uint32_t)part) ? repl : packed;
  }
  sbyte = E - 2u;
  if (PP) idx |= delta << 5;
  if (flush || nonfinite) {
    packed = 0;
    idx = 0;
    sbyte = nonfinite ? 255u : 0u;
  }
  return packed;
}

template <bool BF16>
__device__ __forceinline__ void load_group(const void* __restrict__ src, int64_t q, int64_t nbk, int64_t ld, bool dense,
                                           uint32_t (&w)[8]) {
  int64_t off;
  if (dense) {
    off = q * 8;
  } else {
    const int64_t g = q >> 2;
    const int64_t row = g / nbk;
    off = row * ld + (g - row * nbk) * 32 + (q & 3) * 8;
  }
  if (BF16) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(src) + off));
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    w[4] = w[5] = w[6] = w[7] = 0;
  } else {
    const u32x4* p = reinterpret_cast<const u32x4*>(static_cast<const float*>(src) + off);
    const u32x4 v0 = __builtin_nontemporal_load(p), v1 = __builtin_nontemporal_load(p + 1);
    w[0] = v0.x; w[1] = v0.y; w[2] = v0.z; w[3] = v0.w;
    w[4] = v1.x; w[5] = v1.y; w[6] = v1.z; w[7] = v1.w;
  }
}

// nq = number of 8-element groups (= 4 * blocks).  The loop is uniform per 16-lane row, so DPP exchanges never
// read a lane that left the loop; lanes past the end compute on zeros and store nothing.
template <bool BF16, int MODE, int U>
__global__ void __launch_bounds__(256) quantize_kernel(const void* __restrict__ src, int64_t nbk, int64_t ld, int dense,
                                                       int64_t nq, uint32_t* __restrict__ elems,
                                                       uint8_t* __restrict__ scales, uint8_t* __restrict__ bm_idx) {
  constexpr bool PLUS = MODE >= 1;
  const int part = threadIdx.x & 3;
  const int quad_in_row = (threadIdx.x & 15) >> 2;
  const int64_t stride = (int64_t)gridDim.x * 256;
  const int64_t nblocks = nq >> 2;
  for (int64_t q0 = (int64_t)blockIdx.x * 256 + threadIdx.x; (q0 & ~(int64_t)15) < nq; q0 += stride * U) {
    uint32_t w[U][8];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = q0 + u * stride;
      if (q < nq) {
        load_group<BF16>(src, q, nbk, ld, dense != 0, w[u]);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) w[u][i] = 0;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = q0 + u * stride;
      if ((q & ~(int64_t)15) >= nq) break;
      uint32_t sbyte, idx;
      const uint32_t packed = encode_group<BF16, MODE>(w[u], part, sbyte, idx);
      if (q < nq) __builtin_nontemporal_store(packed, elems + q);
      // gather the four blocks of this 16-lane row into its lane 12
      uint32_t sv = (part == 0) ? (sbyte << (8 * quad_in_row)) : 0u;
      sv |= dpp_mov<kRowShr8>(sv);
      sv |= dpp_mov<kRowShr4>(sv);
      uint32_t iv = 0;
      if (PLUS) {
        iv = (part == 0) ? (idx << (8 * quad_in_row)) : 0u;
        iv |= dpp_mov<kRowShr8>(iv);
        iv |= dpp_mov<kRowShr4>(iv);
      }
      const int64_t g0 = (q & ~(int64_t)15) >> 2;   // first block of the row
      if (g0 + 4 <= nblocks) {
        if ((threadIdx.x & 15) == 12) {
          *reinterpret_cast<uint32_t*>(scales + g0) = sv;
          if (PLUS) *reinterpret_cast<uint32_t*>(bm_idx + g0) = iv;
        }
      } else if (part == 0 && q < nq) {
        scales[q >> 2] = (uint8_t)sbyte;
        if (PLUS) bm_idx[q >> 2] = (uint8_t)idx;
      }
    }
  }
}

// Dense source (row stride = K): the tensor is one run of nq 8-element groups.  A workgroup walks chunks of 256 * U
// groups (U x 4 KiB of bf16, contiguous); lane t of the workgroup takes groups u * 256 + t of the chunk, so every
// load, every element store and every scale / index dword store of a wavefront is one contiguous run.  Whole chunks
// run without per-lane bounds tests; the last, partial chunk takes the checked path.
template <bool BF16, int MODE, int U>
__global__ void __launch_bounds__(256) quantize_dense_kernel(const void* __restrict__ src, int64_t nq, uint32_t* __restrict__ elems,
                                                             uint8_t* __restrict__ scales, uint8_t* __restrict__ bm_idx) {
  constexpr bool PLUS = MODE >= 1;
  const uint32_t t = threadIdx.x, part = t & 3u, quad_in_row = (t & 15u) >> 2;
  constexpr int64_t kChunk = 256 * U;
  const int64_t n_chunks = (nq + kChunk - 1) / kChunk;
  for (int64_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    const int64_t q_base = c * kChunk;                               // uniform
    const bool whole = q_base + kChunk <= nq;
    uint32_t w[U][8];
    if (BF16) {
      const u32x4* p = reinterpret_cast<const u32x4*>(src) + q_base;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        u32x4 v = {0, 0, 0, 0};
        if (whole || q_base + u * 256 + t < nq) v = __builtin_nontemporal_load(p + u * 256 + t);
        w[u][0] = v.x; w[u][1] = v.y; w[u][2] = v.z; w[u][3] = v.w;
        w[u][4] = w[u][5] = w[u][6] = w[u][7] = 0;
      }
    } else {
      const u32x4* p = reinterpret_cast<const u32x4*>(src) + 2 * q_base;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        u32x4 v0 = {0, 0, 0, 0}, v1 = {0, 0, 0, 0};
        if (whole || q_base + u * 256 + t < nq) {
          v0 = __builtin_nontemporal_load(p + 2 * (u * 256 + t));
          v1 = __builtin_nontemporal_load(p + 2 * (u * 256 + t) + 1);
        }
        w[u][0] = v0.x; w[u][1] = v0.y; w[u][2] = v0.z; w[u][3] = v0.w;
        w[u][4] = v1.x; w[u][5] = v1.y; w[u][6] = v1.z; w[u][7] = v1.w;
      }
    }
    uint32_t* e_out = elems + q_base;
    uint8_t* s_out = scales + (q_base >> 2);
    uint8_t* i_out = bm_idx + (q_base >> 2);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      uint32_t sbyte, idx;
      const uint32_t packed = encode_group<BF16, MODE>(w[u], (int)part, sbyte, idx);
      // gather the four blocks of this 16-lane row into its lane 12
      uint32_t sv = (part == 0) ? (sbyte << (8 * quad_in_row)) : 0u;
      sv |= dpp_mov<kRowShr8>(sv);
      sv |= dpp_mov<kRowShr4>(sv);
      uint32_t iv = 0;
      if (PLUS) {
        iv = (part == 0) ? (idx << (8 * quad_in_row)) : 0u;
        iv |= dpp_mov<kRowShr8>(iv);
        iv |= dpp_mov<kRowShr4>(iv);
      }
      const uint32_t ql = u * 256 + t;                               // group within the chunk
      if (whole) {
        __builtin_nontemporal_store(packed, e_out + ql);
        if ((t & 15u) == 12u) {
          *reinterpret_cast<uint32_t*>(s_out + (ql >> 2) - 3) = sv;
          if (PLUS) *reinterpret_cast<uint32_t*>(i_out + (ql >> 2) - 3) = iv;
        }
      } else if (q_base + ql < nq) {
        __builtin_nontemporal_store(packed, e_out + ql);
        if (q_base + (ql | 15u) < nq) {                              // the row's four blocks all exist
          if ((t & 15u) == 12u) {
            *reinterpret_cast<uint32_t*>(s_out + (ql >> 2) - 3) = sv;
            if (PLUS) *reinterpret_cast<uint32_t*>(i_out + (ql >> 2) - 3) = iv;
          }
        } else if (part == 0) {
          s_out[ql >> 2] = (uint8_t)sbyte;
          if (PLUS) i_out[ql >> 2] = (uint8_t)idx;
        }
      }
    }
  }
}

// ---- channel-reordered source (Sec. 9, "Scattering Outliers with Channel Reordering"): block element k of a row is
// source channel perm[k], so that outlier channels can be dealt one per block.  The reordering costs no extra pass: the
// lane gathers its eight elements through the permutation (entries are clamped to the row, so a bad table cannot
// read outside it) and the encoding and the stores are those of the ordinary kernel.
template <bool BF16, int MODE>
__global__ void __launch_bounds__(256) quantize_gather_kernel(const void* __restrict__ src, int64_t nbk, int64_t ld,
                                                              const int32_t* __restrict__ perm, int64_t n_src, int64_t nq,
                                                              uint32_t* __restrict__ elems, uint8_t* __restrict__ scales,
                                                              uint8_t* __restrict__ bm_idx) {
  constexpr bool PLUS = MODE >= 1;
  const int part = threadIdx.x & 3;
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; (q & ~(int64_t)3) < nq; q += stride) {
    uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const bool ok = q < nq;                                  // nq is a multiple of 4: a quad is in or out as a whole
    if (ok) {
      const int64_t g = q >> 2, row = g / nbk, kb = g - row * nbk;
      const int32_t* pp = perm + kb * 32 + part * 8;
      uint32_t v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        int64_t c = pp[i];
        c = c < 0 ? 0 : (c >= n_src ? n_src - 1 : c);
        v[i] = BF16 ? (uint32_t) static_cast<const uint16_t*>(src)[row * ld + c] : static_cast<const uint32_t*>(src)[row * ld + c];
      }
      if (BF16) {
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = v[2 * j] | (v[2 * j + 1] << 16);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = v[i];
      }
    }
    uint32_t sbyte, idx;
    const uint32_t packed = encode_group<BF16, MODE>(w, part, sbyte, idx);
    if (ok) {
      __builtin_nontemporal_store(packed, elems + q);
      if (part == 0) {
        scales[q >> 2] = (uint8_t)sbyte;
        if (PLUS) bm_idx[q >> 2] = (uint8_t)idx;
      }
    }
  }
}

// Same, for rows that fit in LDS (the usual case: a few thousand channels).  A workgroup walks rows; a row is read the
// way it lies in memory (16 bytes per lane) into LDS and the lanes gather their elements from there, so HBM sees only
// full-width loads.  Lane t encodes groups t, t + 256, ... of every row it meets, hence its part of the permutation is
// read once, up front, and kept in registers (as byte offsets into the LDS row).
template <bool BF16, int MODE, int GP>
__global__ void __launch_bounds__(256) quantize_gather_lds_kernel(const void* __restrict__ src, int64_t rows, int64_t nbk, int64_t ld,
                                                                  const int32_t* __restrict__ perm, int64_t n_src,
                                                                  uint32_t* __restrict__ elems, uint8_t* __restrict__ scales,
                                                                  uint8_t* __restrict__ bm_idx) {
  constexpr bool PLUS = MODE >= 1;
  constexpr int ESZ = BF16 ? 2 : 4;
  extern __shared__ __attribute__((aligned(16))) uint8_t row_lds[];
  const int t = threadIdx.x, part = t & 3;
  const int64_t groups = nbk * 4;                            // 8-element groups per output row (a multiple of 4)
  uint32_t off[GP][8];
#pragma unroll
  for (int u = 0; u < GP; ++u) {
    const int64_t g = t + 256 * u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int64_t c = g < groups ? perm[g * 8 + i] : 0;
      c = c < 0 ? 0 : (c >= n_src ? n_src - 1 : c);
      off[u][i] = (uint32_t)c * ESZ;
    }
  }
  const int64_t row_bytes = n_src * ESZ;
  const bool vec_ok = (ld * ESZ) % 16 == 0;                  // rows start 16-byte aligned (src is)
  for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
    const uint8_t* rp = static_cast<const uint8_t*>(src) + row * ld * ESZ;
    __syncthreads();                                         // everyone is done with the previous row
    if (vec_ok) {
      for (int64_t o = (int64_t)t * 16; o < row_bytes; o += 256 * 16) {
        if (o + 16 <= row_bytes) {
          *reinterpret_cast<u32x4*>(row_lds + o) = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(rp + o));
        } else {
          for (int64_t b = o; b < row_bytes; b += ESZ) {
            if (BF16) *reinterpret_cast<uint16_t*>(row_lds + b) = *reinterpret_cast<const uint16_t*>(rp + b);
            else *reinterpret_cast<uint32_t*>(row_lds + b) = *reinterpret_cast<const uint32_t*>(rp + b);
          }
        }
      }
    } else {
      for (int64_t b = (int64_t)t * ESZ; b < row_bytes; b += 256 * ESZ) {
        if (BF16) *reinterpret_cast<uint16_t*>(row_lds + b) = *reinterpret_cast<const uint16_t*>(rp + b);
        else *reinterpret_cast<uint32_t*>(row_lds + b) = *reinterpret_cast<const uint32_t*>(rp + b);
      }
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < GP; ++u) {
      const int64_t g = t + 256 * u;
      if ((g & ~(int64_t)3) >= groups) break;                // whole quads leave together (DPP exchanges inside the encode)
      uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      if (BF16) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          w[j] = (uint32_t)*reinterpret_cast<const uint16_t*>(row_lds + off[u][2 * j]) |
                 ((uint32_t)*reinterpret_cast<const uint16_t*>(row_lds + off[u][2 * j + 1]) << 16);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = *reinterpret_cast<const uint32_t*>(row_lds + off[u][i]);
      }
      uint32_t sbyte, idx;
      const uint32_t packed = encode_group<BF16, MODE>(w, part, sbyte, idx);
      const int64_t q = row * groups + g;
      __builtin_nontemporal_store(packed, elems + q);
      if (part == 0) {
        scales[q >> 2] = (uint8_t)sbyte;
        if (PLUS) bm_idx[q >> 2] = (uint8_t)idx;
      }
    }
  }
}

// ---- K-strided source -------------------------------------------------------------------------------------------
// One lane encodes a whole block held in registers as 32 fp32 patterns (same decisions as encode_group: Eq. 1,
// Sec. 4.1-4.3, lowest-position maximum).
template <int MODE>
__device__ __forceinline__ void encode_block_serial(const uint32_t (&x)[32], uint32_t (&out)[4], uint32_t& sbyte,
                                                    uint32_t& idx) {
  constexpr bool PLUS = MODE >= 1, PP = MODE == 2;
  uint32_t mx = 0;
#pragma unroll
  for (int i = 0; i < 32; ++i) mx = umax(mx, x[i] & 0x7FFFFFFFu);
  idx = 32;
#pragma unroll
  for (int i = 31; i >= 0; --i) idx = ((x[i] & 0x7FFFFFFFu) == mx) ? (uint32_t)i : idx;
  const uint32_t E = mx >> 23;
  uint32_t delta = 0;
  if (PP) {                                                         // Sec. 4.3: finer scale for the NBMs
    uint32_t m2 = 0;
#pragma unroll
    for (int i = 0; i < 32; ++i) m2 = umax(m2, (uint32_t)i == idx ? 0u : (x[i] & 0x7FFFFFFFu));
    const uint32_t sb = E - 2u, E2 = m2 >> 23;
    const uint32_t lo = sb > 7u ? sb - 7u : 0u;
    uint32_t nb = E2 == 0u ? lo : umin(umax(E2 - 1u, lo), sb);
    nb = umax(nb, 1u);
    delta = sb - nb;
  }
  const float scale = __uint_as_float((E - 2u - delta) << 23);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    uint32_t p = 0;
    p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, __uint_as_float(x[8 * j + 0]), __uint_as_float(x[8 * j + 1]), scale, 0);
    p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, __uint_as_float(x[8 * j + 2]), __uint_as_float(x[8 * j + 3]), scale, 1);
    p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, __uint_as_float(x[8 * j + 4]), __uint_as_float(x[8 * j + 5]), scale, 2);
    p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, __uint_as_float(x[8 * j + 6]), __uint_as_float(x[8 * j + 7]), scale, 3);
    out[j] = p;
  }
  if (PLUS) {
    const uint32_t m3 = bm_mantissa(mx & 0x7FFFFFu);
    const uint32_t sh = (idx & 7u) * 4u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t nib = ((out[j] >> sh) & 8u) | m3;
      const uint32_t repl = (out[j] & ~(0xFu << sh)) | (nib << sh);
      out[j] = ((idx >> 3) == (uint32_t)j) ? repl : out[j];
    }
  }
  sbyte = E - 2u;
  if (PP) idx |= delta << 5;
  if (E <= 2u || E == 255u) {
    out[0] = out[1] = out[2] = out[3] = 0;
    idx = 0;
    sbyte = (E == 255u) ? 255u : 0u;
  }
}

// The same for a block held as 16 words of two bf16 values each (value 2j in the low half of word j).  As in
// encode_group the position rides in the low bits of an unsigned key, so one maximum yields the BM and its position,
// and the hardware conversion takes the bf16 pairs as they are.
template <int MODE>
__device__ __forceinline__ void encode_block_serial_bf16(const uint32_t (&w)[16], uint32_t (&out)[4], uint32_t& sbyte,
                                                         uint32_t& idx) {
  constexpr bool PLUS = MODE >= 1, PP = MODE == 2;
  uint32_t key[32];
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    key[2 * j] = ((w[j] << 16) & 0x7FFF0000u) | (uint32_t)(31 - 2 * j);
    key[2 * j + 1] = (w[j] & 0x7FFF0000u) | (uint32_t)(30 - 2 * j);
  }
  uint32_t k = 0;
#pragma unroll
  for (int i = 0; i < 32; ++i) k = umax(k, key[i]);
  const uint32_t mx = k & 0xFFFF0000u;
  idx = 31u - (k & 31u);
  const uint32_t E = mx >> 23;
  uint32_t delta = 0;
  if (PP) {                                                         // Sec. 4.3: finer scale for the NBMs
    uint32_t k2 = 0;
#pragma unroll
    for (int i = 0; i < 32; ++i) k2 = umax(k2, key[i] == k ? 0u : key[i]);   // keys are unique
    const uint32_t sb = E - 2u, E2 = k2 >> 23;
    const uint32_t lo = sb > 7u ? sb - 7u : 0u;
    uint32_t nb = E2 == 0u ? lo : umin(umax(E2 - 1u, lo), sb);
    nb = umax(nb, 1u);
    delta = sb - nb;
  }
  const float scale = __uint_as_float((E - 2u - delta) << 23);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    uint32_t p = 0;
    union { uint32_t u; v2bf v; } c0, c1, c2, c3;
    c0.u = w[4 * j]; c1.u = w[4 * j + 1]; c2.u = w[4 * j + 2]; c3.u = w[4 * j + 3];
    p = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(p, c0.v, scale, 0);
    p = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(p, c1.v, scale, 1);
    p = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(p, c2.v, scale, 2);
    p = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(p, c3.v, scale, 3);
    out[j] = p;
  }
  if (PLUS) {
    const uint32_t m3 = bm_mantissa(mx & 0x7FFFFFu);
    const uint32_t sh = (idx & 7u) * 4u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t nib = ((out[j] >> sh) & 8u) | m3;
      const uint32_t repl = (out[j] & ~(0xFu << sh)) | (nib << sh);
      out[j] = ((idx >> 3) == (uint32_t)j) ? repl : out[j];
    }
  }
  sbyte = E - 2u;
  if (PP) idx |= delta << 5;
  if (E <= 2u || E == 255u) {
    out[0] = out[1] = out[2] = out[3] = 0;
    idx = 0;
    sbyte = (E == 255u) ? 255u : 0u;
  }
}

// General form (any row stride, any alignment): one thread per block, 32 strided loads that are coalesced across the
// rows of a wavefront; each lane stores its 16 element bytes and its scale / index byte on its own.
template <bool BF16, int MODE>
__global__ void __launch_bounds__(256) quantize_t_kernel(const void* __restrict__ src, int64_t rows, int64_t nbk, int64_t ld,
                                                         uint4* __restrict__ elems, uint8_t* __restrict__ scales,
                                                         uint8_t* __restrict__ bm_idx) {
  constexpr bool PLUS = MODE >= 1;
  const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t kb = blockIdx.y;
  if (r >= rows) return;
  uint32_t x[32];
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    const int64_t off = (kb * 32 + i) * ld + r;
    x[i] = BF16 ? ((uint32_t) static_cast<const uint16_t*>(src)[off]) << 16 : static_cast<const uint32_t*>(src)[off];
  }
  uint32_t out[4], sbyte, idx;
  encode_block_serial<MODE>(x, out, sbyte, idx);
  const int64_t b = r * nbk + kb;
  elems[b] = make_uint4(out[0], out[1], out[2], out[3]);
  scales[b] = (uint8_t)sbyte;
  if (PLUS) bm_idx[b] = (uint8_t)idx;
}

// Tiled form (even row stride, source aligned to two elements).  A workgroup owns kTRows = 128 rows x kTRun blocks
// of K and walks them 4 blocks at a time.  Wavefront kb of the workgroup takes block kb of the pass; its lane rp loads
// the row pair 2rp, 2rp+1, one 4- or 8-byte load per value of K, so each load instruction of a wavefront reads one
// full 256- (bf16) or 512-byte (fp32) run of a source line; the loads of the next pass are in flight while this one
// is encoded.  The lane encodes its two blocks and drops them into LDS at [row][kb].  After ACC passes the tile
// leaves row by row: ACC x 64 contiguous element bytes and ACC x 4 scale and index bytes per row (short runs per
// row are what the write side of HBM likes least: ACC = 1 costs 40 % more time than ACC = 8).
constexpr int kBufferFlags = 0x00020000;                             // raw buffer descriptor, dword 3: 32-bit data
constexpr int kTRows = 128, kTRun = 32, kTAcc = 8;

template <bool BF16, int MODE, int ACC>
__global__ void __launch_bounds__(256) quantize_t_tiled_kernel(const void* __restrict__ src, int64_t rows, int64_t nbk,
                                                               int64_t ld, uint4* __restrict__ elems,
                                                               uint8_t* __restrict__ scales, uint8_t* __restrict__ bm_idx) {
  constexpr bool PLUS = MODE >= 1;
  constexpr int R = kTRows, B = 4, C = ACC * B;                      // C = blocks of K per row in the LDS tile
  static_assert(kTRun % C == 0, "a run of K is a whole number of LDS tiles");
  __shared__ u32x4 e_lds[R][C + 1];                                  // + 1: rows land on different banks
  __shared__ __attribute__((aligned(4))) uint8_t s_lds[R][C];
  __shared__ __attribute__((aligned(4))) uint8_t i_lds[R][C];
  const uint32_t t = threadIdx.x, rp = t & 63u;
  // 64 row pairs: a wavefront shares its block of K, so the K part of every address is wave-uniform
  const uint32_t kbl = (uint32_t)__builtin_amdgcn_readfirstlane((int)(t >> 6));
  const int64_t row0 = (int64_t)blockIdx.x * R;
  const int64_t r = row0 + 2 * rp;                                   // this lane's row pair
  const int64_t kb_first = (int64_t)blockIdx.y * kTRun;
  const int64_t kb_end = kb_first + kTRun < nbk ? kb_first + kTRun : nbk;
  // 4-byte scale / index stores stay aligned
  const bool wide_meta = ((nbk | (int64_t)reinterpret_cast<uintptr_t>(scales) | (int64_t)reinterpret_cast<uintptr_t>(bm_idx)) & 3) == 0;
  // Source line k of a block starts at tile_src + k * step.  Buffer loads keep that wave-uniform part in scalar
  // registers (descriptor base + scalar offset) and the lane part in one 32-bit vector offset.  raw[k] = the lane's
  // row pair at line k of the block (one row, zero-extended, for the last row of an odd row count; zeros outside).
  constexpr int64_t kEsize = BF16 ? 2 : 4;
  using Raw = typename std::conditional<BF16, uint32_t, u32x2>::type;
  const int32_t step = (int32_t)(ld * kEsize);                       // the launcher keeps 32 * step below 2^31
  const int32_t lane_off = (int32_t)(rp * 2 * kEsize);
  auto load_block = [&](int64_t kb, Raw (&raw)[32]) {
    const uint8_t* tile_src = static_cast<const uint8_t*>(src) + (kb * 32 * ld + row0) * kEsize;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(tile_src), 0, 0x7FFFFFFF, kBufferFlags);
    if (kb < nbk && row0 + R <= rows) {                              // wave-uniform: all 64 row pairs exist
#pragma unroll
      for (int i = 0; i < 32; ++i) {
        if constexpr (BF16) raw[i] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, lane_off, i * step, 0);
        else raw[i] = __builtin_amdgcn_raw_buffer_load_b64(rsrc, lane_off, i * step, 0);
      }
    } else if (kb < nbk && r + 1 < rows) {
#pragma unroll
      for (int i = 0; i < 32; ++i) {
        if constexpr (BF16) raw[i] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, lane_off, i * step, 0);
        else raw[i] = __builtin_amdgcn_raw_buffer_load_b64(rsrc, lane_off, i * step, 0);
      }
    } else if (kb < nbk && r < rows) {
#pragma unroll
      for (int i = 0; i < 32; ++i) {
        if constexpr (BF16) raw[i] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(rsrc, lane_off, i * step, 0) & 0xFFFFu;
        else raw[i] = u32x2{(uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rsrc, lane_off, i * step, 0), 0u};
      }
    } else {
#pragma unroll
      for (int i = 0; i < 32; ++i) {
        if constexpr (BF16) raw[i] = 0u;
        else raw[i] = u32x2{0u, 0u};
      }
    }
  };
  // two blocks per lane: as 32 fp32 patterns each, or (bf16) as 16 words of two consecutive values of K each
  constexpr int NW = BF16 ? 16 : 32;
  uint32_t xa[NW], xb[NW];
  auto unpack = [&](const Raw (&raw)[32]) {
    if constexpr (BF16) {
#pragma unroll
      for (int j = 0; j < 16; ++j) {                                 // regroup into (k, k+1) pairs per row
        xa[j] = __builtin_amdgcn_perm(raw[2 * j + 1], raw[2 * j], 0x05040100u);
        xb[j] = __builtin_amdgcn_perm(raw[2 * j + 1], raw[2 * j], 0x07060302u);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 32; ++i) {
        xa[i] = raw[i].x;
        xb[i] = raw[i].y;
      }
    }
  };
  {
    Raw raw[32];
    load_block(kb_first + kbl, raw);
    unpack(raw);
  }
  uint32_t col0 = 0;                                                 // column of this pass in the LDS tile
  for (int64_t kb0 = kb_first; kb0 < kb_end; kb0 += B) {
    // the next pass's lines are requested before this pass is encoded and taken over once it has been
    Raw raw[32];
    const bool more = kb0 + B < kb_end;
    if (more) load_block(kb0 + B + kbl, raw);
    __builtin_amdgcn_sched_barrier(0);                               // (keep the loads above the encode)
    uint32_t out[4], sbyte, idx;
    const uint32_t col = col0 + kbl;
    if constexpr (BF16) encode_block_serial_bf16<MODE>(xa, out, sbyte, idx);
    else encode_block_serial<MODE>(xa, out, sbyte, idx);
    e_lds[2 * rp][col] = u32x4{out[0], out[1], out[2], out[3]};
    s_lds[2 * rp][col] = (uint8_t)sbyte;
    if (PLUS) i_lds[2 * rp][col] = (uint8_t)idx;
    if constexpr (BF16) encode_block_serial_bf16<MODE>(xb, out, sbyte, idx);
    else encode_block_serial<MODE>(xb, out, sbyte, idx);
    e_lds[2 * rp + 1][col] = u32x4{out[0], out[1], out[2], out[3]};
    s_lds[2 * rp + 1][col] = (uint8_t)sbyte;
    if (PLUS) i_lds[2 * rp + 1][col] = (uint8_t)idx;
    col0 += B;
    if (col0 < (uint32_t)C && more) {                                // uniform: the tile takes another pass
      unpack(raw);
      continue;
    }
    // ---- the tile is full (or the run ends): blocks kbf0 .. kbf0 + valid of rows row0 .. row0 + R leave
    const int64_t kbf0 = kb0 + B - col0;
    const uint32_t valid = (uint32_t)(kb_end - kbf0 < (int64_t)col0 ? kb_end - kbf0 : (int64_t)col0);
    __syncthreads();
    for (uint32_t m = t; m < (uint32_t)(R * C); m += 256u) {
      const uint32_t lr = m / C, piece = m % C;
      const int64_t gr = row0 + lr;
      if (gr < rows && piece < valid)
        __builtin_nontemporal_store(e_lds[lr][piece], reinterpret_cast<u32x4*>(elems) + gr * nbk + kbf0 + piece);
    }
    constexpr uint32_t kWords = C / 4;                               // 4-byte words of scale (index) bytes per row
    for (uint32_t m = t; m < (PLUS ? 2u : 1u) * R * kWords; m += 256u) {
      const bool is_scale = m < (uint32_t)R * kWords;
      const uint32_t mm = is_scale ? m : m - R * kWords;
      const uint32_t lr = mm / kWords, word = mm % kWords;
      const int64_t gr = row0 + lr;
      const uint8_t* from = (is_scale ? s_lds[lr] : i_lds[lr]) + 4 * word;
      uint8_t* to = (is_scale ? scales : bm_idx) + gr * nbk + kbf0 + 4 * word;
      if (gr < rows && 4 * word < valid) {
        if (wide_meta) {                                             // then valid is a multiple of 4 as well
          *reinterpret_cast<uint32_t*>(to) = *reinterpret_cast<const uint32_t*>(from);
        } else {
          for (uint32_t j = 0; j < 4 && 4 * word + j < valid; ++j) to[j] = from[j];
        }
      }
    }
    __syncthreads();
    col0 = 0;
    if (more) unpack(raw);
  }
}

// ---- quantize straight into the MFMA-ready image (optionally also the canonical arrays) -------------------------
// The GEMM consumes E2M3 tiles, so for an operand that is only multiplied (activations, Sec. 7.2) the canonical
// bytes need not make a round trip through HBM.  A workgroup takes 32 rows x 4 k-tiles (8 blocks per row): in each of
// its 4 passes a wavefront reads two 512-byte row segments, encodes them exactly as quantize_kernel does, widens the
// eight 4-bit codes of a lane to 48 bits of E2M3 (code << 2; the BM becomes sign | 11 | mmm, Sec. 4.2), and drops
// them at the block's slot of its tile in LDS.  The four finished tiles are contiguous in the image (6 KiB) and leave
// with full-width stores.  Padding rows / blocks are zero elements with a unit scale, as the prepack kernel writes.
// `wg`: the workgroup's number in the patch walk; `tiles` (4 * kTileBytes, 16-byte aligned) and `tile_scales` (256 bytes): its
// LDS staging.
template <bool BF16, bool PLUS>
__device__ __forceinline__ void quantize_image_body(uint32_t wg, uint8_t* tiles, uint8_t* tile_scales, const void* __restrict__ src,
                                                    int64_t rows, int64_t nbk, int64_t ld, int64_t k_tiles,
                                                    uint32_t* __restrict__ elems, uint8_t* __restrict__ scales,
                                                    uint8_t* __restrict__ bm_idx, uint8_t* __restrict__ img_elems,
                                                    uint8_t* __restrict__ img_scales, int skip_padding_tiles) {
  const uint32_t t = threadIdx.x, part = t & 3u, quad_in_row = (t & 15u) >> 2;
  const PatchMap pm = patch_of_workgroup(wg, (uint32_t)((k_tiles + 3) / 4), (uint32_t)(((rows + kRowPad - 1) / kRowPad) * 2));
  if (!pm.valid) return;
  const int64_t rt = pm.rt, kt0 = pm.kg * 4;
  const bool canon = elems != nullptr;
  // pass u covers rows 8u .. 8u+7 of the row tile; this lane: row 8u + r0, K-block kb_in (the same in every pass)
  const uint32_t r0 = t >> 5, kb_in = (t >> 2) & 7u;
  const int64_t row0 = rt * kTileRows + r0, kb = kt0 * 2 + kb_in;
  const bool whole = rt * kTileRows + kTileRows <= rows && kt0 * 2 + 8 <= nbk;   // uniform: no lane of the workgroup is padding
  if (rt * kTileRows >= rows) {
    // a row tile of pure padding (rows are padded to 256): zero elements, unit scales, nothing to encode; left
    // unwritten when the only reader is the few-row product, which touches the tiles that hold rows only
    if (skip_padding_tiles) return;
    const int64_t nt0 = k_tiles - kt0 < 4 ? k_tiles - kt0 : 4;
    uint8_t* out0 = img_elems + (rt * k_tiles + kt0) * (int64_t)kTileBytes;
    const u32x4 z = {0, 0, 0, 0};
    for (uint32_t o = t * 16u; o < (uint32_t)nt0 * kTileBytes; o += 256u * 16u) MXP_IMAGE_STORE(z, reinterpret_cast<u32x4*>(out0 + o));
    if ((int64_t)(t >> 6) < nt0) img_scales[(((rt >> 2) * k_tiles + kt0 + (t >> 6)) * 64 + (t & 63u)) * 4 + (rt & 3)] = 127;
    return;
  }
  const bool kb_ok = kb < nbk;
  const int64_t off0 = row0 * ld + kb * 32 + part * 8, off_step = 8 * ld;         // source element offsets
  uint32_t w[4][8];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    if (whole || (kb_ok && row0 + 8 * u < rows)) {
      const int64_t off = off0 + u * off_step;
      if (BF16) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(src) + off));
        w[u][0] = v.x; w[u][1] = v.y; w[u][2] = v.z; w[u][3] = v.w;
        w[u][4] = w[u][5] = w[u][6] = w[u][7] = 0;
      } else {
        const u32x4* p = reinterpret_cast<const u32x4*>(static_cast<const float*>(src) + off);
        const u32x4 v0 = __builtin_nontemporal_load(p), v1 = __builtin_nontemporal_load(p + 1);
        w[u][0] = v0.x; w[u][1] = v0.y; w[u][2] = v0.z; w[u][3] = v0.w;
        w[u][4] = v1.x; w[u][5] = v1.y; w[u][6] = v1.z; w[u][7] = v1.w;
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) w[u][i] = 0;
    }
  }
  // LDS destinations.  Bytes [6 part, 6 part + 6) of the block's 24: the first 16 bytes of a block sit in the low run
  // of its tile (16 B per slot), the last 8 in the high run (8 B per slot); slot = 32 (K-block % 2) + row.
  const uint32_t slot0 = (kb_in & 1u) * 32u + r0;
  const uint32_t lo0 = (kb_in >> 1) * kTileBytes + slot0 * 16u, hi0 = (kb_in >> 1) * kTileBytes + 1024u + slot0 * 8u;
  const uint32_t a32 = part == 0 ? lo0 : part == 1 ? lo0 + 8u : part == 2 ? lo0 + 12u : hi0 + 4u;
  const uint32_t a16 = part == 0 ? lo0 + 4u : part == 1 ? lo0 + 6u : part == 2 ? hi0 : hi0 + 2u;
  const uint32_t s32 = part == 3 ? 64u : 128u, s16 = part >= 2 ? 64u : 128u;      // 8 slots further per pass
  const bool odd = (part & 1u) != 0;
  const int64_t g0 = row0 * nbk + kb, g_step = 8 * nbk;
  const bool dword_meta = (nbk & 3) == 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const bool valid = whole || (kb_ok && row0 + 8 * u < rows);
    uint32_t sbyte, idx;
    const uint32_t packed = encode_group<BF16, PLUS>(w[u], (int)part, sbyte, idx);
    if (canon) {
      const int64_t g = g0 + u * g_step;
      if (valid) __builtin_nontemporal_store(packed, elems + g * 4 + part);
      if (dword_meta) {
        // the four blocks of a 16-lane row are consecutive blocks of one matrix row: one dword of scales, one of indices
        uint32_t sv = (part == 0) ? (sbyte << (8 * quad_in_row)) : 0u;
        sv |= dpp_mov<kRowShr8>(sv);
        sv |= dpp_mov<kRowShr4>(sv);
        uint32_t iv = 0;
        if (PLUS) {
          iv = (part == 0) ? (idx << (8 * quad_in_row)) : 0u;
          iv |= dpp_mov<kRowShr8>(iv);
          iv |= dpp_mov<kRowShr4>(iv);
        }
        if (valid && (t & 15u) == 12u) {
          *reinterpret_cast<uint32_t*>(scales + g - 3) = sv;
          if (PLUS) *reinterpret_cast<uint32_t*>(bm_idx + g - 3) = iv;
        }
      } else if (valid && part == 0) {
        scales[g] = (uint8_t)sbyte;
        if (PLUS) bm_idx[g] = (uint8_t)idx;
      }
    }
    // 48 bits of E2M3 codes for this lane's eight elements
    uint32_t c0 = widen4(packed & 0xFFFFu), c1 = widen4(packed >> 16);           // 24 bits each
    if (PLUS) {
      const uint32_t pos = idx & 7u;
      const uint32_t nib = (packed >> (4u * pos)) & 15u;
      const uint32_t code = ((nib & 8u) << 2) | 0x18u | (nib & 7u);
      const bool mine = sbyte != 0u && sbyte != 255u && (idx >> 3) == part;
      const uint32_t sh = 6u * (pos & 3u);
      const uint32_t patched0 = (c0 & ~(0x3Fu << sh)) | (code << sh), patched1 = (c1 & ~(0x3Fu << sh)) | (code << sh);
      c0 = (mine && pos < 4u) ? patched0 : c0;
      c1 = (mine && pos >= 4u) ? patched1 : c1;
    }
    const uint32_t low32 = c0 | (c1 << 24), high16 = c1 >> 8;                     // bits [0,32) and [32,48)
    const uint32_t v32 = odd ? (low32 >> 16) | (high16 << 16) : low32;
    const uint32_t v16 = odd ? low32 & 0xFFFFu : high16;
    *reinterpret_cast<uint32_t*>(tiles + a32 + u * s32) = v32;
    *reinterpret_cast<uint16_t*>(tiles + a16 + u * s16) = (uint16_t)v16;
    if (part == 0) tile_scales[(kb_in >> 1) * 64u + slot0 + 8u * u] = valid ? (uint8_t)sbyte : (uint8_t)127;
  }
  __syncthreads();
  const int64_t nt = k_tiles - kt0 < 4 ? k_tiles - kt0 : 4;          // tiles of this workgroup that exist
  uint8_t* out = img_elems + (rt * k_tiles + kt0) * (int64_t)kTileBytes;
  const uint32_t nbytes = (uint32_t)nt * kTileBytes;
  for (uint32_t o = t * 16u; o < nbytes; o += 256u * 16u)
    MXP_IMAGE_STORE(*reinterpret_cast<const u32x4*>(tiles + o), reinterpret_cast<u32x4*>(out + o));
  if ((int64_t)(t >> 6) < nt) img_scales[(((rt >> 2) * k_tiles + kt0 + (t >> 6)) * 64 + (t & 63u)) * 4 + (rt & 3)] = tile_scales[t];
}

template <bool BF16, bool PLUS>
__global__ void __launch_bounds__(256) quantize_image_kernel(const void* __restrict__ src, int64_t rows, int64_t nbk, int64_t ld,
                                                             int64_t k_tiles, uint32_t* __restrict__ elems,
                                                             uint8_t* __restrict__ scales, uint8_t* __restrict__ bm_idx,
                                                             uint8_t* __restrict__ img_elems, uint8_t* __restrict__ img_scales,
                                                             int skip_padding_tiles) {
  __shared__ __attribute__((aligned(16))) uint8_t tiles[4 * kTileBytes];
  __shared__ uint8_t tile_scales[4 * 64];
  quantize_image_body<BF16, PLUS>(blockIdx.x, tiles, tile_scales, src, rows, nbk, ld, k_tiles, elems, scales, bm_idx, img_elems,
                                  img_scales, skip_padding_tiles);
}

// Both conversions of a product with un-quantized activations and canonical weights in ONE launch: the first n_a
// workgroups walk the activation patches (source -> canonical arrays + E2M3 image), the rest the weight patches
// (canonical -> E2M3 image).  The two jobs are independent; as separate launches each pays its own ramp-up and tail
// (10-25 us kernels), as one grid the weight patches fill the compute units the activation job's tail leaves idle.
struct ConvertPairArgs {
  const void* src; int64_t rows_a, nbk, ld, k_tiles;
  uint32_t* a_elems; uint8_t *a_scales, *a_idx, *a_img_elems, *a_img_scales;
  const img_u32x4* w_elems; const uint8_t *w_scales, *w_idx; int64_t rows_w;
  uint8_t *w_img_elems, *w_img_scales;
  uint32_t n_a;
};
template <bool BF16, bool PLUS_A, bool PLUS_W>
__global__ void __launch_bounds__(256) convert_pair_kernel(const ConvertPairArgs p) {
  __shared__ __attribute__((aligned(16))) uint8_t tiles[4 * kTileBytes];
  __shared__ uint8_t tile_scales[4 * 64];
  const bool is_a = blockIdx.x < p.n_a;
  const uint32_t wg = is_a ? blockIdx.x : blockIdx.x - p.n_a;
  if (is_a)
    quantize_image_body<BF16, PLUS_A>(wg, tiles, tile_scales, p.src, p.rows_a, p.nbk, p.ld, p.k_tiles, p.a_elems, p.a_scales,
                                      p.a_idx, p.a_img_elems, p.a_img_scales, 0);
  else
    prepack_body<PLUS_W>(wg, tiles, tile_scales, p.w_elems, p.w_scales, p.w_idx, p.rows_w, p.nbk, p.k_tiles,
                         p.w_img_elems, p.w_img_scales);
}

// The same one-pass conversion for MXFP4++ (Sec. 4.3), whose GEMM operand is an E4M3 image: with the image's scale
// byte set to scale byte - delta + 2 an ordinary element (E2M1 value v) becomes v / 4 and the BM 1.mmm * 2^delta, both
// FP8 E4M3 numbers.  A lane's eight codes are eight bytes; the FP8 operand registers of a lane hold k = 16 (lane / 32)
// + 0..15 in their first half and the same + 32 in the second, so block (kb % 2) of a tile fills register half
// (kb % 2) of the two lanes of its row: codes 0..15 in lane r, 16..31 in lane r + 32.
template <bool BF16>
__global__ void __launch_bounds__(256) quantize_image_e4m3_kernel(const void* __restrict__ src, int64_t rows, int64_t nbk, int64_t ld,
                                                                  int64_t k_tiles, uint32_t* __restrict__ elems,
                                                                  uint8_t* __restrict__ scales, uint8_t* __restrict__ bm_idx,
                                                                  uint8_t* __restrict__ img_elems, uint8_t* __restrict__ img_scales,
                                                                  int skip_padding_tiles) {
  __shared__ __attribute__((aligned(16))) uint8_t tiles[4 * kTileBytesE4M3];
  __shared__ uint8_t tile_scales[4 * 64];
  const uint32_t t = threadIdx.x, part = t & 3u;
  const PatchMap pm = patch_of_workgroup(blockIdx.x, (uint32_t)((k_tiles + 3) / 4), (uint32_t)(((rows + kRowPad - 1) / kRowPad) * 2));
  if (!pm.valid) return;
  const int64_t rt = pm.rt, kt0 = pm.kg * 4;
  if (skip_padding_tiles && rt * kTileRows >= rows) return;   // (see quantize_image_kernel)
  const bool canon = elems != nullptr;
  const uint32_t r0 = t >> 5, kb_in = (t >> 2) & 7u;
  const int64_t row0 = rt * kTileRows + r0, kb = kt0 * 2 + kb_in;
  const bool kb_ok = kb < nbk;
  const int64_t off0 = row0 * ld + kb * 32 + part * 8, off_step = 8 * ld;
  uint32_t w[4][8];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
#pragma unroll
    for (int i = 0; i < 8; ++i) w[u][i] = 0;
    if (kb_ok && row0 + 8 * u < rows) {
      const int64_t off = off0 + u * off_step;
      if (BF16) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(src) + off));
        w[u][0] = v.x; w[u][1] = v.y; w[u][2] = v.z; w[u][3] = v.w;
      } else {
        const u32x4* p = reinterpret_cast<const u32x4*>(static_cast<const float*>(src) + off);
        const u32x4 v0 = __builtin_nontemporal_load(p), v1 = __builtin_nontemporal_load(p + 1);
        w[u][0] = v0.x; w[u][1] = v0.y; w[u][2] = v0.z; w[u][3] = v0.w;
        w[u][4] = v1.x; w[u][5] = v1.y; w[u][6] = v1.z; w[u][7] = v1.w;
      }
    }
  }
  const int64_t g0 = row0 * nbk + kb, g_step = 8 * nbk;
  // LDS destination of this lane's 8 bytes in pass u: tile kb_in / 2, register half kb_in % 2, lane (part / 2) * 32 + row
  const uint32_t dst0 = (kb_in >> 1) * kTileBytesE4M3 + (kb_in & 1u) * 1024u + ((part >> 1) * 32u + r0) * 16u + (part & 1u) * 8u;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const bool valid = kb_ok && row0 + 8 * u < rows;
    uint32_t sbyte, idx;
    const uint32_t packed = encode_group<BF16, 2>(w[u], (int)part, sbyte, idx);
    if (canon && valid) {
      const int64_t g = g0 + u * g_step;
      __builtin_nontemporal_store(packed, elems + g * 4 + part);
      if (part == 0) {
        scales[g] = (uint8_t)sbyte;
        bm_idx[g] = (uint8_t)idx;
      }
    }
    uint32_t c0 = nibbles4_to_e4m3(packed & 0xFFFFu), c1 = nibbles4_to_e4m3(packed >> 16);
    if (sbyte == 0u) c0 = c1 = 0u;                                               // flushed block: plain zeros
    const uint32_t delta = idx >> 5, pos = idx & 31u;
    const bool live = sbyte != 0u && sbyte != 255u;
    if (live && (pos >> 3) == part) {
      const uint32_t pi = pos & 7u, nib = (packed >> (4u * pi)) & 15u;
      const uint32_t code = ((nib & 8u) << 4) | ((delta + 7u) << 3) | (nib & 7u);
      const uint32_t sh = (pi & 3u) * 8u;
      if (pi < 4u) c0 = (c0 & ~(0xFFu << sh)) | (code << sh);
      else c1 = (c1 & ~(0xFFu << sh)) | (code << sh);
    }
    *reinterpret_cast<u32x2*>(tiles + dst0 + u * 128u) = u32x2{c0, c1};          // 8 rows further per pass
    if (part == 0) {
      const uint32_t sb = !valid ? 127u : (sbyte == 255u ? 255u : (sbyte == 0u ? 127u : sbyte - delta + 2u));
      tile_scales[(kb_in >> 1) * 64u + (kb_in & 1u) * 32u + r0 + 8u * u] = (uint8_t)sb;
    }
  }
  __syncthreads();
  const int64_t nt = k_tiles - kt0 < 4 ? k_tiles - kt0 : 4;
  uint8_t* out = img_elems + (rt * k_tiles + kt0) * (int64_t)kTileBytesE4M3;
  const uint32_t nbytes = (uint32_t)nt * kTileBytesE4M3;
  for (uint32_t o = t * 16u; o < nbytes; o += 256u * 16u)
    MXP_IMAGE_STORE(*reinterpret_cast<const u32x4*>(tiles + o), reinterpret_cast<u32x4*>(out + o));
  if ((int64_t)(t >> 6) < nt) img_scales[(((rt >> 2) * k_tiles + kt0 + (t >> 6)) * 64 + (t & 63u)) * 4 + (rt & 3)] = tile_scales[t];
}

int check_common(const void* src, int src_dtype, int64_t rows, int64_t K, int fmt, const uint8_t* elems,
                 const uint8_t* scales, const uint8_t* bm_idx) {
  if (fmt != MXP_FMT_MXFP4 && fmt != MXP_FMT_MXFP4P && fmt != MXP_FMT_MXFP4PP) return MXP_ERR_FORMAT;
  if (src_dtype != MXP_F32 && src_dtype != MXP_BF16) return MXP_ERR_DTYPE;
  if (rows < 0 || K < 0 || K % kBlock != 0) return MXP_ERR_SHAPE;
  if (rows == 0 || K == 0) return MXP_OK;
  if (!src || !elems || !scales || (fmt != MXP_FMT_MXFP4 && !bm_idx)) return MXP_ERR_NULL;
  if (!aligned16(src) || !aligned16(elems) || !aligned16(scales) || (bm_idx && !aligned16(bm_idx))) return MXP_ERR_ALIGN;
  return MXP_OK;
}

}  // namespace

namespace mxp {

template <bool BF16, int MODE, int U>
static void quantize_dispatch_mode(const void* src, int64_t nbk, int64_t ld_src, int dense, int64_t nq, int grid, uint32_t* e32,
                                   uint8_t* scales, uint8_t* bm_idx, hipStream_t stream) {
  if (dense) hipLaunchKernelGGL((quantize_dense_kernel<BF16, MODE, U>), dim3(grid), dim3(256), 0, stream, src, nq, e32, scales, bm_idx);
  else hipLaunchKernelGGL((quantize_kernel<BF16, MODE, U>), dim3(grid), dim3(256), 0, stream, src, nbk, ld_src, dense, nq, e32, scales, bm_idx);
}

template <int U>
static void quantize_dispatch(const void* src, int src_dtype, int64_t nbk, int64_t ld_src, int dense, int64_t nq, int fmt,
                              int64_t cap, uint8_t* elems, uint8_t* scales, uint8_t* bm_idx, hipStream_t stream) {
  const int64_t want = (nq + 256 * U - 1) / (256 * U);
  const int grid = (int)(want < cap ? want : cap);
  uint32_t* e32 = reinterpret_cast<uint32_t*>(elems);
  const bool bf = src_dtype == MXP_BF16;
  if (fmt == MXP_FMT_MXFP4PP) {
    if (bf) quantize_dispatch_mode<true, 2, U>(src, nbk, ld_src, dense, nq, grid, e32, scales, bm_idx, stream);
    else quantize_dispatch_mode<false, 2, U>(src, nbk, ld_src, dense, nq, grid, e32, scales, bm_idx, stream);
  } else if (fmt == MXP_FMT_MXFP4P) {
    if (bf) quantize_dispatch_mode<true, 1, U>(src, nbk, ld_src, dense, nq, grid, e32, scales, bm_idx, stream);
    else quantize_dispatch_mode<false, 1, U>(src, nbk, ld_src, dense, nq, grid, e32, scales, bm_idx, stream);
  } else {
    if (bf) quantize_dispatch_mode<true, 0, U>(src, nbk, ld_src, dense, nq, grid, e32, scales, bm_idx, stream);
    else quantize_dispatch_mode<false, 0, U>(src, nbk, ld_src, dense, nq, grid, e32, scales, bm_idx, stream);
  }
}

// Launch shape from a sweep over loads per lane (2, 4, 8) and resident workgroups per CU (4 .. 32): 4 independent
// 16-byte loads per lane on up to 32 workgroups per CU is the best or within 1 % of it for every size tried
// (bf16: 6.0-6.2 TB/s on 128-235 MB tensors, 10 us for 32 MiB; fp32: 5.4 TB/s).
int quantize_launch(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t ld_src, int fmt, uint8_t* elems,
                    uint8_t* scales, uint8_t* bm_idx, hipStream_t stream) {
  const int64_t nbk = K / kBlock;
  const int64_t nq = rows * nbk * 4;
  const int dense = (ld_src == K) ? 1 : 0;
  quantize_dispatch<4>(src, src_dtype, nbk, ld_src, dense, nq, fmt, (int64_t)kNumCU * 32, elems, scales, bm_idx, stream);
  return launch_status();
}

// Also used by the GEMM entry point that takes unquantized activations.  Canonical pointers may all be null.
int quantize_image_launch(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t ld_src, int fmt, uint8_t* elems,
                          uint8_t* scales, uint8_t* bm_idx, void* image, hipStream_t stream, bool skip_padding_tiles) {
  const int skip = skip_padding_tiles ? 1 : 0;
  const bool pp = fmt == MXP_FMT_MXFP4PP;
  const ImageGeom g = image_geom(rows, K, pp ? kTileBytesE4M3 : kTileBytes);
  const int64_t n_wg = patch_grid((g.k_tiles + 3) / 4, g.row_tiles / 4);
  if (n_wg > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  uint8_t* ie = static_cast<uint8_t*>(image);
  uint8_t* is = ie + g.elem_bytes;
  dim3 grid((unsigned)n_wg);
  uint32_t* e32 = reinterpret_cast<uint32_t*>(elems);
  const int64_t nbk = K / kBlock;
  const bool bf = src_dtype == MXP_BF16, plus = fmt == MXP_FMT_MXFP4P;
  if (pp) {
    if (bf) hipLaunchKernelGGL((quantize_image_e4m3_kernel<true>), grid, dim3(256), 0, stream, src, rows, nbk, ld_src, g.k_tiles, e32, scales, bm_idx, ie, is, skip);
    else hipLaunchKernelGGL((quantize_image_e4m3_kernel<false>), grid, dim3(256), 0, stream, src, rows, nbk, ld_src, g.k_tiles, e32, scales, bm_idx, ie, is, skip);
    return launch_status();
  }
  if (bf && plus) hipLaunchKernelGGL((quantize_image_kernel<true, true>), grid, dim3(256), 0, stream, src, rows, nbk, ld_src, g.k_tiles, e32, scales, bm_idx, ie, is, skip);
  else if (bf) hipLaunchKernelGGL((quantize_image_kernel<true, false>), grid, dim3(256), 0, stream, src, rows, nbk, ld_src, g.k_tiles, e32, scales, bm_idx, ie, is, skip);
  else if (plus) hipLaunchKernelGGL((quantize_image_kernel<false, true>), grid, dim3(256), 0, stream, src, rows, nbk, ld_src, g.k_tiles, e32, scales, bm_idx, ie, is, skip);
  else hipLaunchKernelGGL((quantize_image_kernel<false, false>), grid, dim3(256), 0, stream, src, rows, nbk, ld_src, g.k_tiles, e32, scales, bm_idx, ie, is, skip);
  return launch_status();
}

}  // namespace mxp

extern "C" int mxp_quantize_image(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t ld_src, int fmt,
                                  uint8_t* elems, uint8_t* scales, uint8_t* bm_idx, void* image, size_t image_bytes,
                                  void* stream) {
  using namespace mxp;
  if (fmt != MXP_FMT_MXFP4 && fmt != MXP_FMT_MXFP4P && fmt != MXP_FMT_MXFP4PP) return MXP_ERR_FORMAT;
  if (src_dtype != MXP_F32 && src_dtype != MXP_BF16) return MXP_ERR_DTYPE;
  if (rows < 0 || K < 0 || K % kBlock != 0) return MXP_ERR_SHAPE;
  if (rows == 0 || K == 0) return MXP_OK;
  if (!src || !image) return MXP_ERR_NULL;
  const bool canon = elems || scales || bm_idx;
  if (canon && (!elems || !scales || (fmt != MXP_FMT_MXFP4 && !bm_idx))) return MXP_ERR_NULL;
  if (ld_src < K) return MXP_ERR_SHAPE;
  const int64_t esz = src_dtype == MXP_BF16 ? 2 : 4;
  if (!aligned16(src) || !aligned16(image) || (ld_src * esz) % 16 != 0) return MXP_ERR_ALIGN;
  if (canon && (!aligned16(elems) || !aligned16(scales) || (bm_idx && !aligned16(bm_idx)))) return MXP_ERR_ALIGN;
  if (image_bytes < (size_t)image_geom(rows, K, fmt == MXP_FMT_MXFP4PP ? kTileBytesE4M3 : kTileBytes).total()) return MXP_ERR_WORKSPACE;
  return quantize_image_launch(src, src_dtype, rows, K, ld_src, fmt, canon ? elems : nullptr, scales, bm_idx, image,
                               static_cast<hipStream_t>(stream), false);
}

extern "C" int mxp_convert_operands(const void* A, int a_dtype, int64_t M, int64_t K, int64_t lda, int fmtA, uint8_t* A_elems,
                                    uint8_t* A_scales, uint8_t* A_idx, void* A_image, size_t a_image_bytes,
                                    const uint8_t* W_elems, const uint8_t* W_scales, const uint8_t* W_idx, int fmtW, int64_t N,
                                    void* W_image, size_t w_image_bytes, void* stream) {
  using namespace mxp;
  if (fmtA == MXP_FMT_MXFP4PP || fmtW == MXP_FMT_MXFP4PP) return MXP_ERR_UNSUPPORTED;
  if ((fmtA != MXP_FMT_MXFP4 && fmtA != MXP_FMT_MXFP4P) || (fmtW != MXP_FMT_MXFP4 && fmtW != MXP_FMT_MXFP4P)) return MXP_ERR_FORMAT;
  if (a_dtype != MXP_F32 && a_dtype != MXP_BF16) return MXP_ERR_DTYPE;
  if (M < 0 || N < 0 || K < 0 || K % kBlock != 0) return MXP_ERR_SHAPE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // an empty side: the other one alone
  if (K == 0 || (M == 0 && N == 0)) return MXP_OK;
  if (M == 0) return mxp_prepack(W_elems, W_scales, W_idx, fmtW, N, K, W_image, w_image_bytes, stream);
  if (N == 0) return mxp_quantize_image(A, a_dtype, M, K, lda, fmtA, A_elems, A_scales, A_idx, A_image, a_image_bytes, stream);
  if (!A || !A_image || !W_elems || !W_scales || !W_image || (fmtW == MXP_FMT_MXFP4P && !W_idx)) return MXP_ERR_NULL;
  const bool canon = A_elems || A_scales || A_idx;
  if (canon && (!A_elems || !A_scales || (fmtA != MXP_FMT_MXFP4 && !A_idx))) return MXP_ERR_NULL;
  if (lda < K) return MXP_ERR_SHAPE;
  const int64_t esz = a_dtype == MXP_BF16 ? 2 : 4;
  if (!aligned16(A) || !aligned16(A_image) || (lda * esz) % 16 != 0 || !aligned16(W_elems) || !aligned16(W_scales) ||
      !aligned16(W_image) || (W_idx && !aligned16(W_idx)))
    return MXP_ERR_ALIGN;
  if (canon && (!aligned16(A_elems) || !aligned16(A_scales) || (A_idx && !aligned16(A_idx)))) return MXP_ERR_ALIGN;
  const ImageGeom ga = image_geom(M, K), gw = image_geom(N, K);
  if (a_image_bytes < (size_t)ga.total() || w_image_bytes < (size_t)gw.total()) return MXP_ERR_WORKSPACE;
  const int64_t n_a = patch_grid((ga.k_tiles + 3) / 4, ga.row_tiles / 4), n_w = patch_grid((gw.k_tiles + 3) / 4, gw.row_tiles / 4);
  if (n_a + n_w > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  ConvertPairArgs p;
  p.src = A; p.rows_a = M; p.nbk = K / kBlock; p.ld = lda; p.k_tiles = ga.k_tiles;
  p.a_elems = canon ? reinterpret_cast<uint32_t*>(A_elems) : nullptr; p.a_scales = A_scales; p.a_idx = A_idx;
  p.a_img_elems = static_cast<uint8_t*>(A_image); p.a_img_scales = p.a_img_elems + ga.elem_bytes;
  p.w_elems = reinterpret_cast<const img_u32x4*>(W_elems); p.w_scales = W_scales; p.w_idx = W_idx; p.rows_w = N;
  p.w_img_elems = static_cast<uint8_t*>(W_image); p.w_img_scales = p.w_img_elems + gw.elem_bytes;
  p.n_a = (uint32_t)n_a;
  const dim3 grid((unsigned)(n_a + n_w)), block(256);
  const bool bf = a_dtype == MXP_BF16, pa = fmtA == MXP_FMT_MXFP4P, pw = fmtW == MXP_FMT_MXFP4P;
#define MXP_PAIR(B, PA, PW) hipLaunchKernelGGL((convert_pair_kernel<B, PA, PW>), grid, block, 0, s, p)
  if (bf) { if (pa) { if (pw) MXP_PAIR(true, true, true); else MXP_PAIR(true, true, false); } else { if (pw) MXP_PAIR(true, false, true); else MXP_PAIR(true, false, false); } }
  else    { if (pa) { if (pw) MXP_PAIR(false, true, true); else MXP_PAIR(false, true, false); } else { if (pw) MXP_PAIR(false, false, true); else MXP_PAIR(false, false, false); } }
#undef MXP_PAIR
  return launch_status();
}

extern "C" int mxp_quantize(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t ld_src, int fmt,
                            uint8_t* elems, uint8_t* scales, uint8_t* bm_idx, void* stream) {
  using namespace mxp;
  const bool wide = is_wide_format(fmt);
  // the six- and eight-bit formats share every argument rule; their plain forms, like MXFP4, take no index array
  int rc = check_common(src, src_dtype, rows, K, wide ? (plain_wide_format(fmt) ? MXP_FMT_MXFP4 : MXP_FMT_MXFP4P) : fmt,
                        elems, scales, bm_idx);
  if (rc != MXP_OK || rows == 0 || K == 0) return rc;
  if (ld_src < K) return MXP_ERR_SHAPE;
  const int64_t esz = src_dtype == MXP_BF16 ? 2 : 4;
  if ((ld_src * esz) % 16 != 0) return MXP_ERR_ALIGN;
  if (wide) return wide_quantize_launch(src, src_dtype, rows, K, ld_src, fmt, elems, scales, bm_idx, static_cast<hipStream_t>(stream));
  return quantize_launch(src, src_dtype, rows, K, ld_src, fmt, elems, scales, bm_idx, static_cast<hipStream_t>(stream));
}

extern "C" int mxp_quantize_gather(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t n_src, int64_t ld_src,
                                   const int32_t* perm, int fmt, uint8_t* elems, uint8_t* scales, uint8_t* bm_idx, void* stream) {
  using namespace mxp;
  int rc = check_common(src, src_dtype, rows, K, fmt, elems, scales, bm_idx);
  if (rc != MXP_OK || rows == 0 || K == 0) return rc;
  if (!perm) return MXP_ERR_NULL;
  if (n_src <= 0 || ld_src < n_src) return MXP_ERR_SHAPE;
  if (!aligned16(perm)) return MXP_ERR_ALIGN;
  const int64_t nbk = K / kBlock, nq = rows * nbk * 4;
  const int64_t want = (nq + 255) / 256, cap = (int64_t)kNumCU * 32;
  const dim3 grid((unsigned)(want < cap ? want : cap));
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint32_t* e32 = reinterpret_cast<uint32_t*>(elems);
  const bool bf = src_dtype == MXP_BF16;
  // rows that fit in LDS (64 KiB) with at most 8 groups per lane (K <= 16384) go through the LDS kernel
  const int64_t row_bytes = n_src * (bf ? 2 : 4), gp = (nbk * 4 + 255) / 256;
  if (row_bytes <= 64 * 1024 && gp <= 8) {
    const size_t lds = (size_t)((row_bytes + 15) & ~(int64_t)15);
    const dim3 grid_r((unsigned)(rows < (int64_t)kNumCU * 4 ? rows : (int64_t)kNumCU * 4));
#define MXP_LAUNCH_GL3(B, MD, G) hipLaunchKernelGGL((quantize_gather_lds_kernel<B, MD, G>), grid_r, dim3(256), lds, s, src, rows, nbk, ld_src, perm, n_src, e32, scales, bm_idx)
#define MXP_LAUNCH_GL2(B, MD) do { if (gp <= 1) MXP_LAUNCH_GL3(B, MD, 1); else if (gp <= 2) MXP_LAUNCH_GL3(B, MD, 2); else if (gp <= 4) MXP_LAUNCH_GL3(B, MD, 4); else MXP_LAUNCH_GL3(B, MD, 8); } while (0)
    if (fmt == MXP_FMT_MXFP4PP) { if (bf) MXP_LAUNCH_GL2(true, 2); else MXP_LAUNCH_GL2(false, 2); }
    else if (fmt == MXP_FMT_MXFP4P) { if (bf) MXP_LAUNCH_GL2(true, 1); else MXP_LAUNCH_GL2(false, 1); }
    else { if (bf) MXP_LAUNCH_GL2(true, 0); else MXP_LAUNCH_GL2(false, 0); }
#undef MXP_LAUNCH_GL2
#undef MXP_LAUNCH_GL3
    return launch_status();
  }
#define MXP_LAUNCH_GATHER(B, MD) hipLaunchKernelGGL((quantize_gather_kernel<B, MD>), grid, dim3(256), 0, s, src, nbk, ld_src, perm, n_src, nq, e32, scales, bm_idx)
  if (fmt == MXP_FMT_MXFP4PP) { if (bf) MXP_LAUNCH_GATHER(true, 2); else MXP_LAUNCH_GATHER(false, 2); }
  else if (fmt == MXP_FMT_MXFP4P) { if (bf) MXP_LAUNCH_GATHER(true, 1); else MXP_LAUNCH_GATHER(false, 1); }
  else { if (bf) MXP_LAUNCH_GATHER(true, 0); else MXP_LAUNCH_GATHER(false, 0); }
#undef MXP_LAUNCH_GATHER
  return launch_status();
}

extern "C" int mxp_quantize_t(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t ld_src, int fmt,
                              uint8_t* elems, uint8_t* scales, uint8_t* bm_idx, void* stream) {
  using namespace mxp;
  int rc = check_common(src, src_dtype, rows, K, fmt, elems, scales, bm_idx);
  if (rc != MXP_OK || rows == 0 || K == 0) return rc;
  if (ld_src < rows) return MXP_ERR_SHAPE;
  const int64_t nbk = K / kBlock;
  if (nbk > 65535) return MXP_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint4* e = reinterpret_cast<uint4*>(elems);
  const bool bf = src_dtype == MXP_BF16;
  // the tiled kernel loads row pairs: every pair must start on a 4-byte (bf16) / 8-byte (fp32) boundary
  // and addresses a block's 32 source lines with 32-bit offsets
  const bool pairs_ok = (ld_src & 1) == 0 && (reinterpret_cast<uintptr_t>(src) & (bf ? 3u : 7u)) == 0 &&
                        ld_src * (bf ? 2 : 4) * 32 < (int64_t)0x7FFFFFFF;
  if (pairs_ok) {
    dim3 grid((unsigned)((rows + kTRows - 1) / kTRows), (unsigned)((nbk + kTRun - 1) / kTRun));
#define MXP_LAUNCH_QT(B, MD) hipLaunchKernelGGL((quantize_t_tiled_kernel<B, MD, kTAcc>), grid, dim3(256), 0, s, src, rows, nbk, ld_src, e, scales, bm_idx)
    if (fmt == MXP_FMT_MXFP4PP) { if (bf) MXP_LAUNCH_QT(true, 2); else MXP_LAUNCH_QT(false, 2); }
    else if (fmt == MXP_FMT_MXFP4P) { if (bf) MXP_LAUNCH_QT(true, 1); else MXP_LAUNCH_QT(false, 1); }
    else { if (bf) MXP_LAUNCH_QT(true, 0); else MXP_LAUNCH_QT(false, 0); }
#undef MXP_LAUNCH_QT
    return launch_status();
  }
  dim3 grid((unsigned)((rows + 255) / 256), (unsigned)nbk);
  if (fmt == MXP_FMT_MXFP4PP) {
    if (bf) hipLaunchKernelGGL((quantize_t_kernel<true, 2>), grid, dim3(256), 0, s, src, rows, nbk, ld_src, e, scales, bm_idx);
    else hipLaunchKernelGGL((quantize_t_kernel<false, 2>), grid, dim3(256), 0, s, src, rows, nbk, ld_src, e, scales, bm_idx);
  } else if (fmt == MXP_FMT_MXFP4P) {
    if (bf) hipLaunchKernelGGL((quantize_t_kernel<true, 1>), grid, dim3(256), 0, s, src, rows, nbk, ld_src, e, scales, bm_idx);
    else hipLaunchKernelGGL((quantize_t_kernel<false, 1>), grid, dim3(256), 0, s, src, rows, nbk, ld_src, e, scales, bm_idx);
  } else {
    if (bf) hipLaunchKernelGGL((quantize_t_kernel<true, 0>), grid, dim3(256), 0, s, src, rows, nbk, ld_src, e, scales, bm_idx);
    else hipLaunchKernelGGL((quantize_t_kernel<false, 0>), grid, dim3(256), 0, s, src, rows, nbk, ld_src, e, scales, bm_idx);
  }
  return launch_status();
}
