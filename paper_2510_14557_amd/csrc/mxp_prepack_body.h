// Device code shared by the kernels that write E2M3 images from canonical MXFP4 / MXFP4+ storage (Sec. 4.2: the BM is an
// E2M3 number at exponent e_max, every other element an E2M1 number and so an E2M3 number too).
#pragma once
#include "mxp_common.h"

namespace mxp {
typedef uint32_t img_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t img_u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t img_u32x6 __attribute__((ext_vector_type(6)));
typedef __bf16 img_v2bf __attribute__((ext_vector_type(2)));
typedef __bf16 img_v32bf __attribute__((ext_vector_type(32)));

// 4 nibbles (16 bit) -> 4 six-bit codes (24 bit), code = nibble << 2.  Two multiplies spread the even and the odd
// nibbles to their positions: bit offsets 4i -> 6i + 2.
__device__ __forceinline__ uint32_t widen4(uint32_t h) {
  const uint32_t x = h & 0x0F0Fu, y = h & 0xF0F0u;
  return ((x * 0x44u) & 0x0003C03Cu) | ((y * 0x110u) & 0x00F00F00u);
}

// One thread widens one 32-element block into its 24-byte E2M3 operand.  A 256-thread group covers 32 rows x 8
// consecutive K-blocks (4 k-tiles): thread t takes row t / 8, block t % 8, so the eight lanes of a row read 128
// contiguous bytes.  The finished blocks are dropped at their lane slots of the four tiles in LDS; the tiles are
// neighbours in the image (6 KiB), which then leaves the workgroup in full 16-byte-per-lane stores.
// `wg` is the workgroup's number in the patch walk; `tiles` (4 * kTileBytes, 16-byte aligned) and `tile_scales` (256 bytes)
// are the workgroup's LDS staging.
template <bool PLUS>
__device__ __forceinline__ void prepack_body(uint32_t wg, uint8_t* tiles, uint8_t* tile_scales, const img_u32x4* __restrict__ elems,
                                             const uint8_t* __restrict__ scales, const uint8_t* __restrict__ bm_idx, int64_t rows,
                                             int64_t nbk, int64_t k_tiles, uint8_t* __restrict__ img_elems,
                                             uint8_t* __restrict__ img_scales) {
  const uint32_t t = threadIdx.x;
  const uint32_t r_in = t >> 3, kb_in = t & 7u;
  const PatchMap pm = patch_of_workgroup(wg, (uint32_t)((k_tiles + 3) / 4), (uint32_t)(((rows + kRowPad - 1) / kRowPad) * 2));
  if (!pm.valid) return;
  const int64_t kt0 = pm.kg * 4;
  const int64_t rt = pm.rt;
  const uint32_t slot = (kb_in & 1u) * 32u + r_in;     // slot of this block in its tile: row % 32, K-block % 2
  const int64_t row = rt * kTileRows + r_in;
  const int64_t kb = kt0 * 2 + kb_in;
  uint32_t n[4] = {0, 0, 0, 0};
  uint32_t sbyte = 127u, bm = 64u;
  if (row < rows && kb < nbk) {
    const int64_t b = row * nbk + kb;
    const img_u32x4 v = __builtin_nontemporal_load(elems + b);
    n[0] = v.x; n[1] = v.y; n[2] = v.z; n[3] = v.w;
    sbyte = scales[b];
    if (PLUS && sbyte != 0u && sbyte != 255u) bm = bm_idx[b] & 31u;
    if (sbyte == 0u) n[0] = n[1] = n[2] = n[3] = 0u;          // flushed block: zero whatever the nibbles say
  }
  // E2M1 -> E2M3 by the conversion hardware: every E2M1 number is an E2M3 number (same exponent bias, mantissa m00), so
  // 16 two-element conversions to bf16 and one 32-element conversion to six-bit codes are exact and yield code = nibble << 2
  // at bit 6 i of the lane's 192-bit operand -- about a fifth of the vector instructions of spreading the nibbles by hand.
  union { uint32_t u[16]; img_v32bf v; } c;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    union { uint32_t u; img_v2bf v; } c0, c1, c2, c3;
    c0.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(n[j], 1.0f, 0);
    c1.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(n[j], 1.0f, 1);
    c2.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(n[j], 1.0f, 2);
    c3.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(n[j], 1.0f, 3);
    c.u[4 * j] = c0.u; c.u[4 * j + 1] = c1.u; c.u[4 * j + 2] = c2.u; c.u[4 * j + 3] = c3.u;
  }
  const img_u32x6 cv = __builtin_amdgcn_cvt_scalef32_pk32_fp6_bf16(c.v, 1.0f);
  uint32_t d[6] = {cv[0], cv[1], cv[2], cv[3], cv[4], cv[5]};
  if (PLUS) {
    // the BM's code is sign | 11 | mmm (E2M3 at exponent e_max, Sec. 4.2) instead of nibble << 2: the difference of the two
    // is XORed onto the six bits at 6 bm, which may straddle two dwords
    const uint32_t w = bm >> 3;
    const uint32_t nw = w == 0u ? n[0] : w == 1u ? n[1] : w == 2u ? n[2] : n[3];
    const uint32_t nib = (nw >> ((bm & 7u) * 4u)) & 15u;
    const uint32_t want = ((nib & 8u) << 2) | 0x18u | (nib & 7u);
    const uint32_t x6 = bm < 32u ? ((nib << 2) ^ want) : 0u;
    const uint32_t pos = bm * 6u, q = pos >> 5;
    const uint64_t x64 = (uint64_t)x6 << (pos & 31u);
    const uint32_t xlo = (uint32_t)x64, xhi = (uint32_t)(x64 >> 32);
#pragma unroll
    for (int j = 0; j < 6; ++j) d[j] ^= (q == (uint32_t)j ? xlo : 0u) ^ (j > 0 && q + 1u == (uint32_t)j ? xhi : 0u);
  }
  uint8_t* tile = tiles + (kb_in >> 1) * kTileBytes;
  img_u32x4 lo4 = {d[0], d[1], d[2], d[3]};
  img_u32x2 hi2 = {d[4], d[5]};
  *reinterpret_cast<img_u32x4*>(tile + slot * 16u) = lo4;
  *reinterpret_cast<img_u32x2*>(tile + 1024u + slot * 8u) = hi2;
  tile_scales[(kb_in >> 1) * 64u + slot] = (uint8_t)sbyte;
  __syncthreads();
  const int64_t nt = k_tiles - kt0 < 4 ? k_tiles - kt0 : 4;          // tiles of this workgroup that exist
  uint8_t* out = img_elems + (rt * k_tiles + kt0) * (int64_t)kTileBytes;
  const uint32_t nbytes = (uint32_t)nt * kTileBytes;
  for (uint32_t o = t * 16u; o < nbytes; o += 256u * 16u)
    MXP_IMAGE_STORE(*reinterpret_cast<const img_u32x4*>(tiles + o), reinterpret_cast<img_u32x4*>(out + o));
  if ((int64_t)(t >> 6) < nt) img_scales[(((rt >> 2) * k_tiles + kt0 + (t >> 6)) * 64 + (t & 63u)) * 4 + (rt & 3)] = tile_scales[t];
}

}  // namespace mxp
