// mxp_dequantize : canonical MXFP4 / MXFP4+ -> fp32 / bf16   (de-conversion, Eq. 2)
// mxp_prepack    : canonical -> MFMA-ready E2M3 image          (the "BM prepare" step of Sec. 5.2, done once per
//                  operand instead of once per MMA fragment: on CDNA4 the BM is directly an operand value)
#include "mxp_common.h"
#include "mxp_prepack_body.h"
#include "mxp_decode.h"

namespace {

using namespace mxp;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <bool OUT_BF16>
__device__ __forceinline__ void store_group(void* __restrict__ dst, int64_t off, const uint32_t (&out)[8]) {
  if (OUT_BF16) {
    u32x4 v = {out[0], out[1], out[2], out[3]};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(static_cast<uint16_t*>(dst) + off));
  } else {
    u32x4* p = reinterpret_cast<u32x4*>(static_cast<float*>(dst) + off);
    u32x4 v0 = {out[0], out[1], out[2], out[3]}, v1 = {out[4], out[5], out[6], out[7]};
    __builtin_nontemporal_store(v0, p);
    __builtin_nontemporal_store(v1, p + 1);
  }
}

// General destination (row stride ld): one group per lane and grid step.
template <int MODE, bool OUT_BF16>
__global__ void __launch_bounds__(256) dequantize_kernel(const uint32_t* __restrict__ elems, const uint8_t* __restrict__ scales,
                                                         const uint8_t* __restrict__ bm_idx, int64_t nbk, int64_t ld,
                                                         int64_t nq, void* __restrict__ dst) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < nq; q += stride) {
    const uint32_t dw = __builtin_nontemporal_load(elems + q);
    const int64_t g = q >> 2;
    const uint32_t part = (uint32_t)(q & 3);
    const uint32_t sbyte = scales[g];
    const uint32_t ib = MODE >= 1 ? (uint32_t)bm_idx[g] : 64u;
    uint32_t out[8];
    decode_group<(MODE >= 1), OUT_BF16>(dw, sbyte, MODE >= 1 ? ib & 31u : 64u, part, out, MODE == 2 ? ib >> 5 : 0u);
    const int64_t row = g / nbk;
    store_group<OUT_BF16>(dst, row * ld + (g - row * nbk) * 32 + part * 8, out);
  }
}

// Dense destination (row stride = K): the tensor is one run of nq groups.  A workgroup walks chunks of 256 * U groups;
// all loads of a chunk are issued before the first decode, and whole chunks run without bounds tests.
template <int MODE, bool OUT_BF16, int U>
__global__ void __launch_bounds__(256) dequantize_dense_kernel(const uint32_t* __restrict__ elems, const uint8_t* __restrict__ scales,
                                                               const uint8_t* __restrict__ bm_idx, int64_t nq,
                                                               void* __restrict__ dst) {
  const uint32_t t = threadIdx.x, part = t & 3u;
  constexpr int64_t kChunk = 256 * U;
  const int64_t n_chunks = (nq + kChunk - 1) / kChunk;
  for (int64_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    const int64_t q_base = c * kChunk;
    const bool whole = q_base + kChunk <= nq;
    const uint32_t* e_in = elems + q_base;
    const uint8_t* s_in = scales + (q_base >> 2);
    const uint8_t* i_in = bm_idx + (q_base >> 2);
    uint32_t dw[U], sb[U], bm[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t ql = u * 256 + t;
      dw[u] = 0; sb[u] = 0; bm[u] = 64u;
      if (whole || q_base + ql < nq) {
        dw[u] = __builtin_nontemporal_load(e_in + ql);
        sb[u] = s_in[ql >> 2];
        if (MODE >= 1) bm[u] = i_in[ql >> 2];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t ql = u * 256 + t;
      uint32_t out[8];
      decode_group<(MODE >= 1), OUT_BF16>(dw[u], sb[u], MODE >= 1 ? bm[u] & 31u : 64u, part, out, MODE == 2 ? bm[u] >> 5 : 0u);
      if (whole || q_base + ql < nq) store_group<OUT_BF16>(dst, (q_base + ql) * 8, out);
    }
  }
}

// Dense fp32 destination: a lane takes 4 elements (2 bytes of codes -> one 16-byte store), so that every store
// instruction of a wavefront writes 1 KiB contiguously; with 8 elements per lane its two 16-byte stores would each
// cover every other 16 bytes of the wavefront's 2 KiB.  The decode is the 8-element one applied to the lane's half.
template <int MODE, int U>
__global__ void __launch_bounds__(256) dequantize_dense_f32_kernel(const uint16_t* __restrict__ elems16, const uint8_t* __restrict__ scales,
                                                                   const uint8_t* __restrict__ bm_idx, int64_t nh,
                                                                   float* __restrict__ dst) {
  const uint32_t t = threadIdx.x, half = t & 1u, part = (t >> 1) & 3u;     // 8 lanes per block
  constexpr int64_t kChunk = 256 * U;
  const int64_t n_chunks = (nh + kChunk - 1) / kChunk;
  for (int64_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    const int64_t h_base = c * kChunk;
    const bool whole = h_base + kChunk <= nh;
    uint32_t dw[U], sb[U], bm[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t h = h_base + u * 256 + t;
      dw[u] = 0; sb[u] = 0; bm[u] = 64u;
      if (whole || h < nh) {
        dw[u] = (uint32_t)elems16[h] << (16u * half);
        sb[u] = scales[h >> 3];
        if (MODE >= 1) bm[u] = bm_idx[h >> 3];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t h = h_base + u * 256 + t;
      uint32_t out[8];
      decode_group<(MODE >= 1), false>(dw[u], sb[u], MODE >= 1 ? bm[u] & 31u : 64u, part, out, MODE == 2 ? bm[u] >> 5 : 0u);
      u32x4 v = {half ? out[4] : out[0], half ? out[5] : out[1], half ? out[6] : out[2], half ? out[7] : out[3]};
      if (whole || h < nh) __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dst + h * 4));
    }
  }
}

// canonical block -> 24-byte E2M3 operand, staged through LDS: see prepack_body
template <bool PLUS>
__global__ void __launch_bounds__(256) prepack_kernel(const u32x4* __restrict__ elems, const uint8_t* __restrict__ scales,
                                                      const uint8_t* __restrict__ bm_idx, int64_t rows, int64_t nbk,
                                                      int64_t k_tiles, uint8_t* __restrict__ img_elems,
                                                      uint8_t* __restrict__ img_scales) {
  __shared__ __attribute__((aligned(16))) uint8_t tiles[4 * kTileBytes];
  __shared__ uint8_t tile_scales[4 * 64];
  prepack_body<PLUS>(blockIdx.x, tiles, tile_scales, elems, scales, bm_idx, rows, nbk, k_tiles, img_elems, img_scales);
}

// ---- images of several K segments for four-bit operands (the exact MXFP4++ product, Sec. 4.3) ----------------------
// An MXFP4++ block has two scales: its BM is scaled by 2^shared_exp, every other element by 2^(shared_exp - delta).  One
// block-scaled MFMA operand carries one scale per block, so the operand is laid out as two K segments side by side --
// N: all elements but the BM (its place zero), scale byte lowered by delta; B: the BM alone as the E2M3 code
// sign | 11 | mmm (Sec. 4.2), the block's own scale byte -- and the other operand of the product, an MXFP4 / MXFP4+
// operand, as its whole image twice (role W).  [N | B] x [W | W]^T is then the exact product, formed by the same kernels
// over a K of two segments: every element is an E2M3 number under its segment's scale.  `roles` holds two bits per
// segment (0 W, 1 N, 2 B); each segment is K rounded up to 128 wide.  Patch walk and LDS staging as in prepack_body.
constexpr uint32_t kRoleWhole = 0, kRoleNbm = 1, kRoleBm = 2;

template <int MODE>   // 0 MXFP4, 1 MXFP4+, 2 MXFP4++
__global__ void __launch_bounds__(256) prepack_seg_kernel(const u32x4* __restrict__ elems, const uint8_t* __restrict__ scales,
                                                          const uint8_t* __restrict__ bm_idx, int64_t rows, int64_t nbk,
                                                          int64_t kts, int n_seg, uint32_t roles,
                                                          uint8_t* __restrict__ img_elems, uint8_t* __restrict__ img_scales) {
  __shared__ __attribute__((aligned(16))) uint8_t tiles[4 * kTileBytes];
  __shared__ uint8_t tile_scales[4 * 64];
  const uint32_t t = threadIdx.x;
  const uint32_t r_in = t >> 3, kb_in = t & 7u;
  const PatchMap pm = patch_of_workgroup(blockIdx.x, (uint32_t)((kts + 3) / 4), (uint32_t)(((rows + kRowPad - 1) / kRowPad) * 2));
  if (!pm.valid) return;
  const int64_t kt0 = pm.kg * 4, rt = pm.rt;
  const int64_t k_tiles = kts * n_seg;                         // k-tiles of the whole image
  const uint32_t slot = (kb_in & 1u) * 32u + r_in;
  const int64_t row = rt * kTileRows + r_in, kb = kt0 * 2 + kb_in;
  uint32_t n[4] = {0, 0, 0, 0};
  uint32_t sbyte = 127u, bm = 64u, delta = 0u;
  if (row < rows && kb < nbk) {
    const int64_t b = row * nbk + kb;
    const u32x4 v = __builtin_nontemporal_load(elems + b);
    n[0] = v.x; n[1] = v.y; n[2] = v.z; n[3] = v.w;
    sbyte = scales[b];
    if (MODE >= 1 && sbyte != 0u && sbyte != 255u) {
      const uint32_t ib = bm_idx[b];
      bm = ib & 31u;
      // (an MXFP4+ index byte has its upper bits reserved; a delta beyond scale byte - 1 is outside what a conversion writes)
      if (MODE == 2) delta = (ib >> 5) < sbyte ? (ib >> 5) : sbyte - 1u;
    }
    if (sbyte == 0u) n[0] = n[1] = n[2] = n[3] = 0u;          // flushed block: zero whatever the nibbles say
  }
  uint32_t r[8];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    r[2 * j] = widen4(n[j] & 0xFFFFu);
    r[2 * j + 1] = widen4(n[j] >> 16);
  }
  // the three forms of the block: whole (BM patched to sign | 11 | mmm), without the BM, the BM alone
  uint32_t whole[8], nbm[8], only[8];
  const uint32_t piece = bm >> 2, sh = (bm & 3u) * 6u;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint32_t c = (r[j] >> sh) & 0x3Fu;                   // s mmm 00
    const uint32_t code = (c & 0x20u) | 0x18u | ((c >> 2) & 7u);
    const bool here = bm < 32u && piece == (uint32_t)j;
    nbm[j] = here ? r[j] & ~(0x3Fu << sh) : r[j];
    only[j] = here ? code << sh : 0u;
    whole[j] = nbm[j] | only[j];
  }
  uint8_t* tile = tiles + (kb_in >> 1) * kTileBytes;
  const int64_t nt = kts - kt0 < 4 ? kts - kt0 : 4;            // tiles of this workgroup that exist (per segment)
  const uint32_t nbytes = (uint32_t)nt * kTileBytes;
  for (int sg = 0; sg < n_seg; ++sg) {
    const uint32_t role = (roles >> (2 * sg)) & 3u;
    if (sg > 0) __syncthreads();                                // the previous segment has left LDS
    uint32_t q[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) q[j] = role == kRoleNbm ? nbm[j] : role == kRoleBm ? only[j] : whole[j];
    const u32x4 lo4 = {q[0] | (q[1] << 24), (q[1] >> 8) | (q[2] << 16), (q[2] >> 16) | (q[3] << 8), q[4] | (q[5] << 24)};
    const u32x2 hi2 = {(q[5] >> 8) | (q[6] << 16), (q[6] >> 16) | (q[7] << 8)};
    *reinterpret_cast<u32x4*>(tile + slot * 16u) = lo4;
    *reinterpret_cast<u32x2*>(tile + 1024u + slot * 8u) = hi2;
    tile_scales[(kb_in >> 1) * 64u + slot] = (uint8_t)(role == kRoleNbm ? sbyte - delta : sbyte);
    __syncthreads();
    const int64_t kt_img = sg * kts + kt0;
    uint8_t* out = img_elems + (rt * k_tiles + kt_img) * (int64_t)kTileBytes;
    for (uint32_t o = t * 16u; o < nbytes; o += 256u * 16u)
      MXP_IMAGE_STORE(*reinterpret_cast<const u32x4*>(tiles + o), reinterpret_cast<u32x4*>(out + o));
    if ((int64_t)(t >> 6) < nt) img_scales[(((rt >> 2) * k_tiles + kt_img + (t >> 6)) * 64 + (t & 63u)) * 4 + (rt & 3)] = tile_scales[t];
  }
}

// Plain MXFP4 operand -> E2M1 image: the canonical 16-byte blocks moved to their lane slots, scales to the scale
// dwords (same patch walk as above; flushed blocks are zeroed, padding is zero elements with a unit scale).
// RES: an MXFP4+ operand kept in 4-bit codes for the few-row product.  The BM (2^2 * 1.m2m1m0) is split as in Eq. 3:
// its nibble becomes the E2M1 code of BM_H = 2^2 * 1.m2 (sign | 11 | m2), and the rest, BM_L = +-(m1 + m0 / 2), goes
// with the BM position into one residual byte per block, sign << 7 | m1 m0 << 5 | index, stored in the lane order of
// the tiles ([row tile][k-tile][64]) behind the scale part.
// RES == 2 (MXFP4++) / 3 (MXFP4+): the BM's nibble left as it is and the residual byte = position | delta << 5 (delta
// taken as 0 for MXFP4+; 0 for all-zero and NaN blocks): the product kernel takes the BM out of the 4-bit operand
// and feeds it as an E2M3 code with the block's own scale, the other elements with the scale lowered by delta (Sec. 4.3).
template <int RES>
__global__ void __launch_bounds__(256) prepack_e2m1_kernel(const u32x4* __restrict__ elems, const uint8_t* __restrict__ scales,
                                                           const uint8_t* __restrict__ bm_idx, int64_t rows, int64_t nbk,
                                                           int64_t k_tiles, uint8_t* __restrict__ img_elems,
                                                           uint8_t* __restrict__ img_scales, uint8_t* __restrict__ img_res) {
  __shared__ __attribute__((aligned(16))) uint8_t tiles[4 * kTileBytesE2M1];
  __shared__ uint8_t tile_scales[4 * 64];
  __shared__ uint8_t tile_res[4 * 64];
  const uint32_t t = threadIdx.x;
  const uint32_t r_in = t >> 3, kb_in = t & 7u;
  const PatchMap pm = patch_of_workgroup(blockIdx.x, (uint32_t)((k_tiles + 3) / 4), (uint32_t)(((rows + kRowPad - 1) / kRowPad) * 2));
  if (!pm.valid) return;
  const int64_t kt0 = pm.kg * 4, rt = pm.rt;
  const uint32_t slot = (kb_in & 1u) * 32u + r_in;
  const int64_t row = rt * kTileRows + r_in, kb = kt0 * 2 + kb_in;
  u32x4 v = {0, 0, 0, 0};
  uint32_t sbyte = RES >= 2 ? 0u : 127u, res = 0u;   // (RES == 2: absent blocks must read as blocks without a BM)
  if (row < rows && kb < nbk) {
    const int64_t b = row * nbk + kb;
    v = __builtin_nontemporal_load(elems + b);
    sbyte = scales[b];
    if (sbyte == 0u) v = (u32x4){0, 0, 0, 0};
    if (RES >= 2 && sbyte != 0u && sbyte != 255u) {
      // MXFP4+ ignores bits 7:5 of the index byte (reserved, Sec. 4.2); an MXFP4++ delta (Sec. 4.3) is kept at most
      // scale byte - 1, the range the conversion writes, so that lowering the scale byte by it never borrows
      const uint32_t ib = bm_idx[b], delta = RES == 3 ? 0u : (ib >> 5);
      res = (ib & 31u) | ((delta < sbyte ? delta : sbyte - 1u) << 5);
    }
    if (RES == 1 && sbyte != 0u && sbyte != 255u) {
      const uint32_t bm = bm_idx[b] & 31u, sh = 4u * (bm & 7u);
      uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t nib = (w[j] >> sh) & 15u;
        const uint32_t hi = (nib & 8u) | 6u | ((nib >> 2) & 1u);
        if ((bm >> 3) == (uint32_t)j) {
          w[j] = (w[j] & ~(15u << sh)) | (hi << sh);
          res = bm | ((nib & 3u) << 5) | ((nib & 8u) << 4);
        }
      }
      v = (u32x4){w[0], w[1], w[2], w[3]};
    }
  }
  *reinterpret_cast<u32x4*>(tiles + (kb_in >> 1) * kTileBytesE2M1 + slot * 16u) = v;
  tile_scales[(kb_in >> 1) * 64u + slot] = (uint8_t)sbyte;
  if (RES) tile_res[(kb_in >> 1) * 64u + slot] = (uint8_t)res;
  __syncthreads();
  const int64_t nt = k_tiles - kt0 < 4 ? k_tiles - kt0 : 4;
  uint8_t* out = img_elems + (rt * k_tiles + kt0) * (int64_t)kTileBytesE2M1;
  if (t * 16u < (uint32_t)nt * kTileBytesE2M1)
    MXP_IMAGE_STORE(*reinterpret_cast<const u32x4*>(tiles + t * 16u), reinterpret_cast<u32x4*>(out + t * 16u));
  if ((int64_t)(t >> 6) < nt) {
    img_scales[(((rt >> 2) * k_tiles + kt0 + (t >> 6)) * 64 + (t & 63u)) * 4 + (rt & 3)] = tile_scales[t];
    if (RES) img_res[(rt * k_tiles + kt0 + (t >> 6)) * 64 + (t & 63u)] = tile_res[t];
  }
}

// MXFP4 / MXFP4+ / MXFP4++ operand -> E4M3 image (the one image kind that can hold the two scales of an MXFP4++
// block, Sec. 4.3).  With the block scale byte raised to scale byte - delta + 2, an ordinary element (E2M1 value v,
// true value v * 2^(shared_exp - delta)) becomes v / 4, i.e. 0, 0.125, 0.25 ... 1.5: sign | LUT[magnitude]; the BM
// (2^2 * 1.mmm * 2^shared_exp) becomes 1.mmm * 2^delta: sign | (delta + 7) << 3 | mmm.  Same patch walk and LDS
// staging as above.
template <int MODE>
__global__ void __launch_bounds__(256) prepack_e4m3_kernel(const u32x4* __restrict__ elems, const uint8_t* __restrict__ scales,
                                                           const uint8_t* __restrict__ bm_idx, int64_t rows, int64_t nbk,
                                                           int64_t k_tiles, uint8_t* __restrict__ img_elems,
                                                           uint8_t* __restrict__ img_scales) {
  __shared__ __attribute__((aligned(16))) uint8_t tiles[4 * kTileBytesE4M3];
  __shared__ uint8_t tile_scales[4 * 64];
  const uint32_t t = threadIdx.x;
  const uint32_t r_in = t >> 3, kb_in = t & 7u;
  const PatchMap pm = patch_of_workgroup(blockIdx.x, (uint32_t)((k_tiles + 3) / 4), (uint32_t)(((rows + kRowPad - 1) / kRowPad) * 2));
  if (!pm.valid) return;
  const int64_t kt0 = pm.kg * 4, rt = pm.rt;
  const uint32_t slot = (kb_in & 1u) * 32u + r_in;
  const int64_t row = rt * kTileRows + r_in, kb = kt0 * 2 + kb_in;
  uint32_t n[4] = {0, 0, 0, 0};
  uint32_t sbyte = 127u, bm = 64u, delta = 0u;
  if (row < rows && kb < nbk) {
    const int64_t b = row * nbk + kb;
    const u32x4 v = __builtin_nontemporal_load(elems + b);
    n[0] = v.x; n[1] = v.y; n[2] = v.z; n[3] = v.w;
    sbyte = scales[b];
    if (MODE >= 1 && sbyte != 0u && sbyte != 255u) {
      const uint32_t ib = bm_idx[b];
      bm = ib & 31u;
      if (MODE == 2) delta = ib >> 5;
    }
    if (sbyte == 0u) n[0] = n[1] = n[2] = n[3] = 0u;          // flushed block: zero whatever the nibbles say
  }
  uint32_t d[8];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    d[2 * j] = nibbles4_to_e4m3(n[j] & 0xFFFFu);
    d[2 * j + 1] = nibbles4_to_e4m3(n[j] >> 16);
  }
  if (MODE >= 1 && bm < 32u) {
    const uint32_t nib = (n[bm >> 3] >> (4u * (bm & 7u))) & 15u;
    const uint32_t code = ((nib & 8u) << 4) | ((delta + 7u) << 3) | (nib & 7u);
    const uint32_t sh = (bm & 3u) * 8u;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if ((bm >> 2) == (uint32_t)j) d[j] = (d[j] & ~(0xFFu << sh)) | (code << sh);
  }
  // scale byte of the image: flushed and padding blocks are zeros with a unit scale, NaN stays NaN
  uint32_t sb = sbyte == 255u ? 255u : (sbyte == 0u ? 127u : sbyte - delta + 2u);
  if (row >= rows || kb >= nbk) sb = 127u;
  uint8_t* tile = tiles + (kb_in >> 1) * kTileBytesE4M3;
  // FP8 operand registers: the first four hold k = 16 (lane / 32) + 0..15, the last four the same + 32, while the
  // scale of lanes 0..31 covers k 0..31 and that of lanes 32..63 k 32..63.  Block (kb_in & 1) of the tile therefore
  // fills register half (kb_in & 1) of both lanes of its row: its codes 0..15 in lane r, 16..31 in lane r + 32.
  const uint32_t half = (kb_in & 1u) * 1024u;
  *reinterpret_cast<u32x4*>(tile + half + r_in * 16u) = u32x4{d[0], d[1], d[2], d[3]};
  *reinterpret_cast<u32x4*>(tile + half + (32u + r_in) * 16u) = u32x4{d[4], d[5], d[6], d[7]};
  tile_scales[(kb_in >> 1) * 64u + slot] = (uint8_t)sb;
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

int prepack_e4m3_launch(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows, int64_t K,
                        void* image, hipStream_t stream) {
  const ImageGeom g = image_geom(rows, K, kTileBytesE4M3);
  uint8_t* ie = static_cast<uint8_t*>(image);
  uint8_t* is = ie + g.elem_bytes;
  const int64_t n_wg = patch_grid((g.k_tiles + 3) / 4, g.row_tiles / 4);
  if (n_wg > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  dim3 grid((unsigned)n_wg);
  const u32x4* e = reinterpret_cast<const u32x4*>(elems);
  if (fmt == MXP_FMT_MXFP4PP)
    hipLaunchKernelGGL((prepack_e4m3_kernel<2>), grid, dim3(256), 0, stream, e, scales, bm_idx, rows, K / kBlock, g.k_tiles, ie, is);
  else if (fmt == MXP_FMT_MXFP4P)
    hipLaunchKernelGGL((prepack_e4m3_kernel<1>), grid, dim3(256), 0, stream, e, scales, bm_idx, rows, K / kBlock, g.k_tiles, ie, is);
  else
    hipLaunchKernelGGL((prepack_e4m3_kernel<0>), grid, dim3(256), 0, stream, e, scales, bm_idx, rows, K / kBlock, g.k_tiles, ie, is);
  return launch_status();
}

int prepack_launch(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows, int64_t K,
                   void* image, hipStream_t stream) {
  const ImageGeom g = image_geom(rows, K);
  uint8_t* ie = static_cast<uint8_t*>(image);
  uint8_t* is = ie + g.elem_bytes;
  const int64_t n_wg = patch_grid((g.k_tiles + 3) / 4, g.row_tiles / 4);
  if (n_wg > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  dim3 grid((unsigned)n_wg);
  const u32x4* e = reinterpret_cast<const u32x4*>(elems);
  if (fmt == MXP_FMT_MXFP4P)
    hipLaunchKernelGGL((prepack_kernel<true>), grid, dim3(256), 0, stream, e, scales, bm_idx, rows, K / kBlock, g.k_tiles, ie, is);
  else
    hipLaunchKernelGGL((prepack_kernel<false>), grid, dim3(256), 0, stream, e, scales, bm_idx, rows, K / kBlock, g.k_tiles, ie, is);
  return launch_status();
}

int prepack_seg_launch(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows, int64_t K, int n_seg,
                       uint32_t roles, void* image, hipStream_t stream) {
  const ImageGeom seg = image_geom(rows, K), g = image_geom(rows, seg.K_p * n_seg);
  uint8_t* ie = static_cast<uint8_t*>(image);
  uint8_t* is = ie + g.elem_bytes;
  const int64_t n_wg = patch_grid((seg.k_tiles + 3) / 4, seg.row_tiles / 4);
  if (n_wg > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)n_wg);
  const u32x4* e = reinterpret_cast<const u32x4*>(elems);
  if (fmt == MXP_FMT_MXFP4PP)
    hipLaunchKernelGGL(prepack_seg_kernel<2>, grid, dim3(256), 0, stream, e, scales, bm_idx, rows, K / kBlock, seg.k_tiles, n_seg, roles, ie, is);
  else if (fmt == MXP_FMT_MXFP4P)
    hipLaunchKernelGGL(prepack_seg_kernel<1>, grid, dim3(256), 0, stream, e, scales, bm_idx, rows, K / kBlock, seg.k_tiles, n_seg, roles, ie, is);
  else
    hipLaunchKernelGGL(prepack_seg_kernel<0>, grid, dim3(256), 0, stream, e, scales, bm_idx, rows, K / kBlock, seg.k_tiles, n_seg, roles, ie, is);
  return launch_status();
}

// mode 0: plain E2M1 image; 1: MXFP4+ operand, BM split, residual bytes behind the scales; 2 / 3: MXFP4++ / MXFP4+
// operand, BM nibble in place, position | delta << 5 behind the scales (delta = 0 for MXFP4+)
int prepack_e2m1_launch(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int64_t rows, int64_t K, void* image,
                        hipStream_t stream, int mode) {
  const ImageGeom g = image_geom(rows, K, kTileBytesE2M1);
  uint8_t* ie = static_cast<uint8_t*>(image);
  uint8_t* is = ie + g.elem_bytes;
  uint8_t* ir = is + g.scale_bytes;
  const int64_t n_wg = patch_grid((g.k_tiles + 3) / 4, g.row_tiles / 4);
  if (n_wg > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)n_wg);
  const u32x4* e = reinterpret_cast<const u32x4*>(elems);
  if (mode == 3) hipLaunchKernelGGL(prepack_e2m1_kernel<3>, grid, dim3(256), 0, stream, e, scales, bm_idx, rows, K / kBlock, g.k_tiles, ie, is, ir);
  else if (mode == 2) hipLaunchKernelGGL(prepack_e2m1_kernel<2>, grid, dim3(256), 0, stream, e, scales, bm_idx, rows, K / kBlock, g.k_tiles, ie, is, ir);
  else if (mode == 1) hipLaunchKernelGGL(prepack_e2m1_kernel<1>, grid, dim3(256), 0, stream, e, scales, bm_idx, rows, K / kBlock, g.k_tiles, ie, is, ir);
  else hipLaunchKernelGGL(prepack_e2m1_kernel<0>, grid, dim3(256), 0, stream, e, scales, bm_idx, rows, K / kBlock, g.k_tiles, ie, is, ir);
  return launch_status();
}

}  // namespace mxp

namespace {
template <int MODE>
int dequantize_launch(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int64_t rows, int64_t K, int64_t nbk,
                      int64_t nq, void* dst, bool bf, int64_t ld_dst, hipStream_t s) {
  using namespace mxp;
  (void)rows;
  const uint32_t* e32 = reinterpret_cast<const uint32_t*>(elems);
  const int64_t cap = (int64_t)kNumCU * 16;
  if (ld_dst == K) {
    constexpr int U = 4;
    if (!bf) {
      const int64_t nh = nq * 2, want4 = (nh + 256 * U - 1) / (256 * U);
      const dim3 grid4((unsigned)(want4 < cap ? want4 : cap));
      hipLaunchKernelGGL((dequantize_dense_f32_kernel<MODE, U>), grid4, dim3(256), 0, s, reinterpret_cast<const uint16_t*>(elems), scales,
                         bm_idx, nh, static_cast<float*>(dst));
      return launch_status();
    }
    const int64_t want = (nq + 256 * U - 1) / (256 * U);
    const dim3 grid((unsigned)(want < cap ? want : cap));
    hipLaunchKernelGGL((dequantize_dense_kernel<MODE, true, U>), grid, dim3(256), 0, s, e32, scales, bm_idx, nq, dst);
    return launch_status();
  }
  const int64_t want = (nq + 255) / 256;
  const dim3 grid((unsigned)(want < cap ? want : cap));
  if (bf) hipLaunchKernelGGL((dequantize_kernel<MODE, true>), grid, dim3(256), 0, s, e32, scales, bm_idx, nbk, ld_dst, nq, dst);
  else hipLaunchKernelGGL((dequantize_kernel<MODE, false>), grid, dim3(256), 0, s, e32, scales, bm_idx, nbk, ld_dst, nq, dst);
  return launch_status();
}
}  // namespace

extern "C" int mxp_dequantize(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows,
                              int64_t K, void* dst, int dst_dtype, int64_t ld_dst, void* stream) {
  using namespace mxp;
  const bool wide = is_wide_format(fmt);
  if (!wide && fmt != MXP_FMT_MXFP4 && fmt != MXP_FMT_MXFP4P && fmt != MXP_FMT_MXFP4PP) return MXP_ERR_FORMAT;
  if (dst_dtype != MXP_F32 && dst_dtype != MXP_BF16) return MXP_ERR_DTYPE;
  if (rows < 0 || K < 0 || K % kBlock != 0) return MXP_ERR_SHAPE;
  if (rows == 0 || K == 0) return MXP_OK;
  if (!elems || !scales || !dst || (fmt != MXP_FMT_MXFP4 && !plain_wide_format(fmt) && !bm_idx)) return MXP_ERR_NULL;
  if (ld_dst < K) return MXP_ERR_SHAPE;
  const int64_t esz = dst_dtype == MXP_BF16 ? 2 : 4;
  if (!aligned16(elems) || !aligned16(scales) || !aligned16(dst) || (bm_idx && !aligned16(bm_idx)) || (ld_dst * esz) % 16 != 0)
    return MXP_ERR_ALIGN;
  const int64_t nbk = K / kBlock, nq = rows * nbk * 4;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (wide) return wide_dequantize_launch(elems, scales, bm_idx, fmt, rows, K, dst, dst_dtype, ld_dst, s);
  const bool bf = dst_dtype == MXP_BF16;
  if (fmt == MXP_FMT_MXFP4PP) return dequantize_launch<2>(elems, scales, bm_idx, rows, K, nbk, nq, dst, bf, ld_dst, s);
  if (fmt == MXP_FMT_MXFP4P) return dequantize_launch<1>(elems, scales, bm_idx, rows, K, nbk, nq, dst, bf, ld_dst, s);
  return dequantize_launch<0>(elems, scales, bm_idx, rows, K, nbk, nq, dst, bf, ld_dst, s);
}

extern "C" size_t mxp_image_bytes(int64_t rows, int64_t K) {
  if (rows < 0 || K < 0) return 0;
  return (size_t)mxp::image_geom(rows, K).total();
}

extern "C" size_t mxp_image_bytes_e2m1(int64_t rows, int64_t K) {
  if (rows < 0 || K < 0) return 0;
  return (size_t)mxp::image_geom(rows, K, mxp::kTileBytesE2M1).total();
}

extern "C" size_t mxp_image_bytes_e4m3(int64_t rows, int64_t K) {
  if (rows < 0 || K < 0) return 0;
  return (size_t)mxp::image_geom(rows, K, mxp::kTileBytesE4M3).total();
}

extern "C" int mxp_prepack_e4m3(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows,
                                int64_t K, void* image, size_t image_bytes, void* stream) {
  using namespace mxp;
  if (fmt != MXP_FMT_MXFP4 && fmt != MXP_FMT_MXFP4P && fmt != MXP_FMT_MXFP4PP) return MXP_ERR_FORMAT;
  if (rows < 0 || K < 0 || K % kBlock != 0) return MXP_ERR_SHAPE;
  if (rows == 0 || K == 0) return MXP_OK;
  if (!elems || !scales || !image || (fmt != MXP_FMT_MXFP4 && !bm_idx)) return MXP_ERR_NULL;
  if (!aligned16(elems) || !aligned16(scales) || !aligned16(image) || (bm_idx && !aligned16(bm_idx))) return MXP_ERR_ALIGN;
  if (image_bytes < (size_t)image_geom(rows, K, kTileBytesE4M3).total()) return MXP_ERR_WORKSPACE;
  return prepack_e4m3_launch(elems, scales, bm_idx, fmt, rows, K, image, static_cast<hipStream_t>(stream));
}

extern "C" int mxp_prepack_e2m1(const uint8_t* elems, const uint8_t* scales, int64_t rows, int64_t K, void* image,
                                size_t image_bytes, void* stream) {
  using namespace mxp;
  if (rows < 0 || K < 0 || K % kBlock != 0) return MXP_ERR_SHAPE;
  if (rows == 0 || K == 0) return MXP_OK;
  if (!elems || !scales || !image) return MXP_ERR_NULL;
  if (!aligned16(elems) || !aligned16(scales) || !aligned16(image)) return MXP_ERR_ALIGN;
  if (image_bytes < (size_t)image_geom(rows, K, kTileBytesE2M1).total()) return MXP_ERR_WORKSPACE;
  return prepack_e2m1_launch(elems, scales, nullptr, rows, K, image, static_cast<hipStream_t>(stream), 0);
}

extern "C" size_t mxp_image_bytes_e2m1r(int64_t rows, int64_t K) {
  if (rows < 0 || K < 0) return 0;
  const mxp::ImageGeom g = mxp::image_geom(rows, K, mxp::kTileBytesE2M1);
  return (size_t)(g.total() + g.row_tiles * g.k_tiles * 64);
}

extern "C" int mxp_prepack_e2m1r(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int64_t rows, int64_t K,
                                 void* image, size_t image_bytes, void* stream) {
  using namespace mxp;
  if (rows < 0 || K < 0 || K % kBlock != 0) return MXP_ERR_SHAPE;
  if (rows == 0 || K == 0) return MXP_OK;
  if (!elems || !scales || !bm_idx || !image) return MXP_ERR_NULL;
  if (!aligned16(elems) || !aligned16(scales) || !aligned16(bm_idx) || !aligned16(image)) return MXP_ERR_ALIGN;
  if (image_bytes < mxp_image_bytes_e2m1r(rows, K)) return MXP_ERR_WORKSPACE;
  return prepack_e2m1_launch(elems, scales, bm_idx, rows, K, image, static_cast<hipStream_t>(stream), 1);
}

extern "C" int mxp_prepack_e2m1x(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows, int64_t K,
                                 void* image, size_t image_bytes, void* stream) {
  using namespace mxp;
  if (fmt != MXP_FMT_MXFP4P && fmt != MXP_FMT_MXFP4PP) return fmt == MXP_FMT_MXFP4 ? MXP_ERR_UNSUPPORTED : MXP_ERR_FORMAT;
  if (rows < 0 || K < 0 || K % kBlock != 0) return MXP_ERR_SHAPE;
  if (rows == 0 || K == 0) return MXP_OK;
  if (!elems || !scales || !bm_idx || !image) return MXP_ERR_NULL;
  if (!aligned16(elems) || !aligned16(scales) || !aligned16(bm_idx) || !aligned16(image)) return MXP_ERR_ALIGN;
  if (image_bytes < mxp_image_bytes_e2m1r(rows, K)) return MXP_ERR_WORKSPACE;
  return prepack_e2m1_launch(elems, scales, bm_idx, rows, K, image, static_cast<hipStream_t>(stream), fmt == MXP_FMT_MXFP4P ? 3 : 2);
}

extern "C" int mxp_prepack_seg(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows, int64_t K,
                               int n_seg, unsigned roles, void* image, size_t image_bytes, void* stream) {
  using namespace mxp;
  if (fmt != MXP_FMT_MXFP4 && fmt != MXP_FMT_MXFP4P && fmt != MXP_FMT_MXFP4PP) return MXP_ERR_FORMAT;
  if (rows < 0 || K < 0 || K % kBlock != 0 || n_seg < 1 || n_seg > 4 || (roles >> (2 * n_seg)) != 0u) return MXP_ERR_SHAPE;
  for (int sg = 0; sg < n_seg; ++sg) {
    const unsigned role = (roles >> (2 * sg)) & 3u;
    if (role == 3u) return MXP_ERR_SHAPE;
    // an MXFP4++ operand only exists as its two parts; a plain MXFP4 operand has no BM to split off
    if (fmt == MXP_FMT_MXFP4PP && role == 0u) return MXP_ERR_UNSUPPORTED;
    if (fmt == MXP_FMT_MXFP4 && role != 0u) return MXP_ERR_UNSUPPORTED;
  }
  if (rows == 0 || K == 0) return MXP_OK;
  if (!elems || !scales || !image || (fmt != MXP_FMT_MXFP4 && !bm_idx)) return MXP_ERR_NULL;
  if (!aligned16(elems) || !aligned16(scales) || !aligned16(image) || (bm_idx && !aligned16(bm_idx))) return MXP_ERR_ALIGN;
  if (image_bytes < mxp_image_bytes_fp6(rows, K, n_seg)) return MXP_ERR_WORKSPACE;
  return prepack_seg_launch(elems, scales, bm_idx, fmt, rows, K, n_seg, roles, image, static_cast<hipStream_t>(stream));
}

extern "C" int mxp_prepack(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows,
                           int64_t K, void* image, size_t image_bytes, void* stream) {
  using namespace mxp;
  if (fmt == MXP_FMT_MXFP4PP) return MXP_ERR_UNSUPPORTED;
  if (fmt != MXP_FMT_MXFP4 && fmt != MXP_FMT_MXFP4P) return MXP_ERR_FORMAT;
  if (rows < 0 || K < 0 || K % kBlock != 0) return MXP_ERR_SHAPE;
  if (rows == 0 || K == 0) return MXP_OK;
  if (!elems || !scales || !image || (fmt == MXP_FMT_MXFP4P && !bm_idx)) return MXP_ERR_NULL;
  if (!aligned16(elems) || !aligned16(scales) || !aligned16(image) || (bm_idx && !aligned16(bm_idx))) return MXP_ERR_ALIGN;
  if (image_bytes < (size_t)image_geom(rows, K).total()) return MXP_ERR_WORKSPACE;
  return prepack_launch(elems, scales, bm_idx, fmt, rows, K, image, static_cast<hipStream_t>(stream));
}
