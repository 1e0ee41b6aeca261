// mxp_gemm_w4a16 : D[M][N] = A[M][K] (bf16, not quantized) x deq(W)[N][K]^T, W in canonical MXFP4 / MXFP4+ / MXFP4++
// (few rows: a weight-read-bound kernel; many rows: a tiled kernel, which also takes MXFP6(+) / MXFP8(+) weights and, for
// the MXFP8+ products of mxp_gemm, quantized eight-bit activations).
//
// The conversion-based use of the formats (Sec. 5: on hardware that lacks low-precision units, or for weight-only
// quantization, the blocks are de-converted to a wider type the hardware multiplies, Eq. 2 inside the kernel; the BM
// needs one extra select per block).  Here the wider type is bf16 and the multiplier is the bf16 MFMA; the weights are
// read in their canonical 4.25 / 4.5-bit form, so for few activation rows the product is bound by 0.53-0.56 bytes per
// weight element.
#include "mxp_common.h"
#include "mxp_decode.h"

namespace {

using namespace mxp;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t f32_to_bf16_rne_bits(float v) {
  uint32_t u = __float_as_uint(v);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ v8bf as_v8bf(const uint32_t (&d)[4]) {
  union { u32x4 u; v8bf b; } c;
  c.u = (u32x4){d[0], d[1], d[2], d[3]};
  return c.b;
}

// ---- few activation rows (M <= 64): one workgroup per 32 weight rows, K split over its wavefronts ------------------
// A 32x32x16 bf16 MFMA operand lane l holds row l % 32 and eight k-slots 8 (l / 32) .. +7.  The sum over k does not care
// which k sits in which slot as long as both operands agree, so the two lane halves take two different MX blocks: in
// "super-step" t (64 elements of K) lane (n, h) de-converts block 2t + h of weight row n and feeds its 32 values to four
// MFMAs, eight at a time; the activation lane (m, h) loads the same eight k per MFMA.  The W operand goes first, so
// accumulator register r of lane l is D[m = l % 32][n = 8 (r / 4) + 4 (l / 32) + r % 4].
// A wavefront takes groups of 8 blocks (256 elements of K) of the 32 rows: it reads them the way they lie in memory
// (8 lanes per row: 128 contiguous bytes), passes them through a private LDS patch, and picks them up in operand order.
constexpr int kW4RowStride = 144;                            // 8 blocks x 16 B + 16 B padding against bank conflicts
constexpr int kW4PatchBytes = 32 * kW4RowStride + 256 + 256; // elements, scale bytes [32][8], index bytes [32][8]

// 32 codes -> 32 bf16 (16 dwords of pairs), Eq. 2.  The unpack-convert instruction runs over the whole block with the
// NBM scale, the BM is overwritten once, and the reserved scale codes are a select (0: zeros, 255: NaN).  Only when some
// lane of the wavefront holds a block whose values reach below the bf16 normal range (scale byte - delta < 2) does the
// wavefront take the general de-conversion, which builds those patterns from integer fields.
template <int MODE>
__device__ __forceinline__ void decode_block_bf16(const u32x4 q, uint32_t sbyte, uint32_t ib, uint32_t (&w)[16]) {
  const uint32_t dw[4] = {q.x, q.y, q.z, q.w};
  const uint32_t delta = MODE == 2 ? ib >> 5 : 0u;
  const bool tiny = sbyte != 0u && sbyte < 2u + delta;
  if (__builtin_amdgcn_ballot_w64(tiny) != 0) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      uint32_t out[8];
      decode_group<(MODE >= 1), true>(dw[s], sbyte, MODE >= 1 ? ib & 31u : 64u, (uint32_t)s, out, delta);
      w[4 * s] = out[0]; w[4 * s + 1] = out[1]; w[4 * s + 2] = out[2]; w[4 * s + 3] = out[3];
    }
    return;
  }
  const float X = __uint_as_float((sbyte - delta) << 23);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    union { v2bf v; uint32_t u; } c0, c1, c2, c3;
    c0.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(dw[j], X, 0);
    c1.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(dw[j], X, 1);
    c2.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(dw[j], X, 2);
    c3.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(dw[j], X, 3);
    w[4 * j] = c0.u; w[4 * j + 1] = c1.u; w[4 * j + 2] = c2.u; w[4 * j + 3] = c3.u;
  }
  if (MODE >= 1) {
    const uint32_t idx = ib & 31u;
    const uint32_t qd = idx < 8u ? dw[0] : idx < 16u ? dw[1] : idx < 24u ? dw[2] : dw[3];
    const uint32_t nib = (qd >> (4u * (idx & 7u))) & 15u;
    const float XB = __uint_as_float(sbyte << 23);
    const uint32_t bm = ((nib & 8u) << 12) | (__float_as_uint((float)(8u + (nib & 7u)) * (XB * 0.5f)) >> 16);   // exact: 4 bits
    const uint32_t sh = (idx & 1u) * 16u;
    const uint32_t keep = ~(0xFFFFu << sh), put = bm << sh;
#pragma unroll
    for (int j = 0; j < 16; ++j) w[j] = (idx >> 1) == (uint32_t)j ? (w[j] & keep) | put : w[j];
  }
  if (sbyte == 0u || sbyte == 255u) {                       // reserved codes: an all-zero block, a block that held NaN / Inf
    const uint32_t v = sbyte == 0u ? 0u : 0x7FC07FC0u;
#pragma unroll
    for (int j = 0; j < 16; ++j) w[j] = v;
  }
}

template <int MODE, int TMR, bool OUT_BF16, int WAVES>
__global__ void __launch_bounds__(64 * WAVES) w4a16_skinny_kernel(const uint16_t* __restrict__ A, int64_t lda,
                                                                  const u32x4* __restrict__ w_el, const uint8_t* __restrict__ w_sc,
                                                                  const uint8_t* __restrict__ w_ix, int64_t nbk, int64_t M, int64_t N,
                                                                  void* __restrict__ Dv, int64_t ldd) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  uint8_t* patch = lds_raw + wave * kW4PatchBytes;          // private to this wavefront (LDS operations of a wavefront run in order)
  uint8_t* p_sc = patch + 32 * kW4RowStride;
  uint8_t* p_ix = p_sc + 256;
  const int h = lane >> 5, nl = lane & 31;
  const int64_t n0 = (int64_t)blockIdx.x * 32;
  const int64_t groups = (nbk + 7) / 8;
  const bool meta_dwords = (nbk & 3) == 0;                  // scale / index bytes of 4 blocks can be read as one dword
  v16f acc[TMR];
  const uint16_t* a_row[TMR];
  bool a_ok[TMR];
#pragma unroll
  for (int i = 0; i < TMR; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    a_ok[i] = 32 * i + nl < M;
    a_row[i] = A + (a_ok[i] ? (int64_t)(32 * i + nl) * lda : 0) + h * 32;
  }

  // loads of one group in memory order: elements, 8 lanes per row; scale and index bytes, 2 lanes per row
  u32x4 q[4];
  uint32_t sc4, ix4;
  auto load_group = [&](int64_t g) {
    const int64_t kb0 = 8 * g;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t n = n0 + 8 * i + (lane >> 3), kb = kb0 + (lane & 7);
      q[i] = (u32x4){0, 0, 0, 0};
      if (n < N && kb < nbk) q[i] = __builtin_nontemporal_load(w_el + n * nbk + kb);
    }
    sc4 = 0;
    ix4 = 0;
    const int64_t n = n0 + (lane >> 1), kb = kb0 + 4 * (lane & 1);
    if (n < N && kb < nbk) {
      const int64_t b = n * nbk + kb;
      if (meta_dwords) {
        sc4 = *reinterpret_cast<const uint32_t*>(w_sc + b);
        if (MODE >= 1) ix4 = *reinterpret_cast<const uint32_t*>(w_ix + b);
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (kb + j < nbk) {
            sc4 |= (uint32_t)w_sc[b + j] << (8 * j);
            if (MODE >= 1) ix4 |= (uint32_t)w_ix[b + j] << (8 * j);
          }
        }
      }
    }
  };
  if (wave < groups) load_group(wave);
  for (int64_t g = wave; g < groups; g += WAVES) {
    const int64_t kb0 = 8 * g;
    // ---- through the patch into operand order
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<u32x4*>(patch + (8 * i + (lane >> 3)) * kW4RowStride + (lane & 7) * 16) = q[i];
    *reinterpret_cast<uint32_t*>(p_sc + (lane >> 1) * 8 + 4 * (lane & 1)) = sc4;
    if (MODE >= 1) *reinterpret_cast<uint32_t*>(p_ix + (lane >> 1) * 8 + 4 * (lane & 1)) = ix4;
    if (g + WAVES < groups) load_group(g + WAVES);          // the next group's loads fly while this one is multiplied
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int bl = 2 * t + h;                             // block of the group this lane de-converts
      // activations: lane (m, h) needs, for MFMA s, eight k of the same block (they stay in cache: A is small)
      u32x4 a[TMR][4];
#pragma unroll
      for (int i = 0; i < TMR; ++i) {
        const uint16_t* ap = a_row[i] + kb0 * 32 + t * 64;   // a_row already points at this lane's row and block half
        const bool ok = a_ok[i] && kb0 + bl < nbk;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          a[i][s] = (u32x4){0, 0, 0, 0};
          if (ok) a[i][s] = *reinterpret_cast<const u32x4*>(ap + 8 * s);
        }
      }
      const u32x4 qq = *reinterpret_cast<const u32x4*>(patch + nl * kW4RowStride + bl * 16);
      const uint32_t sb = p_sc[nl * 8 + bl];
      const uint32_t ib = MODE >= 1 ? (uint32_t)p_ix[nl * 8 + bl] : 0u;
      uint32_t w[16];
      decode_block_bf16<MODE>(qq, sb, ib, w);               // blocks past K or N were loaded as zeros with scale byte 0
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const uint32_t w4[4] = {w[4 * s], w[4 * s + 1], w[4 * s + 2], w[4 * s + 3]};
        const v8bf wv = as_v8bf(w4);
#pragma unroll
        for (int i = 0; i < TMR; ++i) {
          const uint32_t a4[4] = {a[i][s].x, a[i][s].y, a[i][s].z, a[i][s].w};
          acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, as_v8bf(a4), acc[i], 0, 0, 0);
        }
      }
    }
  }
  __syncthreads();                                          // the patches are dead: the same LDS now collects the partial tiles
  float (*part)[TMR][16][64] = reinterpret_cast<float (*)[TMR][16][64]>(lds_raw);
#pragma unroll
  for (int i = 0; i < TMR; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) part[wave][i][r][lane] = acc[i][r];
  __syncthreads();
  for (int e = tid; e < TMR * 16 * 64; e += 64 * WAVES) {
    const int l = e & 63, r = (e >> 6) & 15, i = e >> 10;
    float v = 0.0f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) v += part[w][i][r][l];
    const int64_t row = 32 * i + (l & 31);
    const int64_t col = n0 + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
    if (row < M && col < N) {
      if (OUT_BF16) static_cast<uint16_t*>(Dv)[row * ldd + col] = (uint16_t)f32_to_bf16_rne_bits(v);
      else static_cast<float*>(Dv)[row * ldd + col] = v;
    }
  }
}

template <int MODE, int TMR, bool OUT_BF16>
void launch_skinny(dim3 grid, hipStream_t s, const void* A, int64_t lda, const uint8_t* we, const uint8_t* ws, const uint8_t* wi,
                   int64_t nbk, int64_t M, int64_t N, void* D, int64_t ldd) {
  // two row tiles need more than the 128 registers a lane gets with 16 wavefronts (the compiler spilled ~90): 8 then
  constexpr int WAVES = TMR == 1 ? 16 : 8;
  constexpr int lds_part = WAVES * TMR * 16 * 64 * 4, lds_patch = WAVES * kW4PatchBytes;
  constexpr int lds = lds_part > lds_patch ? lds_part : lds_patch;
  static_assert(lds <= 160 * 1024, "LDS");
  allow_dynamic_lds<&w4a16_skinny_kernel<MODE, TMR, OUT_BF16, WAVES>>((int)lds);
  hipLaunchKernelGGL((w4a16_skinny_kernel<MODE, TMR, OUT_BF16, WAVES>), grid, dim3(64 * WAVES), lds, s,
                     static_cast<const uint16_t*>(A), lda, reinterpret_cast<const u32x4*>(we), ws, wi, nbk, M, N, D, ldd);
}

template <int MODE>
int dispatch_skinny(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const uint8_t* we, const uint8_t* ws,
                    const uint8_t* wi, void* D, int d_dtype, int64_t ldd, hipStream_t s) {
  const int64_t ct = (N + 31) / 32;
  if (ct > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)ct);
  const int64_t nbk = K / kBlock;
  const bool bf = d_dtype == MXP_BF16;
  if (M <= 32) {
    if (bf) launch_skinny<MODE, 1, true>(grid, s, A, lda, we, ws, wi, nbk, M, N, D, ldd);
    else launch_skinny<MODE, 1, false>(grid, s, A, lda, we, ws, wi, nbk, M, N, D, ldd);
  } else {
    if (bf) launch_skinny<MODE, 2, true>(grid, s, A, lda, we, ws, wi, nbk, M, N, D, ldd);
    else launch_skinny<MODE, 2, false>(grid, s, A, lda, we, ws, wi, nbk, M, N, D, ldd);
  }
  return launch_status();
}

// ---- tiled product on de-converted operands: 256 x 256 output tiles ------------------------------------------------
// Many activation rows (prefill with weight-only quantization), weights of any block format; and the product of two
// quantized operands whose BM fits no block-scaled MFMA element (MXFP8+): every format's values are bf16 numbers, so
// the product of the de-converted operands on the bf16 MFMA is the exact product (fp32 accumulation).
// A workgroup of 2 x 4 wavefronts (two per SIMD, so that one's conversions and LDS traffic run under the other's MFMAs)
// computes 256 rows of A x 256 rows of W; each wavefront 4 x 2 MFMA tiles of 32 x 32.  K is walked in steps of 64 (two
// MX blocks: the two lane halves of an operand take one each, as above).  Both operands of a step lie in LDS as bf16,
// 256 rows each, double-buffered: un-quantized activations are copied, quantized operands are de-converted (Eq. 2) on
// the way in -- thread (n, b) of the workgroup owns block b of row n in every step, one block per thread and step, so
// each block is converted once per workgroup.  Rows are 144 bytes apart in LDS (128 + 16 of padding): the 16 lanes that
// read the same chunk of 16 consecutive rows then hit 16 different 16-byte bank groups (9 r mod 16), and the chunk is an
// immediate offset of the read.  Global loads run one step (un-quantized rows) or two (codes) ahead of the MFMAs that
// use them and are written to the other LDS stage behind the MFMAs of the step before; one barrier per step.
constexpr int kTRow = 144;                                   // bytes per operand row in LDS: 64 bf16 + 16 B of padding
constexpr int kTOperand = 256 * kTRow;                       // one operand of one step: 256 rows x 64 bf16
constexpr int kTStage = 2 * kTOperand;                       // activations, then weights
constexpr int kTiledLds = 2 * kTStage;
constexpr int kTiledThreads = 512;

// operand kinds
constexpr int kRawBf16 = 0, kFp4 = 1 /* + MODE: 1, 2, 3 */, kFp6 = 4, kFp8 = 6;   // six- / eight-bit: plain or + by a flag

struct QBlock {                                              // one block of codes with its scale and index bytes
  uint32_t raw[8];
  uint32_t sb, ib;
};

template <int KIND>
__device__ __forceinline__ QBlock q_load(bool ok, const uint8_t* el, const uint8_t* sc, const uint8_t* ix, int64_t b, bool has_ix) {
  QBlock r;
#pragma unroll
  for (int j = 0; j < 8; ++j) r.raw[j] = 0;
  r.sb = 0;                                                  // blocks past the matrix: scale byte 0, an all-zero block
  r.ib = 0;
  if (ok) {
    if (KIND == kFp6) {
      const u32x2* p = reinterpret_cast<const u32x2*>(el + b * 24);
      const u32x2 d0 = p[0], d1 = p[1], d2 = p[2];
      r.raw[0] = d0.x; r.raw[1] = d0.y; r.raw[2] = d1.x; r.raw[3] = d1.y; r.raw[4] = d2.x; r.raw[5] = d2.y;
    } else if (KIND == kFp8) {
      const u32x4* p = reinterpret_cast<const u32x4*>(el + b * 32);
      const u32x4 d0 = p[0], d1 = p[1];
      r.raw[0] = d0.x; r.raw[1] = d0.y; r.raw[2] = d0.z; r.raw[3] = d0.w;
      r.raw[4] = d1.x; r.raw[5] = d1.y; r.raw[6] = d1.z; r.raw[7] = d1.w;
    } else {
      const u32x4 d0 = *reinterpret_cast<const u32x4*>(el + b * 16);
      r.raw[0] = d0.x; r.raw[1] = d0.y; r.raw[2] = d0.z; r.raw[3] = d0.w;
    }
    r.sb = sc[b];
    if (has_ix) r.ib = ix[b];
  }
  return r;
}

// Four-bit block -> 64 bytes of bf16 at `dst`.  As decode_block_bf16, except that the rare cases are kept out of the
// registers: the 32 elements are converted with the NBM scale and stored, then the BM is written over its two bytes
// with one LDS store, and blocks with a reserved scale byte (all-zero, NaN) are overwritten by the lanes that hold one
// (LDS operations of a wavefront execute in order).  Wavefronts with a block below the bf16 normal range take the
// general routine.
template <int MODE>
__device__ __forceinline__ void q_store_fp4(const QBlock& r, uint8_t* dst) {
  const uint32_t delta = MODE == 2 ? r.ib >> 5 : 0u;
  const bool tiny = r.sb != 0u && r.sb < 2u + delta;
  if (__builtin_amdgcn_ballot_w64(tiny) != 0) {
    uint32_t w[16];
    decode_block_bf16<MODE>((u32x4){r.raw[0], r.raw[1], r.raw[2], r.raw[3]}, r.sb, r.ib, w);
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4)
      *reinterpret_cast<u32x4*>(dst + 16 * s4) = (u32x4){w[4 * s4], w[4 * s4 + 1], w[4 * s4 + 2], w[4 * s4 + 3]};
    return;
  }
  const bool special = r.sb == 0u || r.sb == 255u;
  const float X = __uint_as_float((special ? 127u : r.sb - delta) << 23);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    union { v2bf v; uint32_t u; } c0, c1, c2, c3;
    c0.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(r.raw[j], X, 0);
    c1.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(r.raw[j], X, 1);
    c2.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(r.raw[j], X, 2);
    c3.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(r.raw[j], X, 3);
    *reinterpret_cast<u32x4*>(dst + 16 * j) = (u32x4){c0.u, c1.u, c2.u, c3.u};
  }
  if (MODE >= 1 && !special) {
    const uint32_t idx = r.ib & 31u;
    const uint32_t qd = idx < 8u ? r.raw[0] : idx < 16u ? r.raw[1] : idx < 24u ? r.raw[2] : r.raw[3];
    const uint32_t nib = (qd >> (4u * (idx & 7u))) & 15u;
    const float XB = __uint_as_float(r.sb << 23);
    const uint32_t bm = ((nib & 8u) << 12) | (__float_as_uint((float)(8u + (nib & 7u)) * (XB * 0.5f)) >> 16);   // exact: 4 bits
    *reinterpret_cast<uint16_t*>(dst + 2u * idx) = (uint16_t)bm;
  }
  if (__builtin_amdgcn_ballot_w64(special) != 0) {
    if (special) {
      const uint32_t v = r.sb == 0u ? 0u : 0x7FC07FC0u;
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) *reinterpret_cast<u32x4*>(dst + 16 * s4) = (u32x4){v, v, v, v};
    }
  }
}

// de-convert the block and store its 64 bytes of bf16 at `dst` (the block's place in its LDS row)
template <int KIND>
__device__ __forceinline__ void q_store(const QBlock& r, bool plus, uint8_t* dst) {
  if constexpr (KIND >= 1 && KIND <= 3) {
    q_store_fp4<KIND - 1>(r, dst);
    return;
  }
  uint32_t w[16];
  if (KIND == kFp6 || KIND == kFp8) {
    constexpr int BITS = KIND == kFp6 ? 6 : 8;
    const bool general = __builtin_amdgcn_ballot_w64(!wide_block_is_plain<BITS>(r.raw, r.sb, plus ? (r.ib & 31u) : 64u)) != 0;
    decode_wide_block_bf16<BITS>(r.raw, r.sb, r.ib, plus, general, w);
  } else {
    decode_block_bf16<(KIND >= 1 && KIND <= 3 ? KIND - 1 : 0)>((u32x4){r.raw[0], r.raw[1], r.raw[2], r.raw[3]}, r.sb, r.ib, w);
  }
#pragma unroll
  for (int s4 = 0; s4 < 4; ++s4)
    *reinterpret_cast<u32x4*>(dst + 16 * s4) = (u32x4){w[4 * s4], w[4 * s4 + 1], w[4 * s4 + 2], w[4 * s4 + 3]};
}

struct QOperand {                                            // a quantized operand: codes, scale bytes, index bytes
  const uint8_t *el, *sc, *ix;
  int plus;                                                  // six- / eight-bit kinds: the + form
};

template <int AK, int WK, bool OUT_BF16, int WI>
__global__ void __launch_bounds__(kTiledThreads) deconv_tiled_kernel(const uint16_t* __restrict__ A, int64_t lda, QOperand qa,
                                                                     QOperand qw, int64_t nbk, int64_t M, int64_t N,
                                                                     void* __restrict__ Dv, int64_t ldd, int tiles_n) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // WI row tiles per wavefront: 4 -> 256 rows of A per workgroup; 2 -> 128 rows, for launches that would otherwise leave
  // most compute units without a tile
  constexpr int NJ = 2, WAVES_N = 4, TROWS = 64 * WI, PA = TROWS * 8 / kTiledThreads;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N, h = lane >> 5, nl = lane & 31;
  const int64_t m0 = (int64_t)(blockIdx.x / tiles_n) * TROWS, n0 = (int64_t)(blockIdx.x % tiles_n) * 256;
  const int64_t nks = (nbk + 1) / 2;

  v16f acc[WI][NJ];
#pragma unroll
  for (int i = 0; i < WI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // un-quantized activations: chunk kc = tid % 8 of rows tid / 8 + 64 u
  const int a_row = tid >> 3, a_kc = tid & 7;
  const uint32_t a_off = (uint32_t)(a_row * kTRow + (a_kc << 4));
  constexpr int A_STEP = kTiledThreads / 8;
  const uint16_t* a_ptr[PA];
  bool a_ok[PA];
#pragma unroll
  for (int u = 0; u < PA; ++u) {
    a_ok[u] = AK == kRawBf16 && m0 + a_row + A_STEP * u < M;
    a_ptr[u] = A + (a_ok[u] ? (m0 + a_row + A_STEP * u) * lda : 0) + a_kc * 8;
  }
  // quantized operands: block b = tid % 2 of row tid / 2 in every step
  const int q_row = tid >> 1, q_b = tid & 1;
  const uint32_t q_off = (uint32_t)(q_row * kTRow + 64 * q_b);
  const bool qa_ok = AK != kRawBf16 && q_row < TROWS && m0 + q_row < M, qw_ok = n0 + q_row < N;
  const int64_t qa_base = qa_ok ? (m0 + q_row) * nbk + q_b : 0, qw_base = qw_ok ? (n0 + q_row) * nbk + q_b : 0;
  const bool a_has_ix = AK == 2 || AK == 3 || ((AK == kFp6 || AK == kFp8) && qa.plus);
  const bool w_has_ix = WK == 2 || WK == 3 || ((WK == kFp6 || WK == kFp8) && qw.plus);

  struct ABlock {
    u32x4 v[PA];
  };
  auto load_a = [&](int64_t ks) {
    ABlock r;
    const bool k_ok = 2 * ks + (a_kc >> 2) < nbk;            // the chunk's block exists (K % 32 == 0: chunks are whole)
#pragma unroll
    for (int u = 0; u < PA; ++u) {
      r.v[u] = (u32x4){0, 0, 0, 0};
      if (a_ok[u] && k_ok) r.v[u] = *reinterpret_cast<const u32x4*>(a_ptr[u] + ks * 64);
    }
    return r;
  };
  auto store_a = [&](int buf, const ABlock& r) {
#pragma unroll
    for (int u = 0; u < PA; ++u) *reinterpret_cast<u32x4*>(lds_raw + buf * kTStage + a_off + u * (A_STEP * kTRow)) = r.v[u];
  };
  auto load_qa = [&](int64_t ks) { return q_load<AK>(qa_ok && 2 * ks + q_b < nbk, qa.el, qa.sc, qa.ix, qa_base + 2 * ks, a_has_ix); };
  auto load_qw = [&](int64_t ks) { return q_load<WK>(qw_ok && 2 * ks + q_b < nbk, qw.el, qw.sc, qw.ix, qw_base + 2 * ks, w_has_ix); };

  // operand reads: lane (nl, h) of tile row / column r takes chunk 4 h + s4 (an immediate offset from these bases)
  uint32_t rd_a[WI], rd_w[NJ];
#pragma unroll
  for (int i = 0; i < WI; ++i) rd_a[i] = (uint32_t)((wm * (32 * WI) + 32 * i + nl) * kTRow + 64 * h);
#pragma unroll
  for (int j = 0; j < NJ; ++j) rd_w[j] = (uint32_t)(kTOperand + (wn * (32 * NJ) + 32 * j + nl) * kTRow + 64 * h);

  ABlock a1;
  QBlock qa1, qa2, qw1, qw2;
  if (AK == kRawBf16) {
    a1 = load_a(0);
    store_a(0, a1);
  } else {
    qa1 = load_qa(0);
    q_store<AK>(qa1, qa.plus != 0, lds_raw + q_off);
    qa1 = load_qa(1);
  }
  qw1 = load_qw(0);
  q_store<WK>(qw1, qw.plus != 0, lds_raw + kTOperand + q_off);
  qw1 = load_qw(1);
  __syncthreads();
  for (int64_t ks = 0; ks < nks; ++ks) {
    const bool more = ks + 1 < nks;
    const uint8_t* st = lds_raw + (ks & 1) * kTStage;
    uint8_t* nxt = lds_raw + ((ks + 1) & 1) * kTStage;
    if (AK == kRawBf16) {
      if (more) a1 = load_a(ks + 1);
    } else {
      qa2 = load_qa(ks + 2);
    }
    qw2 = load_qw(ks + 2);
    // the MFMAs of one eighth of K per slice (k-slots 8 s4 .. 8 s4 + 7 of both blocks)
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      v8bf wv[NJ];
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(st + rd_w[j] + 16 * s4);
        const uint32_t v4[4] = {v.x, v.y, v.z, v.w};
        wv[j] = as_v8bf(v4);
      }
#pragma unroll
      for (int i = 0; i < WI; ++i) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(st + rd_a[i] + 16 * s4);
        const uint32_t v4[4] = {v.x, v.y, v.z, v.w};
        const v8bf a8 = as_v8bf(v4);
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a8, wv[j], acc[i][j], 0, 0, 0);
      }
    }
    // the next step's operands go into the other stage.  (Measured alternatives that were slower: stores placed between
    // the MFMA slices -- the branches of the de-conversion cut the MFMA sequence --, activations loaded two steps ahead,
    // the two wavefronts of a SIMD running half a step out of phase, 2 x 2 wavefronts of 4 x 4 tiles.)
    if (more) {
      if (AK == kRawBf16) store_a((int)((ks + 1) & 1), a1);
      else q_store<AK>(qa1, qa.plus != 0, nxt + q_off);
      q_store<WK>(qw1, qw.plus != 0, nxt + kTOperand + q_off);
    }
    if (AK != kRawBf16) qa1 = qa2;
    qw1 = qw2;
    __syncthreads();
  }
  // accumulator register r of lane l: D[8 (r / 4) + 4 (l / 32) + r % 4][l % 32] of the 32 x 32 tile
  const bool whole = m0 + TROWS <= M && n0 + 256 <= N;
#pragma unroll
  for (int i = 0; i < WI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int64_t col = n0 + wn * (32 * NJ) + 32 * j + nl;
      const int64_t row0 = m0 + wm * (32 * WI) + 32 * i + 4 * h;
      if (whole) {                                           // tile inside the matrix (uniform): no per-element tests
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int64_t o = (row0 + 8 * (r >> 2) + (r & 3)) * ldd + col;
          if (OUT_BF16) static_cast<uint16_t*>(Dv)[o] = (uint16_t)f32_to_bf16_rne_bits(acc[i][j][r]);
          else static_cast<float*>(Dv)[o] = acc[i][j][r];
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int64_t row = row0 + 8 * (r >> 2) + (r & 3);
          if (row < M && col < N) {
            if (OUT_BF16) static_cast<uint16_t*>(Dv)[row * ldd + col] = (uint16_t)f32_to_bf16_rne_bits(acc[i][j][r]);
            else static_cast<float*>(Dv)[row * ldd + col] = acc[i][j][r];
          }
        }
      }
    }
}

template <int AK, int WK, int WI = 4>
int launch_deconv(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const QOperand& qa, const QOperand& qw, void* D,
                  int d_dtype, int64_t ldd, hipStream_t s) {
  const int64_t tm = (M + 64 * WI - 1) / (64 * WI), tn = (N + 255) / 256;
  if (tm * tn > 2147483647LL || tn > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)(tm * tn));
  const int64_t nbk = K / kBlock;
  static_assert(kTiledLds <= 160 * 1024, "LDS");
  if (d_dtype == MXP_BF16) {
    allow_dynamic_lds<&deconv_tiled_kernel<AK, WK, true, WI>>(kTiledLds);
    hipLaunchKernelGGL((deconv_tiled_kernel<AK, WK, true, WI>), grid, dim3(kTiledThreads), kTiledLds, s, static_cast<const uint16_t*>(A),
                       lda, qa, qw, nbk, M, N, D, ldd, (int)tn);
  } else {
    allow_dynamic_lds<&deconv_tiled_kernel<AK, WK, false, WI>>(kTiledLds);
    hipLaunchKernelGGL((deconv_tiled_kernel<AK, WK, false, WI>), grid, dim3(kTiledThreads), kTiledLds, s, static_cast<const uint16_t*>(A),
                       lda, qa, qw, nbk, M, N, D, ldd, (int)tn);
  }
  return launch_status();
}

// kind of the tiled kernel's operand loader for a block format, and whether it is the + form
inline int kind_of(int fmt) {
  switch (fmt) {
    case MXP_FMT_MXFP4: return 1;
    case MXP_FMT_MXFP4P: return 2;
    case MXP_FMT_MXFP4PP: return 3;
    case MXP_FMT_MXFP6: case MXP_FMT_MXFP6P: return kFp6;
    default: return kFp8;
  }
}
inline int plus_of(int fmt) { return fmt == MXP_FMT_MXFP6P || fmt == MXP_FMT_MXFP8P; }

// un-quantized bf16 activations x weights of any block format
int dispatch_tiled(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const uint8_t* we, const uint8_t* ws,
                   const uint8_t* wi, int fmtW, void* D, int d_dtype, int64_t ldd, hipStream_t s) {
  const QOperand none = {nullptr, nullptr, nullptr, 0}, qw = {we, ws, wi, plus_of(fmtW)};
  // fewer than ~200 tiles of 256 rows: tiles of 128 rows, twice as many workgroups (four-bit weights only)
  const bool small = ((M + 255) / 256) * ((N + 255) / 256) < 200 && M > 128;
  if (small && kind_of(fmtW) <= 3) {
    switch (kind_of(fmtW)) {
      case 1: return launch_deconv<kRawBf16, 1, 2>(M, N, K, A, lda, none, qw, D, d_dtype, ldd, s);
      case 2: return launch_deconv<kRawBf16, 2, 2>(M, N, K, A, lda, none, qw, D, d_dtype, ldd, s);
      default: return launch_deconv<kRawBf16, 3, 2>(M, N, K, A, lda, none, qw, D, d_dtype, ldd, s);
    }
  }
  switch (kind_of(fmtW)) {
    case 1: return launch_deconv<kRawBf16, 1>(M, N, K, A, lda, none, qw, D, d_dtype, ldd, s);
    case 2: return launch_deconv<kRawBf16, 2>(M, N, K, A, lda, none, qw, D, d_dtype, ldd, s);
    case 3: return launch_deconv<kRawBf16, 3>(M, N, K, A, lda, none, qw, D, d_dtype, ldd, s);
    case kFp6: return launch_deconv<kRawBf16, kFp6>(M, N, K, A, lda, none, qw, D, d_dtype, ldd, s);
    default: return launch_deconv<kRawBf16, kFp8>(M, N, K, A, lda, none, qw, D, d_dtype, ldd, s);
  }
}

}  // namespace

namespace mxp {
// Both operands quantized, at least one of them eight-bit (MXFP8 / MXFP8+ with each other or with any narrower format), or
// a six-bit format next to MXFP4++: the product of the de-converted operands.
int deconv_gemm_launch(int64_t M, int64_t N, int64_t K, const uint8_t* ae, const uint8_t* as, const uint8_t* ai, int fmtA,
                           const uint8_t* be, const uint8_t* bs, const uint8_t* bi, int fmtB, void* D, int d_dtype, int64_t ldd,
                           hipStream_t s) {
  const QOperand qa = {ae, as, ai, plus_of(fmtA)}, qb = {be, bs, bi, plus_of(fmtB)};
  const int ka = kind_of(fmtA), kb = kind_of(fmtB);
#define MXP_DECONV(AKV, BKV) return launch_deconv<AKV, BKV>(M, N, K, nullptr, 0, qa, qb, D, d_dtype, ldd, s)
  if (ka == kFp8) {
    switch (kb) {
      case 1: MXP_DECONV(kFp8, 1);
      case 2: MXP_DECONV(kFp8, 2);
      case 3: MXP_DECONV(kFp8, 3);
      case kFp6: MXP_DECONV(kFp8, kFp6);
      default: MXP_DECONV(kFp8, kFp8);
    }
  }
  if (ka == kFp6 && kb == 3) MXP_DECONV(kFp6, 3);              // six-bit next to MXFP4++: no block-scaled image pairing for it
  if (ka == 3 && kb == kFp6) MXP_DECONV(3, kFp6);
  if (kb != kFp8) return MXP_ERR_UNSUPPORTED;
  switch (ka) {
    case 1: MXP_DECONV(1, kFp8);
    case 2: MXP_DECONV(2, kFp8);
    case 3: MXP_DECONV(3, kFp8);
    default: MXP_DECONV(kFp6, kFp8);
  }
#undef MXP_DECONV
}
}  // namespace mxp

extern "C" int mxp_gemm_w4a16(int64_t M, int64_t N, int64_t K, const void* A, int a_dtype, int64_t lda,
                              const uint8_t* W_elems, const uint8_t* W_scales, const uint8_t* W_idx, int fmtW, void* D,
                              int d_dtype, int64_t ldd, void* stream) {
  using namespace mxp;
  if (fmtW < MXP_FMT_MXFP4 || fmtW > MXP_FMT_MXFP8P) return MXP_ERR_FORMAT;
  const bool wide_w = fmtW >= MXP_FMT_MXFP6;
  if (a_dtype != MXP_BF16 && a_dtype != MXP_F32) return MXP_ERR_DTYPE;
  const int rc0 = check_gemm(M, N, K, D, d_dtype, ldd);
  if (rc0 != MXP_OK || M == 0 || N == 0) return rc0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (K == 0) return zero_output(D, d_dtype, M, N, ldd, s);
  if (!A || !W_elems || !W_scales || (fmtW != MXP_FMT_MXFP4 && !plain_wide_format(fmtW) && !W_idx)) return MXP_ERR_NULL;
  if (lda < K) return MXP_ERR_SHAPE;
  if (a_dtype != MXP_BF16) return MXP_ERR_UNSUPPORTED;      // the activations are multiplied as bf16
  if (!aligned16(A) || !aligned16(W_elems) || !aligned16(W_scales) || (W_idx && !aligned16(W_idx)) || (lda * 2) % 16 != 0)
    return MXP_ERR_ALIGN;
  // six- and eight-bit weights: the tiled kernel at any number of rows
  if (wide_w) return dispatch_tiled(M, N, K, A, lda, W_elems, W_scales, W_idx, fmtW, D, d_dtype, ldd, s);
  if (M > 64 && M <= 128) {
    // two passes of the few-row kernel read the weights twice and still beat one row of 256 x 256 tiles here
    const int64_t esz = d_dtype == MXP_BF16 ? 2 : 4;
    for (int64_t r0 = 0; r0 < M; r0 += 64) {
      const int64_t mr = M - r0 < 64 ? M - r0 : 64;
      const void* Ar = static_cast<const uint16_t*>(A) + r0 * lda;
      void* Dr = static_cast<uint8_t*>(D) + r0 * ldd * esz;
      const int rc = fmtW == MXP_FMT_MXFP4PP  ? dispatch_skinny<2>(mr, N, K, Ar, lda, W_elems, W_scales, W_idx, Dr, d_dtype, ldd, s)
                     : fmtW == MXP_FMT_MXFP4P ? dispatch_skinny<1>(mr, N, K, Ar, lda, W_elems, W_scales, W_idx, Dr, d_dtype, ldd, s)
                                              : dispatch_skinny<0>(mr, N, K, Ar, lda, W_elems, W_scales, W_idx, Dr, d_dtype, ldd, s);
      if (rc != MXP_OK) return rc;
    }
    return MXP_OK;
  }
  if (M > 64) return dispatch_tiled(M, N, K, A, lda, W_elems, W_scales, W_idx, fmtW, D, d_dtype, ldd, s);
  if (fmtW == MXP_FMT_MXFP4PP) return dispatch_skinny<2>(M, N, K, A, lda, W_elems, W_scales, W_idx, D, d_dtype, ldd, s);
  if (fmtW == MXP_FMT_MXFP4P) return dispatch_skinny<1>(M, N, K, A, lda, W_elems, W_scales, W_idx, D, d_dtype, ldd, s);
  return dispatch_skinny<0>(M, N, K, A, lda, W_elems, W_scales, W_idx, D, d_dtype, ldd, s);
}
