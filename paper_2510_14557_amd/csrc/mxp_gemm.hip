// mxp_gemm : D[M][N] = A[M][K] x B[N][K]^T on MXFP4 / MXFP4+ operands (Sec. 5.1), fp32 accumulation.
//
// Operands are consumed as E2M3 images (mxp_prepack; a plain MXFP4 operand may stay an E2M1 image: the MFMA takes the
// two formats side by side at the same rate): every E2M1 element is exactly an E2M3 value and the BM of
// an MX+ block is an E2M3 number at exponent e_max (Sec. 4.2), so ONE block-scaled MFMA per block pair yields the
// exact products A_BM x B_NBM, B_BM x A_NBM and A_BM x B_BM that the paper obtains with a BM_H/BM_L split and an
// extra MMA (Sec. 5.2, Alg. 1) or with its BM Compute Unit (Sec. 6.2).  The shared E8M0 scales go to the MFMA as is.
//
// v_mfma_scale_f32_32x32x64_f8f6f4: lane l supplies the 32 K-consecutive elements (= one MX block, 24 bytes as E2M3)
// of operand row l % 32, K-block l / 32, plus that block's scale byte; accumulator register r of lane l is element
// [8 * (r / 4) + 4 * (l / 32) + r % 4][l % 32] of (first operand) x (second operand)^T.
#include "mxp_common.h"
#include <atomic>
#include <mutex>
#include <type_traits>

namespace mxp {
int prepack_launch(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows, int64_t K,
                   void* image, hipStream_t stream);
int prepack_e2m1_launch(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int64_t rows, int64_t K, void* image,
                        hipStream_t stream, int mode);
int prepack_e4m3_launch(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows, int64_t K,
                        void* image, hipStream_t stream);
int quantize_image_launch(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t ld_src, int fmt, uint8_t* elems,
                          uint8_t* scales, uint8_t* bm_idx, void* image, hipStream_t stream, bool skip_padding_tiles);
}  // namespace mxp

namespace mxp {
Chip chip() {
  constexpr int kMaxDev = 64;
  // one word per device, (cus << 32) | xcds, 0 = not asked yet: threads that ask at the same time store the same word
  static std::atomic<uint64_t> cache[kMaxDev] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return Chip{0, 0};
  uint64_t word = cache[dev].load(std::memory_order_relaxed);
  if (word == 0) {
    int cus = 0, xcds = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 0x7FFFFFFF;
    if (hipDeviceGetAttribute(&xcds, hipDeviceAttributeNumberOfXccs, dev) != hipSuccess || xcds < 0) xcds = 0;
    word = ((uint64_t)(uint32_t)cus << 32) | (uint32_t)xcds;
    cache[dev].store(word, std::memory_order_relaxed);
  }
  return Chip{(int)(word >> 32), (int)(word & 0xFFFFFFFFu)};
}

// Argument checks common to every product entry point (declared in mxp_common.h).
int check_gemm(int64_t M, int64_t N, int64_t K, const void* D, int d_dtype, int64_t ldd, int64_t max_k) {
  if (d_dtype != MXP_F32 && d_dtype != MXP_BF16) return MXP_ERR_DTYPE;
  if (M < 0 || N < 0 || K < 0 || K % kBlock != 0 || ldd < N) return MXP_ERR_SHAPE;
  if (K > max_k) return MXP_ERR_UNSUPPORTED;
  if (M > 0 && N > 0 && !D) return MXP_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(D) % (d_dtype == MXP_BF16 ? 2 : 4) != 0) return MXP_ERR_ALIGN;
  return MXP_OK;
}

namespace {
// K == 0: the product is an empty sum.
template <bool BF16>
__global__ void zero_kernel(void* D, int64_t M, int64_t N, int64_t ldd) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= M * N) return;
  const int64_t r = i / N, c = i - r * N;
  if (BF16) static_cast<uint16_t*>(D)[r * ldd + c] = 0;
  else static_cast<float*>(D)[r * ldd + c] = 0.0f;
}
}  // namespace

int zero_output(void* D, int d_dtype, int64_t M, int64_t N, int64_t ldd, hipStream_t s) {
  const unsigned grid = (unsigned)((M * N + 255) / 256);
  if (d_dtype == MXP_BF16) hipLaunchKernelGGL(zero_kernel<true>, dim3(grid), dim3(256), 0, s, D, M, N, ldd);
  else hipLaunchKernelGGL(zero_kernel<false>, dim3(grid), dim3(256), 0, s, D, M, N, ldd);
  return launch_status();
}
}  // namespace mxp

namespace {

using namespace mxp;
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kFmtE2M3 = 2;  // cbsz / blgp code of the f8f6f4 MFMA for FP6 E2M3 operands
constexpr int kFmtE4M3 = 0;  // ... for FP8 E4M3 operands (32 bytes per lane; the instruction then runs at half rate)
constexpr int kFmtE2M1 = 4;  // ... for FP4 E2M1 operands (16 bytes per lane: registers 4..7 of the operand are ignored)

// The B tile goes in as the MFMA's first operand and the A tile as its second, i.e. the instruction forms the
// transposed 32x32 tile: accumulator register r of lane l is then D[m = l % 32][n = 8 * (r / 4) + 4 * (l / 32) + r % 4],
// four consecutive columns per register quad, which the epilogue stores as one 16-byte piece.
// FB / FA = element format of the B / A operand: E2M3, or E2M1 for a plain MXFP4 operand kept in 4-bit codes.
template <int OA, int OB, int FB = kFmtE2M3, int FA = kFmtE2M3>
__device__ __forceinline__ v16f mfma(const v8i& a, const v8i& b, const v16f& c, int sa, int sb) {
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b, a, c, FB, FA, OB, sb, OA, sa);
}

template <int I, int J, int FB, int FA>
__device__ __forceinline__ v16f mfma_sel(const v8i& a, const v8i& b, const v16f& c, int sa, int sb) {
  return mfma<(I & 3), (J & 3), FB, FA>(a, b, c, sa, sb);
}

// Tile configuration: a workgroup of WAVES_M x WAVES_N wavefronts, each computing WM x WN MFMA tiles of 32 x 32.
template <int WM_, int WN_, int WAVES_M_, int WAVES_N_, int BT_ = kTileBytes, int AT_ = kTileBytes>
struct Cfg {
  static constexpr int WM = WM_, WN = WN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int BT = BT_;                                 // bytes of a B tile: 1536 (E2M3), 1024 (E2M1) or 2048 (E4M3)
  static constexpr int FB = BT_ == kTileBytes ? kFmtE2M3 : (BT_ == kTileBytesE4M3 ? kFmtE4M3 : kFmtE2M1);
  static constexpr int AT = AT_;                                 // bytes of an A tile, likewise
  static constexpr int FA = AT_ == kTileBytes ? kFmtE2M3 : (AT_ == kTileBytesE4M3 ? kFmtE4M3 : kFmtE2M1);
  static_assert(BT_ == kTileBytes || BT_ == kTileBytesE2M1 || BT_ == kTileBytesE4M3, "B tile kind");
  static_assert(AT_ == kTileBytes || AT_ == kTileBytesE2M1 || AT_ == kTileBytesE4M3, "A tile kind");
  static constexpr int TM = WM * WAVES_M, TN = WN * WAVES_N;   // 32-row tiles per workgroup
  static constexpr int THREADS = 64 * WAVES_M * WAVES_N;
  static constexpr int A_BYTES = TM * AT, B_BYTES = TN * BT;
  static constexpr int SA_BYTES = ((TM + 3) / 4) * 256, SB_BYTES = ((TN + 3) / 4) * 256;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES + SA_BYTES + SB_BYTES;
  static_assert(WM == 1 || WM == 2 || WM == 4 || WM == 8, "WM"); static_assert(WN == 1 || WN == 2 || WN == 4 || WN == 8, "WN");
  static constexpr int CHUNKS = STAGE_BYTES / 16;                 // 16-byte pieces per stage
  static constexpr int PER_THREAD = (CHUNKS + THREADS - 1) / THREADS;
};

// All WM x WN MFMAs of one k-tile.  op_sel picks, from the lane's scale dword, the byte of row tile i / column tile j.
template <class C>
__device__ __forceinline__ void mma_all(v16f (&acc)[C::WM][C::WN], const v8i (&a)[C::WM], const v8i (&b)[C::WN],
                                        const uint32_t (&sa)[(C::WM + 3) / 4], const uint32_t (&sb)[(C::WN + 3) / 4]) {
#pragma unroll
  for (int i = 0; i < C::WM; ++i)
#pragma unroll
    for (int j = 0; j < C::WN; ++j) {
        const int sai = (int)sa[i >> 2], sbj = (int)sb[j >> 2];
        switch ((i & 3) * 4 + (j & 3)) {
          case 0: acc[i][j] = mfma<0, 0, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          case 1: acc[i][j] = mfma<0, 1, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          case 2: acc[i][j] = mfma<0, 2, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          case 3: acc[i][j] = mfma<0, 3, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          case 4: acc[i][j] = mfma<1, 0, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          case 5: acc[i][j] = mfma<1, 1, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          case 6: acc[i][j] = mfma<1, 2, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          case 7: acc[i][j] = mfma<1, 3, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          case 8: acc[i][j] = mfma<2, 0, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          case 9: acc[i][j] = mfma<2, 1, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          case 10: acc[i][j] = mfma<2, 2, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          case 11: acc[i][j] = mfma<2, 3, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          case 12: acc[i][j] = mfma<3, 0, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          case 13: acc[i][j] = mfma<3, 1, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          case 14: acc[i][j] = mfma<3, 2, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
          default: acc[i][j] = mfma<3, 3, C::FB, C::FA>(a[i], b[j], acc[i][j], sai, sbj); break;
        }
      }
}

// Epilogue.  Lane l holds row m = l % 32 of the tile; register quad g holds columns 8g + 4(l / 32) .. +3.  With an
// aligned D each quad is one 16-byte (fp32) or 8-byte (bf16) store: 64 stores per wavefront tile instead of 256, which
// keeps the whole epilogue inside one window of the 6-bit vmcnt counter.
// fp32 -> bf16, round to nearest even, NaN stays NaN: the CDNA4 pack-convert instruction (one per two values).
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  union { bf16x2 v; uint32_t u; } c;
  c.v = __builtin_convertvector((f32x2){lo, hi}, bf16x2);
  return c.u;
}
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float v) { return pack_bf16x2(v, 0.0f) & 0xFFFFu; }

template <int TWM, int TWN, bool OUT_BF16>
__device__ __forceinline__ void store_tile(const v16f (&acc)[TWM][TWN], int64_t tile_m, int64_t tile_n, int lane, int64_t M,
                                           int64_t N, void* __restrict__ Dv, int64_t ldd) {
  const bool vec_ok = (ldd % 4 == 0) && ((reinterpret_cast<uintptr_t>(Dv) & 15u) == 0);
#pragma unroll
  for (int i = 0; i < TWM; ++i) {
    const int64_t row = (tile_m + i) * 32 + (lane & 31);
#pragma unroll
    for (int j = 0; j < TWN; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int64_t col = (tile_n + j) * 32 + 8 * g + 4 * (lane >> 5);
        if (row >= M || col >= N) continue;
        const float v0 = acc[i][j][4 * g], v1 = acc[i][j][4 * g + 1], v2 = acc[i][j][4 * g + 2], v3 = acc[i][j][4 * g + 3];
        if (vec_ok && col + 3 < N) {
          if (OUT_BF16) {
            u32x2 o = {pack_bf16x2(v0, v1), pack_bf16x2(v2, v3)};
            *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(Dv) + row * ldd + col) = o;
          } else {
            typedef float f32x4 __attribute__((ext_vector_type(4)));
            f32x4 o = {v0, v1, v2, v3};
            *reinterpret_cast<f32x4*>(static_cast<float*>(Dv) + row * ldd + col) = o;
          }
        } else {
          const float v[4] = {v0, v1, v2, v3};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            if (col + q < N) {
              if (OUT_BF16) static_cast<uint16_t*>(Dv)[row * ldd + col + q] = (uint16_t)f32_to_bf16_rne(v[q]);
              else static_cast<float*>(Dv)[row * ldd + col + q] = v[q];
            }
          }
        }
      }
    }
  }
}

// Epilogue through LDS for the large kernel.  Stored straight from the accumulator layout, a store instruction touches
// 64 different 128-byte lines with 16 bytes each, and the L2 then sees 4096 partial-line writes per wavefront tile.
// Each 32 x 32 tile is therefore passed through a private 32 x 36-float LDS patch (rows padded by 16 bytes against bank
// conflicts; LDS operations of one wavefront execute in order, so no wait is needed between the write and the read)
// and comes back with 8 consecutive lanes holding the 128 contiguous bytes of one row: every store instruction
// writes 8 full lines.  `patch` is this wavefront's scratch, two patches of kPatchBytes.
constexpr int kPatchStride = 144;                 // bytes per patch row: 32 floats + 16
constexpr int kPatchBytes = 32 * kPatchStride;

template <int TWM, int TWN, bool OUT_BF16>
__device__ __forceinline__ void store_tile_lds(const v16f (&acc)[TWM][TWN], int64_t tile_m, int64_t tile_n, int lane, int64_t M,
                                               int64_t N, void* __restrict__ Dv, int64_t ldd, uint8_t* patch) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  const bool vec_ok = (ldd % 4 == 0) && ((reinterpret_cast<uintptr_t>(Dv) & 15u) == 0);
  const int wr = (lane & 31) * kPatchStride + 16 * (lane >> 5);   // + 32 g
  const int rd = (lane >> 3) * kPatchStride + (lane & 7) * 16;    // + 8 k rows
  if (OUT_BF16 && vec_ok && TWN % 2 == 0) {
    // bf16: a row of one tile is only 64 bytes.  Two neighbouring tiles go through the two patches together and 16
    // consecutive lanes then hold the 128 contiguous bytes of one row (64 columns), so every store writes whole lines.
    const int rd2 = (lane >> 4) * kPatchStride + (lane & 7) * 16;  // + 4 k rows; patch (lane & 15) >> 3
    const uint8_t* pr = patch + ((lane & 15) >> 3) * kPatchBytes;
#pragma unroll
    for (int i = 0; i < TWM; ++i) {
#pragma unroll
      for (int j = 0; j < TWN; j += 2) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            f32x4 q = {acc[i][j + t][4 * g], acc[i][j + t][4 * g + 1], acc[i][j + t][4 * g + 2], acc[i][j + t][4 * g + 3]};
            *reinterpret_cast<f32x4*>(patch + t * kPatchBytes + wr + 32 * g) = q;
          }
        const int64_t col = (tile_n + j) * 32 + 4 * (lane & 15);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const f32x4 v = *reinterpret_cast<const f32x4*>(pr + rd2 + 4 * k * kPatchStride);
          const int64_t row = (tile_m + i) * 32 + 4 * k + (lane >> 4);
          if (row >= M || col >= N) continue;
          if (col + 3 < N) {
            u32x2 o = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
            __builtin_nontemporal_store(o, reinterpret_cast<u32x2*>(static_cast<uint16_t*>(Dv) + row * ldd + col));
          } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
              if (col + q < N) static_cast<uint16_t*>(Dv)[row * ldd + col + q] = (uint16_t)f32_to_bf16_rne(v[q]);
          }
        }
      }
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < TWM; ++i) {
#pragma unroll
    for (int j = 0; j < TWN; ++j) {
      uint8_t* pb = patch + ((i * TWN + j) & 1) * kPatchBytes;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 q = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        *reinterpret_cast<f32x4*>(pb + wr + 32 * g) = q;
      }
      const int64_t col = (tile_n + j) * 32 + 4 * (lane & 7);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(pb + rd + 8 * k * kPatchStride);
        const int64_t row = (tile_m + i) * 32 + 8 * k + (lane >> 3);
        if (row >= M || col >= N) continue;
        if (vec_ok && col + 3 < N) {
          if (OUT_BF16) {
            u32x2 o = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
            __builtin_nontemporal_store(o, reinterpret_cast<u32x2*>(static_cast<uint16_t*>(Dv) + row * ldd + col));
          } else {
            __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(static_cast<float*>(Dv) + row * ldd + col));
          }
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            if (col + q < N) {
              if (OUT_BF16) static_cast<uint16_t*>(Dv)[row * ldd + col + q] = (uint16_t)f32_to_bf16_rne(v[q]);
              else static_cast<float*>(Dv)[row * ldd + col + q] = v[q];
            }
          }
        }
      }
    }
  }
}

// One lane's operand of a tile held in LDS: 24 bytes (E2M3: low 16 + high 8) or 16 bytes (E2M1).
__device__ __forceinline__ v8i read_operand(const uint8_t* tile, int lane) {
  const u32x4 lo = *reinterpret_cast<const u32x4*>(tile + lane * 16);
  const u32x2 hi = *reinterpret_cast<const u32x2*>(tile + 1024 + lane * 8);
  return (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, 0, 0};
}
__device__ __forceinline__ v8i read_operand_e2m1(const uint8_t* tile, int lane) {
  const u32x4 lo = *reinterpret_cast<const u32x4*>(tile + lane * 16);
  return (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, 0, 0, 0, 0};
}
__device__ __forceinline__ v8i read_operand_e4m3(const uint8_t* tile, int lane) {
  const u32x4 lo = *reinterpret_cast<const u32x4*>(tile + lane * 16);
  const u32x4 hi = *reinterpret_cast<const u32x4*>(tile + 1024 + lane * 16);
  return (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
}
template <int TILE_BYTES>
__device__ __forceinline__ v8i read_b(const uint8_t* tile, int lane) {
  if (TILE_BYTES == kTileBytesE4M3) return read_operand_e4m3(tile, lane);
  return TILE_BYTES == kTileBytes ? read_operand(tile, lane) : read_operand_e2m1(tile, lane);
}

// Source address of 16-byte chunk c of a stage (k-tile kt) -- the stage is a concatenation of contiguous image runs.
template <class C>
__device__ __forceinline__ const u32x4* stage_src(int c, int64_t kt, int64_t k_tiles, const uint8_t* a_el, const uint8_t* a_sc,
                                                  const uint8_t* b_el, const uint8_t* b_sc, int64_t tm0, int64_t tn0) {
  constexpr int A_CH = C::A_BYTES / 16, B_CH = C::B_BYTES / 16, SA_CH = C::SA_BYTES / 16;
  const uint8_t* p;
  if (c < A_CH) {
    const int t = c / (C::AT / 16), w = c % (C::AT / 16);
    p = a_el + ((tm0 + t) * k_tiles + kt) * (int64_t)C::AT + w * 16;
  } else if (c < A_CH + B_CH) {
    const int cc = c - A_CH;
    const int t = cc / (C::BT / 16), w = cc % (C::BT / 16);
    p = b_el + ((tn0 + t) * k_tiles + kt) * (int64_t)C::BT + w * 16;
  } else if (c < A_CH + B_CH + SA_CH) {
    const int cc = c - A_CH - B_CH;
    const int g = cc / 16, w = cc % 16;
    p = a_sc + ((tm0 / 4 + g) * k_tiles + kt) * 256 + w * 16;
  } else {
    const int cc = c - A_CH - B_CH - SA_CH;
    const int g = cc / 16, w = cc % 16;
    p = b_sc + ((tn0 / 4 + g) * k_tiles + kt) * 256 + w * 16;
  }
  return reinterpret_cast<const u32x4*>(p);
}

template <class C, bool OUT_BF16>
__global__ void __launch_bounds__(C::THREADS) gemm_kernel(const uint8_t* __restrict__ a_el, const uint8_t* __restrict__ a_sc,
                                                          const uint8_t* __restrict__ b_el, const uint8_t* __restrict__ b_sc,
                                                          int64_t k_tiles, int64_t M, int64_t N, void* __restrict__ Dv, int64_t ldd) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;
  const int64_t tm0 = (int64_t)blockIdx.y * C::TM, tn0 = (int64_t)blockIdx.x * C::TN;

  v16f acc[C::WM][C::WN];
#pragma unroll
  for (int i = 0; i < C::WM; ++i)
#pragma unroll
    for (int j = 0; j < C::WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  u32x4 stg[C::PER_THREAD];
  auto fetch = [&](int64_t kt) {
#pragma unroll
    for (int u = 0; u < C::PER_THREAD; ++u) {
      const int c = tid + u * C::THREADS;
      if (c < C::CHUNKS) stg[u] = *stage_src<C>(c, kt, k_tiles, a_el, a_sc, b_el, b_sc, tm0, tn0);
    }
  };
  auto commit = [&](int buf) {
    u32x4* dst = reinterpret_cast<u32x4*>(lds + buf * C::STAGE_BYTES);
#pragma unroll
    for (int u = 0; u < C::PER_THREAD; ++u) {
      const int c = tid + u * C::THREADS;
      if (c < C::CHUNKS) dst[c] = stg[u];
    }
  };

  fetch(0);
  commit(0);
  __syncthreads();
  for (int64_t kt = 0; kt < k_tiles; ++kt) {
    const int buf = (int)(kt & 1);
    if (kt + 1 < k_tiles) fetch(kt + 1);
    const uint8_t* st = lds + buf * C::STAGE_BYTES;
    v8i a[C::WM], b[C::WN];
#pragma unroll
    for (int i = 0; i < C::WM; ++i) {
      a[i] = read_b<C::AT>(st + (wm * C::WM + i) * C::AT, lane);
    }
#pragma unroll
    for (int j = 0; j < C::WN; ++j) {
      b[j] = read_b<C::BT>(st + C::A_BYTES + (wn * C::WN + j) * C::BT, lane);
    }
    // scale dwords: byte q of group g = row tile 4g + q.  The tiles of one wavefront lie in one group when WM <= 4
    // (WM in {1, 2, 4} and workgroup tile origins are multiples of the workgroup tile); shift so that op_sel = i & 3
    // selects tile i.
    const int64_t ta = tm0 + wm * C::WM, tb = tn0 + wn * C::WN;
    const int ga = (int)((ta >> 2) - (tm0 >> 2)), gb = (int)((tb >> 2) - (tn0 >> 2));
    uint32_t sa[(C::WM + 3) / 4], sb[(C::WN + 3) / 4];
#pragma unroll
    for (int g = 0; g < (C::WM + 3) / 4; ++g)
      sa[g] = *reinterpret_cast<const uint32_t*>(st + C::A_BYTES + C::B_BYTES + (ga + g) * 256 + lane * 4) >> (8 * (int)(ta & 3));
#pragma unroll
    for (int g = 0; g < (C::WN + 3) / 4; ++g)
      sb[g] = *reinterpret_cast<const uint32_t*>(st + C::A_BYTES + C::B_BYTES + C::SA_BYTES + (gb + g) * 256 + lane * 4) >> (8 * (int)(tb & 3));
    mma_all<C>(acc, a, b, sa, sb);
    if (kt + 1 < k_tiles) commit(buf ^ 1);
    __syncthreads();
  }

  store_tile<C::WM, C::WN, OUT_BF16>(acc, tm0 + wm * C::WM, tn0 + wn * C::WN, lane, M, N, Dv, ldd);
}

// ---- pipelined persistent kernel: S-stage LDS ring filled by direct global->LDS loads ---------------------------
// A stage (one k-tile of the workgroup's A and B tiles plus their scale dwords) is a concatenation of contiguous image
// runs, so it is copied with global_load_lds_dwordx4: every lane fetches 16 bytes and the wavefront's 1 KiB lands
// contiguously in LDS at the address held in M0.  The copies bypass the VGPRs, are issued S-1 k-tiles before their use
// and are tracked by hand: the compiler does not see them, so each k-tile waits with an explicit vmcnt for the stage
// it is about to read, then meets the other wavefronts at a barrier.  Operand fragments are double-buffered in
// registers, and the LDS reads and copy issues of the following k-tiles are placed between the MFMAs of the current
// one, so that they issue in the shadow of the 8-pass MFMAs instead of ahead of them.
//
// One workgroup per compute unit walks a list of output tiles.  Full tiles are 256 x 256; some tile columns are cut
// into 256 x 128 half tiles so that (a) every workgroup gets the same amount of work and (b) half of the workgroups
// start with a half tile and the other half end with one: the two groups then run half a tile out of phase, and the
// output bursts of one group (64 MiB of fp32 per 256 tiles, HBM-write bound) overlap the MFMA phase of the other.
template <int N>
__device__ __forceinline__ void wait_dma_and_barrier() {
  // all but the newest N copies of this wavefront have landed; its own LDS reads are done; then meet the others
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// Copy engine state of one wavefront for one output tile: rows [32 tm0, +256), columns [32 tn0, +64 WN).  WN = 4: full
// tile (each wavefront 4 x 4 MFMA tiles, 8 B tiles per stage); WN = 2: half tile (4 x 2, 4 B tiles per stage).  The
// ring slot layout is the same for both: A tiles at 0, B tiles at A_BYTES, scale groups of A then of B behind.
// Everything except the per-lane offsets is wavefront-uniform and lives in SGPRs.  pA/pB/pS point at the runs of the
// next stage to copy and advance by one tile (one scale group) per k-tile; wslot is the LDS address of this
// wavefront's first copy in the next slot: copy u of a stage lands at wslot + 4096 u (element runs, 256 lanes x 16 B
// per round) and the scale dwords at wslot + sdelta.
template <class C, int S, int WN>
struct Copier {
  static constexpr bool B6 = C::BT == kTileBytes, A6 = C::AT == kTileBytes;
  static constexpr bool B8 = C::BT == kTileBytesE4M3, A8 = C::AT == kTileBytesE4M3;
  // copies per wavefront and stage: the 4 KiB rounds of A (E2M1: 2, E2M3: 3, E4M3: 4), of B (full tile: the same; half
  // tile: 1, 2 -- one and a half, the half one issued by every wavefront --, 2), one of scales
  static constexpr int A_ROUNDS = A8 ? 4 : (A6 ? 3 : 2);
  static constexpr int B_ROUNDS = WN == 4 ? (B8 ? 4 : (B6 ? 3 : 2)) : ((B8 || B6) ? 2 : 1);
  static constexpr int PER_STAGE = A_ROUNDS + B_ROUNDS + 1;
  uint32_t offE[4], offB[4], offH, offS;
  const uint8_t *pA, *pB, *pS;
  uint32_t wslot, wslot_end, sdelta, hdelta;

  __device__ __forceinline__ void init(uint32_t lds_base, const uint8_t* a_el, const uint8_t* a_sc, const uint8_t* b_el,
                                       const uint8_t* b_sc, int64_t k_tiles, int64_t tm0, int64_t tn0, int tid, int wave) {
    constexpr int TILE_CH = C::AT / 16;
    constexpr int TILE_CH_B = C::BT / 16;
#pragma unroll
    for (int u = 0; u < 4; ++u) {   // chunk tid + 256 u of an 8-tile run
      const int c = tid + u * C::THREADS;
      offE[u] = (uint32_t)((c / TILE_CH) * k_tiles * C::AT + (c % TILE_CH) * 16);
      offB[u] = (uint32_t)((c / TILE_CH_B) * k_tiles * C::BT + (c % TILE_CH_B) * 16);
    }
    // half tile: the B run has 4 tiles = 384 chunks; its second round is chunks 256..383, fetched by wavefronts 0-1
    // and fetched again (same source, same destination) by wavefronts 2-3 so that every wavefront issues the same
    // number of copies per stage.
    const int ch = 256 + (tid & 127);
    offH = (uint32_t)((ch / TILE_CH_B) * k_tiles * C::BT + (ch % TILE_CH_B) * 16);
    offS = (uint32_t)(tid & 63) * 4u;
    pA = a_el + tm0 * k_tiles * C::AT;
    pB = b_el + tn0 * k_tiles * C::BT;
    // Scale dwords: 256 bytes (64 lanes x 1 dword) per group of 4 row tiles and k-tile.  Wavefronts 0,1 copy A's two
    // groups, wavefronts 2,3 B's two groups (half tile: both copy B's only group; the second lands in an unused place).
    pS = wave < 2 ? a_sc + ((tm0 / 4 + wave) * k_tiles) * 256 : b_sc + ((tn0 / 4 + (WN == 4 ? wave - 2 : 0)) * k_tiles) * 256;
    wslot = lds_base + (uint32_t)wave * 1024u;
    wslot_end = wslot + (uint32_t)S * C::STAGE_BYTES;
    sdelta = (uint32_t)(C::A_BYTES + C::B_BYTES) + (uint32_t)wave * 256u - (uint32_t)wave * 1024u;
    hdelta = (uint32_t)C::A_BYTES + 4096u - (uint32_t)(wave >> 1) * 2048u;
  }
#define MXP_COPY16(voff, sptr, imm) \
  asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3" ::"s"(wslot), "n"(imm), "v"(voff), "s"(sptr) : "memory", "scc")
  // copy number u of the next stage; u = 6 is always the scale copy; 7 and 8 are the fourth rounds of E4M3 operands
  __device__ __forceinline__ void copy(int u) const {
    if (u == 0) MXP_COPY16(offE[0], pA, 0);
    else if (u == 1) MXP_COPY16(offE[1], pA, 4096);
    else if (u == 2 && (A6 || A8)) MXP_COPY16(offE[2], pA, 8192);
    else if (u == 7 && A8) MXP_COPY16(offE[3], pA, 12288);
    else if (u == 3) MXP_COPY16(offB[0], pB, C::A_BYTES);
    else if (u == 4 && (WN == 4 || B8)) MXP_COPY16(offB[1], pB, C::A_BYTES + 4096);
    else if (u == 5 && WN == 4 && (B6 || B8)) MXP_COPY16(offB[2], pB, C::A_BYTES + 8192);
    else if (u == 8 && WN == 4 && B8) MXP_COPY16(offB[3], pB, C::A_BYTES + 12288);
    else if (u == 4 && WN == 2 && B6)
      asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3" ::"s"(wslot), "s"(hdelta), "v"(offH), "s"(pB) : "memory", "scc");
    else if (u == 6)
      asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %2, %3" ::"s"(wslot), "s"(sdelta), "v"(offS), "s"(pS) : "memory", "scc");
  }
#undef MXP_COPY16
  __device__ __forceinline__ void next_stage() {
    pA += C::AT;
    pB += C::BT;
    pS += 256;
    wslot += C::STAGE_BYTES;
    if (wslot == wslot_end) wslot -= (uint32_t)S * C::STAGE_BYTES;
  }
  __device__ __forceinline__ void issue_stage() {
#pragma unroll
    for (int u = 0; u < 9; ++u) copy(u);   // rounds that do not exist for this tile kind are no-ops
    next_stage();
  }
  // same state change as `n` issue_stage() calls, without the copies (they were issued ahead of time)
  __device__ __forceinline__ void skip_stages(int n) {
    pA += (int64_t)n * C::AT;
    pB += (int64_t)n * C::BT;
    pS += (int64_t)n * 256;
    wslot += (uint32_t)n * C::STAGE_BYTES;   // n <= S and the ring starts at slot 0 for every tile
    if (wslot == wslot_end) wslot -= (uint32_t)S * C::STAGE_BYTES;
  }
};

// Where the epilogue patches (4 wavefronts x 2 x kPatchBytes) live.  Behind the ring when both fit in the 160 KiB of LDS.
// With E4M3 operands they do not; the patches then start at the last ring slot: the ring is idle during an epilogue
// (every wavefront has passed the barrier after its last fragment reads), the next tile's prologue, which a wavefront
// issues right after its own stores, only fills slots 0 .. S-2, and the first copy into slot S-1 is issued behind the
// next tile's first barrier, which no wavefront reaches before it has finished its epilogue.
template <class C, int S>
__host__ __device__ constexpr int patch_base() {
  return S * C::STAGE_BYTES + 4 * 2 * kPatchBytes <= 160 * 1024 ? S * C::STAGE_BYTES : (S - 1) * C::STAGE_BYTES;
}

// How many stages are kept issued ahead of the one being multiplied.  Iteration kt issues stage kt + depth right behind
// its barrier, into the slot of stage kt: every wavefront has finished reading that slot by then (it waits for its own LDS
// reads before the barrier).  That is the whole ring, depth = S, when the epilogue patches have LDS of their own; when they
// share the last slot, that slot must stay empty across an epilogue and the depth is S - 1.
// DEEP is chosen per launch: with a single tile per workgroup (few tiles: the launch is bound by how fast one workgroup
// draws its operands) the whole ring measured 5 % faster, with several tiles per workgroup (the chip is busy everywhere)
// 2 - 3 % slower than S - 1.
template <class C, int S, bool DEEP>
__host__ __device__ constexpr int ring_depth() {
  return DEEP && patch_base<C, S>() == S * C::STAGE_BYTES ? S : S - 1;
}

// Stages 0 .. depth-1 of a tile (its prologue), issued either at kernel start or while the previous tile is being stored.
template <class C, int S, bool DEEP, int WN>
__device__ __forceinline__ void issue_prologue(uint8_t* lds, const uint8_t* a_el, const uint8_t* a_sc, const uint8_t* b_el,
                                               const uint8_t* b_sc, int64_t k_tiles, int64_t tm0, int64_t tn0) {
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  Copier<C, S, WN> cp;
  cp.init((uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds, a_el, a_sc, b_el, b_sc, k_tiles, tm0, tn0, tid, wave);
#pragma unroll
  for (int s = 0; s < ring_depth<C, S, DEEP>(); ++s) cp.issue_stage();
}

// One output tile whose prologue copies are already in flight.  Requires k_tiles >= ring depth and even.  `next_kind`
// (0 none, 2 half, 4 full) and its coordinates: the prologue of the following tile is issued before this tile's
// epilogue, so that those copies land while the output is being stored.
template <class C, int S, bool DEEP, int WN, bool OUT_BF16>
__device__ __forceinline__ void run_tile(uint8_t* lds, const uint8_t* __restrict__ a_el, const uint8_t* __restrict__ a_sc,
                                         const uint8_t* __restrict__ b_el, const uint8_t* __restrict__ b_sc, int64_t k_tiles,
                                         int64_t M, int64_t N, void* __restrict__ Dv, int64_t ldd, int64_t tm0, int64_t tn0,
                                         int next_kind, int64_t ntm0, int64_t ntn0) {
  static_assert(C::WM == 4 && C::WN == 4 && C::WAVES_M == 2 && C::WAVES_N == 2, "written for 2 x 2 wavefronts of 4 x 4 tiles");
  static_assert(WN == 4 || WN == 2, "full or half tile");
  static_assert(S >= 4, "ring slots");
  constexpr int DEPTH = ring_depth<C, S, DEEP>();
  static_assert(C::A_BYTES == 8 * C::AT && C::THREADS == 256 && C::SA_BYTES == 512 && C::SB_BYTES == 512, "stage geometry");
  using CP = Copier<C, S, WN>;
  constexpr int PER_STAGE = CP::PER_STAGE;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  CP cp;
  cp.init((uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds, a_el, a_sc, b_el, b_sc, k_tiles, tm0, tn0, tid, wave);
  cp.skip_stages(DEPTH);

  v16f acc[4][WN];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const int64_t ta = tm0 + wm * 4, tb = tn0 + wn * WN;
  const int a_tiles_off = wm * 4 * C::AT;
  const int b_tiles_off = C::A_BYTES + wn * WN * C::BT;
  const int sa_off = C::A_BYTES + C::B_BYTES + wm * 256 + lane * 4;
  // full tile: group wn of B, bytes 0..3 = the wavefront's 4 column tiles; half tile: group 0, bytes 2 wn, 2 wn + 1
  const int sb_off = C::A_BYTES + C::B_BYTES + C::SA_BYTES + (WN == 4 ? wn * 256 : 0) + lane * 4;
  const int sb_shift = WN == 4 ? 0 : 16 * wn;

  v8i a0[4], b0[WN], a1[4], b1[WN];
  uint32_t sa0, sb0, sa1, sb1;

  // Copy accounting.  The copies of one wavefront complete in order, PER_STAGE of them per stage; stores of the
  // previous tile that are still in flight also count in vmcnt, but loads complete in order among themselves, so
  // "at most n operations outstanding" always implies "at most n copies outstanding": a wait can only be longer than
  // needed, never shorter.  The prologue issued stages 0 .. DEPTH-1 and stage 0 is needed: DEPTH-1 newer stages may stay
  // in flight.  Iteration kt waits BEFORE it issues stage kt+DEPTH, so stages up to kt+DEPTH-1 are issued and it needs
  // stage kt+1: DEPTH-2 newer stages may stay in flight.  The last DEPTH iterations issue nothing and wait for
  // correspondingly fewer stages.
  constexpr int KEEP_PROLOGUE = (DEPTH - 1) * PER_STAGE;
  constexpr int KEEP = (DEPTH - 2) * PER_STAGE;

  wait_dma_and_barrier<KEEP_PROLOGUE>();
#pragma unroll
  for (int i = 0; i < 4; ++i) a0[i] = read_b<C::AT>(lds + a_tiles_off + i * C::AT, lane);
#pragma unroll
  for (int j = 0; j < WN; ++j) b0[j] = read_b<C::BT>(lds + b_tiles_off + j * C::BT, lane);
  sa0 = *reinterpret_cast<const uint32_t*>(lds + sa_off);
  sb0 = *reinterpret_cast<const uint32_t*>(lds + sb_off) >> sb_shift;

  int read_off = C::STAGE_BYTES;    // byte offset of the ring slot of k-tile kt + 1

  // One k-tile: 4 WN MFMAs on (ca, cb).  An MFMA keeps the matrix pipe busy for ~35 clocks while the wavefront can
  // issue one other instruction every 4 clocks, so the work for later k-tiles is dealt out a few instructions per gap:
  // the barrier after MFMA 1, then the LDS reads of the next k-tile, then the copies of stage kt + DEPTH.
  // COPY: this iteration issues a stage.  KEEPN: copies that may stay in flight at its wait.  NEXT: there is a next
  // k-tile to wait for and read.
  // Order of the MFMAs of a k-tile: column tile j outermost, row tile i running back and forth, so that consecutive MFMAs
  // share one operand and every step changes the other one only (the raster order changes both at each row end).  The
  // matrix pipe's power draw, which is what limits its clock, depends on how many operand bits toggle: 0.6 % of the
  // launch time on random operands.
#define MXP_J(m) ((m) / 4)
#define MXP_I(m) ((((m) / 4) & 1) ? 3 - (m) % 4 : (m) % 4)
#define MXP_MFMA(m)                                                                                                          \
  acc[MXP_I(m)][MXP_J(m)] = mfma_sel<MXP_I(m), MXP_J(m), C::FB, C::FA>(ca[MXP_I(m)], cb[MXP_J(m)], acc[MXP_I(m)][MXP_J(m)], (int)csa, (int)csb); \
  __builtin_amdgcn_sched_barrier(0)
#define MXP_GAP() __builtin_amdgcn_sched_barrier(0)
#define MXP_READ(stmt) do { if (NEXT) { stmt; } } while (0)
#define MXP_CP(u) do { if (COPY) cp.copy(u); } while (0)
  auto ktile = [&](auto copy_tag, auto keep_tag, auto next_tag, const v8i (&ca)[4], const v8i (&cb)[WN], const uint32_t csa,
                   const uint32_t csb, v8i (&na)[4], v8i (&nb)[WN], uint32_t& nsa, uint32_t& nsb) {
    constexpr bool COPY = decltype(copy_tag)::value;
    constexpr int KEEPN = decltype(keep_tag)::value;
    constexpr bool NEXT = decltype(next_tag)::value;
    MXP_MFMA(0);
    MXP_MFMA(1);
    if (NEXT) wait_dma_and_barrier<KEEPN>();           // stage kt + 1 is complete in LDS for every wavefront
    const uint8_t* st = lds + read_off;
    MXP_GAP();
    if constexpr (WN == 4) {
      MXP_MFMA(2);
      MXP_READ(na[0] = read_b<C::AT>(st + a_tiles_off + 0 * C::AT, lane));
      MXP_GAP();
      MXP_MFMA(3);
      MXP_READ(na[1] = read_b<C::AT>(st + a_tiles_off + 1 * C::AT, lane));
      MXP_GAP();
      MXP_MFMA(4);
      MXP_READ(na[2] = read_b<C::AT>(st + a_tiles_off + 2 * C::AT, lane));
      MXP_GAP();
      MXP_MFMA(5);
      MXP_READ(na[3] = read_b<C::AT>(st + a_tiles_off + 3 * C::AT, lane));
      MXP_GAP();
      MXP_MFMA(6);
      MXP_READ(nb[0] = read_b<C::BT>(st + b_tiles_off + 0 * C::BT, lane));
      MXP_GAP();
      MXP_MFMA(7);
      MXP_READ(nb[1] = read_b<C::BT>(st + b_tiles_off + 1 * C::BT, lane));
      MXP_GAP();
      MXP_MFMA(8);
      MXP_READ(nb[2] = read_b<C::BT>(st + b_tiles_off + 2 * C::BT, lane));
      MXP_READ(nb[3] = read_b<C::BT>(st + b_tiles_off + 3 * C::BT, lane));
      MXP_READ(nsa = *reinterpret_cast<const uint32_t*>(st + sa_off));
      MXP_READ(nsb = *reinterpret_cast<const uint32_t*>(st + sb_off));
      MXP_GAP();
      MXP_MFMA(9);
      MXP_CP(0);
      MXP_GAP();
      MXP_MFMA(10);
      MXP_CP(1);
      MXP_GAP();
      MXP_MFMA(11);
      MXP_CP(2);
      MXP_GAP();
      MXP_MFMA(12);
      MXP_CP(3);
      MXP_GAP();
      MXP_MFMA(13);
      MXP_CP(4);
      MXP_GAP();
      MXP_MFMA(14);
      MXP_CP(5);
      MXP_GAP();
      MXP_MFMA(15);
      MXP_CP(6);
      MXP_CP(7);
      MXP_CP(8);
    } else {
      // (in the order the next k-tile's MFMAs want them: only three MFMAs separate the last read from the first use)
      MXP_MFMA(2);
      MXP_READ(nb[0] = read_b<C::BT>(st + b_tiles_off + 0 * C::BT, lane));
      MXP_READ(na[0] = read_b<C::AT>(st + a_tiles_off + 0 * C::AT, lane));
      MXP_READ(nsa = *reinterpret_cast<const uint32_t*>(st + sa_off));
      MXP_READ(nsb = *reinterpret_cast<const uint32_t*>(st + sb_off) >> sb_shift);
      MXP_GAP();
      MXP_MFMA(3);
      MXP_READ(na[1] = read_b<C::AT>(st + a_tiles_off + 1 * C::AT, lane));
      MXP_READ(na[2] = read_b<C::AT>(st + a_tiles_off + 2 * C::AT, lane));
      MXP_GAP();
      MXP_MFMA(4);
      MXP_READ(na[3] = read_b<C::AT>(st + a_tiles_off + 3 * C::AT, lane));
      MXP_READ(nb[1] = read_b<C::BT>(st + b_tiles_off + 1 * C::BT, lane));
      MXP_GAP();
      MXP_MFMA(5);
      MXP_CP(0);
      MXP_CP(1);
      MXP_GAP();
      MXP_MFMA(6);
      MXP_CP(2);
      MXP_CP(3);
      MXP_GAP();
      MXP_MFMA(7);
      MXP_CP(4);
      MXP_CP(6);
      MXP_CP(7);
    }
    if (COPY) cp.next_stage();
    read_off = read_off + C::STAGE_BYTES == S * C::STAGE_BYTES ? 0 : read_off + C::STAGE_BYTES;
    MXP_GAP();
  };
  using T = std::true_type;
  using F = std::false_type;
  using K1 = std::integral_constant<int, KEEP>;

  // steady state: iterations 0 .. k_tiles-DEPTH-1, each issuing a stage, in pairs (the operand registers alternate);
  // k_tiles is even, so an odd depth leaves one single iteration
  for (int64_t kt = 0; kt + 1 < k_tiles - DEPTH; kt += 2) {
    ktile(T{}, K1{}, T{}, a0, b0, sa0, sb0, a1, b1, sa1, sb1);
    ktile(T{}, K1{}, T{}, a1, b1, sa1, sb1, a0, b0, sa0, sb0);
  }
  if constexpr (DEPTH % 2 == 1) ktile(T{}, K1{}, T{}, a0, b0, sa0, sb0, a1, b1, sa1, sb1);
  // tail: the last DEPTH iterations issue nothing; at the wait of the j-th of them (j = 0 .. DEPTH-1) all stages are issued,
  // stage k_tiles-DEPTH+j+1 is the one needed and DEPTH-2-j newer ones may stay in flight; the last has no successor
  auto tail = [&](auto self, auto jc) {
    constexpr int J = decltype(jc)::value;
    if constexpr (J < DEPTH) {
      constexpr int KEEPJ = (DEPTH - 2 - J > 0 ? DEPTH - 2 - J : 0) * PER_STAGE;
      using KJ = std::integral_constant<int, KEEPJ>;
      using NJ = std::integral_constant<bool, (J < DEPTH - 1)>;
      if constexpr ((DEPTH + J) % 2 == 0) ktile(F{}, KJ{}, NJ{}, a0, b0, sa0, sb0, a1, b1, sa1, sb1);
      else ktile(F{}, KJ{}, NJ{}, a1, b1, sa1, sb1, a0, b0, sa0, sb0);
      self(self, std::integral_constant<int, J + 1>{});
    }
  };
  tail(tail, std::integral_constant<int, 0>{});
#undef MXP_MFMA
#undef MXP_I
#undef MXP_J
#undef MXP_GAP
#undef MXP_READ
#undef MXP_CP
  // every wavefront has read its last fragments: the ring may be refilled
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  store_tile_lds<4, WN, OUT_BF16>(acc, ta, tb, lane, M, N, Dv, ldd, lds + patch_base<C, S>() + wave * (2 * kPatchBytes));
  if (next_kind == 4) issue_prologue<C, S, DEEP, 4>(lds, a_el, a_sc, b_el, b_sc, k_tiles, ntm0, ntn0);
  else if (next_kind == 2) issue_prologue<C, S, DEEP, 2>(lds, a_el, a_sc, b_el, b_sc, k_tiles, ntm0, ntn0);
}

// Work lists.  The hardware deals workgroups round-robin to the 8 XCDs (workgroup c runs on XCD c % 8), each with its
// own L2.  Full tiles and half tiles are each put in band order (bands of kBand tile columns, row-major inside a band)
// and cut into one contiguous run per XCD, sized by the XCD's share of the workgroups; local workgroup j = c / 8 of an
// XCD with Px workgroups takes positions j, j + Px, ... of the run, so the 32 workgroups of an XCD work on 32 consecutive
// positions = an 8 x 4 block of tiles sharing 8 A panels and 4 B panels through that XCD's L2.  The workgroups of even
// XCDs start with one half tile and do their other half tiles last; those of odd XCDs do all their full tiles first: two
// phase groups whose output bursts do not coincide.
constexpr int kBand = 4;

__device__ __forceinline__ void band_decode(int p, int rows, int cols, int& r, int& c, int band_cols = kBand) {
  const int per_band = band_cols * rows;
  const int band = p / per_band, q = p - band * per_band;
  const int c0 = band * band_cols;
  const int w = cols - c0 < band_cols ? cols - c0 : band_cols;
  r = q / w;
  c = c0 + (q - r * w);
}

template <class C, int S, bool DEEP, bool OUT_BF16>
__global__ void __launch_bounds__(C::THREADS) gemm_kernel_dma(const uint8_t* __restrict__ a_el, const uint8_t* __restrict__ a_sc,
                                                              const uint8_t* __restrict__ b_el, const uint8_t* __restrict__ b_sc,
                                                              int64_t k_tiles, int64_t M, int64_t N, void* __restrict__ Dv,
                                                              int64_t ldd, int gm, int gnf, int nhc) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const int c = blockIdx.x, P = gridDim.x;
  const int F = gm * gnf, H = gm * nhc;
  const int x = c & 7, j = c >> 3;
  const int base = P >> 3, rem = P & 7;
  const int Px = base + (x < rem ? 1 : 0);                        // workgroups on this XCD
  const int cum0 = x * base + (x < rem ? x : rem), cum1 = cum0 + Px;
  const int f_begin = (int)((int64_t)F * cum0 / P), f_count = (int)((int64_t)F * cum1 / P) - f_begin;
  const int h_begin = (int)((int64_t)H * cum0 / P), h_count = (int)((int64_t)H * cum1 / P) - h_begin;
  const int jj = j;
  const int nf = jj < f_count ? (f_count - jj + Px - 1) / Px : 0;
  const int nh = jj < h_count ? (h_count - jj + Px - 1) / Px : 0;
  const bool lead_half = (x & 1) == 0 && nh > 0;
  // item `it` of this workgroup: kind (2 half, 4 full) and tile origin in units of 32 rows / columns
  auto item = [&](int it, int& kind, int64_t& tm0, int64_t& tn0) {
    if (it >= nf + nh) { kind = 0; tm0 = tn0 = 0; return; }
    bool half;
    int t;
    if (lead_half) {
      half = it == 0 || it > nf;
      t = it == 0 ? 0 : (it <= nf ? it - 1 : it - nf);
    } else {
      half = it >= nf;
      t = half ? it - nf : it;
    }
    int row, col;
    if (half) {
      band_decode(h_begin + jj + t * Px, gm, nhc, row, col);
      kind = 2; tm0 = (int64_t)row * 8; tn0 = (int64_t)gnf * 8 + col * 4;
    } else {
      band_decode(f_begin + jj + t * Px, gm, gnf, row, col);
      kind = 4; tm0 = (int64_t)row * 8; tn0 = (int64_t)col * 8;
    }
  };
  int kind, nkind;
  int64_t tm0, tn0, ntm0, ntn0;
  item(0, kind, tm0, tn0);
  if (kind == 4) issue_prologue<C, S, DEEP, 4>(lds, a_el, a_sc, b_el, b_sc, k_tiles, tm0, tn0);
  else if (kind == 2) issue_prologue<C, S, DEEP, 2>(lds, a_el, a_sc, b_el, b_sc, k_tiles, tm0, tn0);
  for (int it = 0; kind != 0; ++it) {
    item(it + 1, nkind, ntm0, ntn0);
    if (kind == 2) run_tile<C, S, DEEP, 2, OUT_BF16>(lds, a_el, a_sc, b_el, b_sc, k_tiles, M, N, Dv, ldd, tm0, tn0, nkind, ntm0, ntn0);
    else run_tile<C, S, DEEP, 4, OUT_BF16>(lds, a_el, a_sc, b_el, b_sc, k_tiles, M, N, Dv, ldd, tm0, tn0, nkind, ntm0, ntn0);
    kind = nkind; tm0 = ntm0; tn0 = ntn0;
  }
}

template <class C>
int launch_cfg(const uint8_t* Ai, const uint8_t* Bi, int64_t M, int64_t N, int64_t K, void* D, int d_dtype, int64_t ldd,
               hipStream_t s) {
  const ImageGeom ga = image_geom(M, K, C::AT), gb = image_geom(N, K, C::BT);
  const int64_t gm = (M + C::TM * 32 - 1) / (C::TM * 32), gn = (N + C::TN * 32 - 1) / (C::TN * 32);
  if (gm > 65535 || gn > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  dim3 grid((unsigned)gn, (unsigned)gm);
  const size_t lds = 2 * (size_t)C::STAGE_BYTES;
  if (d_dtype == MXP_BF16) {
    allow_dynamic_lds<&gemm_kernel<C, true>>((int)lds);
    hipLaunchKernelGGL((gemm_kernel<C, true>), grid, dim3(C::THREADS), lds, s, Ai, Ai + ga.elem_bytes, Bi, Bi + gb.elem_bytes,
                       ga.k_tiles, M, N, D, ldd);
  } else {
    allow_dynamic_lds<&gemm_kernel<C, false>>((int)lds);
    hipLaunchKernelGGL((gemm_kernel<C, false>), grid, dim3(C::THREADS), lds, s, Ai, Ai + ga.elem_bytes, Bi, Bi + gb.elem_bytes,
                       ga.k_tiles, M, N, D, ldd);
  }
  return launch_status();
}

// Tile list for the persistent kernel: gn tile columns of 256, of which the last `hc` are cut into two half columns.
// The longest per-workgroup list has ceil(F/P) full + ceil(H/P) half tiles; pick the hc with
// the smallest such makespan and, among equals, the smallest one that gives every workgroup a half tile (H >= P), so
// that the two phase groups exist; else no half tiles.
template <class C, int S>
int launch_dma(const uint8_t* Ai, const uint8_t* Bi, int64_t M, int64_t N, int64_t K, void* D, int d_dtype, int64_t ldd,
               hipStream_t s) {
  const ImageGeom ga = image_geom(M, K, C::AT), gb = image_geom(N, K, C::BT);
  const int64_t gm = (M + 255) / 256, gn = (N + 255) / 256;
  if (gm * gn * 2 > 2000000000LL) return MXP_ERR_UNSUPPORTED;
  // the copies address an 8-tile run of one operand with a 32-bit lane offset: 8 * k_tiles * tile bytes must fit
  if (ga.k_tiles > (int64_t)(0xFFFFFFFFu / (8u * kTileBytesE4M3))) return MXP_ERR_UNSUPPORTED;
  const int64_t total = gm * gn;
  const int P = (int)(2 * total < kNumCU ? 2 * total : kNumCU);   // workgroups: one per CU, fewer only if even half tiles run out
  int64_t best_hc = 0;
  double best = 1e300;
  bool best_phase = false;
  for (int64_t hc = 0; hc <= gn; ++hc) {
    const int64_t F = gm * (gn - hc), H = 2 * gm * hc;
    const double span = (double)((F + P - 1) / P) + 0.5 * (double)((H + P - 1) / P);
    const bool phase = H >= P && F >= P;
    if (span < best - 1e-9 || (span < best + 1e-9 && phase && !best_phase)) {
      best = span;
      best_hc = hc;
      best_phase = phase;
    }
  }
  const int gnf = (int)(gn - best_hc), nhc = (int)(2 * best_hc);
  dim3 grid((unsigned)P);
  // ring + one pair of epilogue patches per wavefront (which may start inside the last ring slot, see patch_base)
  constexpr size_t lds_patched = (size_t)patch_base<C, S>() + 4 * 2 * kPatchBytes, lds_ring = (size_t)S * C::STAGE_BYTES;
  constexpr size_t lds = lds_patched > lds_ring ? lds_patched : lds_ring;
  static_assert(lds <= 160 * 1024, "LDS ring exceeds the 160 KiB of a CDNA4 compute unit");
  // one tile per workgroup at most: the whole ring is kept in flight (see ring_depth)
  const int64_t Fq = gm * gnf, Hq = gm * nhc;
  const bool deep = (Fq + P - 1) / P + (Hq + P - 1) / P <= 1;
#define MXP_GO(DEEPV, BFV)                                                                                                         \
  do {                                                                                                                             \
    allow_dynamic_lds<&gemm_kernel_dma<C, S, DEEPV, BFV>>((int)lds);                                                       \
    hipLaunchKernelGGL((gemm_kernel_dma<C, S, DEEPV, BFV>), grid, dim3(C::THREADS), lds, s, Ai, Ai + ga.elem_bytes, Bi,           \
                       Bi + gb.elem_bytes, ga.k_tiles, M, N, D, ldd, (int)gm, gnf, nhc);                                           \
  } while (0)
  if (d_dtype == MXP_BF16) {
    if (deep) MXP_GO(true, true);
    else MXP_GO(false, true);
  } else {
    if (deep) MXP_GO(true, false);
    else MXP_GO(false, false);
  }
#undef MXP_GO
  return launch_status();
}

// ---- skinny-M kernel (decode: M <= 64) --------------------------------------------------------------------------
// With a handful of activation rows the product is bound by reading the weight image once (Sec. 7.2: the decode stage
// is memory-bound), so the aim is to have every byte of it requested at once.  A workgroup owns CT adjacent 32-column
// tiles of B and splits K over its wavefronts; a wavefront loads its k-tiles of B straight from the image into MFMA
// operand registers (a tile is 1536 contiguous bytes in lane order: no LDS staging needed), the row tiles of A
// likewise (A is tiny and stays in cache), runs the MFMAs, and the partial tiles are summed through LDS.
// Every workgroup re-reads all of A (padded to 32 rows per tile: as many bytes as one column tile of B), and the sum
// of both load streams is what the kernel is limited by (8.5 TB/s combined, measured with E2M3 and with E2M1
// weights); CT > 1 shares one A operand between CT column tiles, for shapes with enough column tiles to go round.
template <int TMR, int CT, bool OUT_BF16, int BT, int AT, int WAVES>
__global__ void __launch_bounds__(64 * WAVES) gemm_skinny_kernel(const uint8_t* __restrict__ a_el, const uint8_t* __restrict__ a_sc,
                                                                 const uint8_t* __restrict__ b_el, const uint8_t* __restrict__ b_sc,
                                                                 int k_tiles, int64_t M, int64_t N, void* __restrict__ Dv, int64_t ldd) {
  // k-tiles whose loads are in flight together per wavefront: as many as the register file allows (128 registers per
  // lane with 16 wavefronts, 256 with 8)
  constexpr int CHUNK = CT == 4 ? 3 : (CT == 2 && WAVES == 16 ? 2 : 4);
  static_assert(CT == 1 || CT == 2 || CT == 4, "column tiles of a workgroup share one scale dword");
  extern __shared__ __attribute__((aligned(16))) uint8_t skinny_lds[];
  float (*part)[TMR * CT][16][64] = reinterpret_cast<float (*)[TMR * CT][16][64]>(skinny_lds);   // [WAVES][TMR * CT][16][64]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t ct = (int64_t)blockIdx.x * CT;              // first column tile of B (32 columns each)
  constexpr int FB = BT == kTileBytes ? kFmtE2M3 : (BT == kTileBytesE4M3 ? kFmtE4M3 : kFmtE2M1);
  constexpr int FA = AT == kTileBytes ? kFmtE2M3 : (AT == kTileBytesE4M3 ? kFmtE4M3 : kFmtE2M1);
  const uint8_t* bt = b_el + ct * (int64_t)k_tiles * BT;
  const uint8_t* bs = b_sc + ((ct >> 2) * (int64_t)k_tiles) * 256 + lane * 4;
  const int b_shift = (int)(ct & 3) * 8;                    // byte j of the shifted dword = column tile ct + j
  v16f acc[TMR][CT];
#pragma unroll
  for (int i = 0; i < TMR; ++i)
#pragma unroll
    for (int j = 0; j < CT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // The runs of two workgroups lie a multiple of 4 KiB x k_tiles apart: walking them in step would have every workgroup
  // on the same memory channels at the same time.  Each workgroup therefore starts its walk over the chunks of K at a
  // different one (and wraps round).
  const int n_chunks = (k_tiles + CHUNK - 1) / CHUNK;
  const int first = (int)((blockIdx.x * 5u) % (uint32_t)n_chunks);
  for (int ci = wave; ci < n_chunks; ci += WAVES) {
    const int q = ci + first < n_chunks ? ci + first : ci + first - n_chunks;
    const int k0 = q * CHUNK;
    v8i b[CHUNK][CT], a[CHUNK][TMR];
    uint32_t sb[CHUNK], sa[CHUNK];
#pragma unroll
    for (int c = 0; c < CHUNK; ++c) {
      const int kt = k0 + c < k_tiles ? k0 + c : k_tiles - 1;     // clamped: the surplus is not used
#pragma unroll
      for (int j = 0; j < CT; ++j) {
        const uint8_t* t = bt + ((int64_t)j * k_tiles + kt) * BT;
        const u32x4 lo = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t + lane * 16));
        u32x4 hi = {0, 0, 0, 0};
        if (BT == kTileBytes) {
          const u32x2 h2 = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(t + 1024 + lane * 8));
          hi.x = h2.x;
          hi.y = h2.y;
        } else if (BT == kTileBytesE4M3) {
          hi = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t + 1024 + lane * 16));
        }
        b[c][j] = (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
      }
      sb[c] = *reinterpret_cast<const uint32_t*>(bs + (int64_t)kt * 256) >> b_shift;
      sa[c] = *reinterpret_cast<const uint32_t*>(a_sc + (int64_t)kt * 256 + lane * 4);
#pragma unroll
      for (int i = 0; i < TMR; ++i) {
        // lanes of rows past M would fetch the image's zero padding: leaving them out saves that part of the A stream
        // (with 8 rows, three quarters of it)
        const uint8_t* ta = a_el + ((int64_t)i * k_tiles + kt) * AT;
        u32x4 alo = {0, 0, 0, 0}, ahi = {0, 0, 0, 0};
        if (32 * i + (lane & 31) < M) {
          alo = *reinterpret_cast<const u32x4*>(ta + lane * 16);
          if (AT == kTileBytes) {
            const u32x2 h2 = *reinterpret_cast<const u32x2*>(ta + 1024 + lane * 8);
            ahi.x = h2.x;
            ahi.y = h2.y;
          } else if (AT == kTileBytesE4M3) {
            ahi = *reinterpret_cast<const u32x4*>(ta + 1024 + lane * 16);
          }
        }
        a[c][i] = (v8i){(int)alo.x, (int)alo.y, (int)alo.z, (int)alo.w, (int)ahi.x, (int)ahi.y, (int)ahi.z, (int)ahi.w};
      }
    }
#pragma unroll
    for (int c = 0; c < CHUNK; ++c) {
      if (k0 + c < k_tiles) {
#pragma unroll
        for (int i = 0; i < TMR; ++i)                         // row tile i: byte i of the lane's A scale dword
#pragma unroll
          for (int j = 0; j < CT; ++j)                        // column tile j: byte j of the shifted B scale dword
            switch (i * 4 + j) {
              case 0: acc[i][j] = mfma<0, 0, FB, FA>(a[c][i], b[c][j], acc[i][j], (int)sa[c], (int)sb[c]); break;
              case 1: acc[i][j] = mfma<0, 1, FB, FA>(a[c][i], b[c][j], acc[i][j], (int)sa[c], (int)sb[c]); break;
              case 2: acc[i][j] = mfma<0, 2, FB, FA>(a[c][i], b[c][j], acc[i][j], (int)sa[c], (int)sb[c]); break;
              case 3: acc[i][j] = mfma<0, 3, FB, FA>(a[c][i], b[c][j], acc[i][j], (int)sa[c], (int)sb[c]); break;
              case 4: acc[i][j] = mfma<1, 0, FB, FA>(a[c][i], b[c][j], acc[i][j], (int)sa[c], (int)sb[c]); break;
              case 5: acc[i][j] = mfma<1, 1, FB, FA>(a[c][i], b[c][j], acc[i][j], (int)sa[c], (int)sb[c]); break;
              case 6: acc[i][j] = mfma<1, 2, FB, FA>(a[c][i], b[c][j], acc[i][j], (int)sa[c], (int)sb[c]); break;
              case 7: acc[i][j] = mfma<1, 3, FB, FA>(a[c][i], b[c][j], acc[i][j], (int)sa[c], (int)sb[c]); break;
              case 8: acc[i][j] = mfma<2, 0, FB, FA>(a[c][i], b[c][j], acc[i][j], (int)sa[c], (int)sb[c]); break;
              case 9: acc[i][j] = mfma<2, 1, FB, FA>(a[c][i], b[c][j], acc[i][j], (int)sa[c], (int)sb[c]); break;
              case 12: acc[i][j] = mfma<3, 0, FB, FA>(a[c][i], b[c][j], acc[i][j], (int)sa[c], (int)sb[c]); break;
              default: acc[i][j] = mfma<3, 1, FB, FA>(a[c][i], b[c][j], acc[i][j], (int)sa[c], (int)sb[c]); break;
            }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < TMR; ++i)
#pragma unroll
    for (int j = 0; j < CT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) part[wave][i * CT + j][r][lane] = acc[i][j][r];
  __syncthreads();
  // all lanes of the workgroup sum the accumulator slots over the wavefronts; slot (i, j, r, l) is
  // D[32 i + (l % 32)][32 (ct + j) + 8 (r / 4) + 4 (l / 32) + r % 4]
  for (int e = tid; e < TMR * CT * 16 * 64; e += 64 * WAVES) {
    const int l = e & 63, r = (e >> 6) & 15, ij = e >> 10;
    const int i = ij / CT, j = ij % CT;
    float v = 0.0f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) v += part[w][ij][r][l];
    const int64_t row = 32 * i + (l & 31);
    const int64_t col = 32 * (ct + j) + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
    if (row < M && col < N) {
      if (OUT_BF16) static_cast<uint16_t*>(Dv)[row * ldd + col] = (uint16_t)f32_to_bf16_rne(v);
      else static_cast<float*>(Dv)[row * ldd + col] = v;
    }
  }
}

template <int TMR, int CT, bool OUT_BF16, int BT, int AT, int WAVES>
void launch_skinny_cfg(int64_t n_ct, hipStream_t s, const uint8_t* ae, const uint8_t* as, const uint8_t* be, const uint8_t* bs, int kt,
                       int64_t M, int64_t N, void* D, int64_t ldd) {
  constexpr int lds = WAVES * TMR * CT * 16 * 64 * 4;
  static_assert(lds <= 128 * 1024, "partial tiles must fit in LDS");
  allow_dynamic_lds<&gemm_skinny_kernel<TMR, CT, OUT_BF16, BT, AT, WAVES>>((int)lds);
  const dim3 grid((unsigned)((n_ct + CT - 1) / CT));
  hipLaunchKernelGGL((gemm_skinny_kernel<TMR, CT, OUT_BF16, BT, AT, WAVES>), grid, dim3(64 * WAVES), lds, s, ae, as, be, bs, kt, M, N, D, ldd);
}

template <int TMR, int CT, int BT, int AT, int WAVES>
void launch_skinny_out(bool bf, int64_t n_ct, hipStream_t s, const uint8_t* ae, const uint8_t* as, const uint8_t* be, const uint8_t* bs,
                       int kt, int64_t M, int64_t N, void* D, int64_t ldd) {
  if (bf) launch_skinny_cfg<TMR, CT, true, BT, AT, WAVES>(n_ct, s, ae, as, be, bs, kt, M, N, D, ldd);
  else launch_skinny_cfg<TMR, CT, false, BT, AT, WAVES>(n_ct, s, ae, as, be, bs, kt, M, N, D, ldd);
}

// Wavefronts per workgroup: 16 when K is long enough to give each at least one chunk (K >= 4096) and the partial
// tiles fit, so that the whole K range of a workgroup is requested at once.  Column tiles per workgroup: as many
// (4, 2, 1) as still leave about one workgroup per compute unit.
template <int BT, int AT>
int launch_skinny(const uint8_t* Ai, const uint8_t* Bi, int64_t M, int64_t N, int64_t K, void* D, int d_dtype, int64_t ldd,
                  hipStream_t s) {
  const ImageGeom ga = image_geom(M, K, AT), gb = image_geom(N, K, BT);
  const int64_t ct = (N + 31) / 32;
  if (ct > 2147483647LL || ga.k_tiles > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  const int kt = (int)ga.k_tiles;
  const uint8_t *ae = Ai, *as = Ai + ga.elem_bytes, *be = Bi, *bs = Bi + gb.elem_bytes;
  const bool bf = d_dtype == MXP_BF16, wide = kt >= 64;
  constexpr int64_t kEnough = 200;                          // workgroups
  constexpr bool kFp8Image = BT == kTileBytesE4M3 || AT == kTileBytesE4M3;
  if (M > 64) {                                             // 65 .. 128 rows: four row tiles, 8 wavefronts (128 KiB of partial tiles)
    if constexpr (kFp8Image) return MXP_ERR_UNSUPPORTED;    // (callers send E4M3 images here with up to 64 rows only)
    else launch_skinny_out<4, 1, BT, AT, 8>(bf, ct, s, ae, as, be, bs, kt, M, N, D, ldd);
  } else if (M <= 32) {
    if (ct / 4 >= kEnough) launch_skinny_out<1, 4, BT, AT, 8>(bf, ct, s, ae, as, be, bs, kt, M, N, D, ldd);
    else if (ct / 2 >= kEnough && wide) launch_skinny_out<1, 2, BT, AT, 16>(bf, ct, s, ae, as, be, bs, kt, M, N, D, ldd);
    else if (ct / 2 >= kEnough) launch_skinny_out<1, 2, BT, AT, 8>(bf, ct, s, ae, as, be, bs, kt, M, N, D, ldd);
    else if (wide) launch_skinny_out<1, 1, BT, AT, 16>(bf, ct, s, ae, as, be, bs, kt, M, N, D, ldd);
    else launch_skinny_out<1, 1, BT, AT, 8>(bf, ct, s, ae, as, be, bs, kt, M, N, D, ldd);
  } else {
    if (ct / 2 >= kEnough) launch_skinny_out<2, 2, BT, AT, 8>(bf, ct, s, ae, as, be, bs, kt, M, N, D, ldd);
    else if (wide && !kFp8Image) {                          // (E4M3 fragments: 16 wavefronts would spill)
      if constexpr (!kFp8Image) launch_skinny_out<2, 1, BT, AT, 16>(bf, ct, s, ae, as, be, bs, kt, M, N, D, ldd);
    } else launch_skinny_out<2, 1, BT, AT, 8>(bf, ct, s, ae, as, be, bs, kt, M, N, D, ldd);
  }
  return launch_status();
}

// ---- skinny-M kernel on MXFP4+ weights kept in 4-bit codes (E2M1 image + residual bytes) --------------------------
// The decode stage is bound by the weight bytes (Sec. 7.2), and the E2M3 image spends 6.25 bits on an element that
// canonical MXFP4+ stores in 4.5.  Here the weights stay 4-bit: the BM's nibble holds BM_H of Eq. 3 as an ordinary E2M1
// code, so the FP4 MFMA forms every product except a[k_BM] * BM_L, one per weight block and activation row -- the extra
// sparse product of Sec. 5.2.  BM_L = +-(m1 + m0 / 2) is itself an E2M1 number (code sign | 0 m1 m0), so the missing
// products are a second MFMA of the same activation tile with a weight tile that is zero except for that one nibble
// per block; in the MFMA operand order a lane holds exactly one weight block, so it builds its 16 bytes of that tile
// from the block's residual byte in registers (a shift and four selects) and nothing but the residual bytes is read
// from memory.  The matrix pipe has the time: the kernel waits for weight bytes.  Everything else as in
// gemm_skinny_kernel, whose launch shapes it shares.
// AT: the activation image's tile bytes -- E2M3, or E4M3 for MXFP4++ activations (Sec. 4.3; the MFMA takes an FP8 and an FP4 operand).
// XM: the image keeps the BM's nibble in place and its residual bytes are the canonical index bytes (position | delta << 5):
// MXFP4+ and MXFP4++ weights (Sec. 4.3).  The first MFMA then takes the 4-bit codes without the BM, scaled by the block's scale
// lowered by delta; the second takes the BM alone as an E2M3 code (sign | 11 | mmm, Sec. 4.2) with the block's own scale.
template <int TMR, int CT, bool OUT_BF16, int WAVES, int AT, bool XM>
__global__ void __launch_bounds__(64 * WAVES) gemm_skinny_res_kernel(const uint8_t* __restrict__ a_el, const uint8_t* __restrict__ a_sc,
                                                                     const uint8_t* __restrict__ b_el, const uint8_t* __restrict__ b_sc,
                                                                     const uint8_t* __restrict__ b_res, int k_tiles, int64_t M,
                                                                     int64_t N, void* __restrict__ Dv, int64_t ldd) {
  constexpr int BT = kTileBytesE2M1;
  constexpr int FA = AT == kTileBytes ? kFmtE2M3 : kFmtE4M3;
  static_assert(AT == kTileBytes || AT == kTileBytesE4M3, "activation image: E2M3 or E4M3");
  constexpr int CHUNK = CT == 4 ? 3 : (CT == 2 && WAVES == 16 ? 2 : 4);
  extern __shared__ __attribute__((aligned(16))) uint8_t skinny_lds[];
  float (*part)[TMR * CT][16][64] = reinterpret_cast<float (*)[TMR * CT][16][64]>(skinny_lds);   // [WAVES][TMR * CT][16][64]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t ct = (int64_t)blockIdx.x * CT;
  const uint8_t* bt = b_el + ct * (int64_t)k_tiles * BT;
  const uint8_t* bs = b_sc + ((ct >> 2) * (int64_t)k_tiles) * 256 + lane * 4;
  const uint8_t* br = b_res + ct * (int64_t)k_tiles * 64 + lane;
  const int b_shift = (int)(ct & 3) * 8;
  v16f acc[TMR][CT];
#pragma unroll
  for (int i = 0; i < TMR; ++i)
#pragma unroll
    for (int j = 0; j < CT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const int n_chunks = (k_tiles + CHUNK - 1) / CHUNK;
  const int first = (int)((blockIdx.x * 5u) % (uint32_t)n_chunks);
  for (int ci = wave; ci < n_chunks; ci += WAVES) {
    const int q = ci + first < n_chunks ? ci + first : ci + first - n_chunks;
    const int k0 = q * CHUNK;
    u32x4 b[CHUNK][CT];
    v8i a[CHUNK][TMR];
    uint32_t sb[CHUNK], sa[CHUNK], rs[CHUNK][CT];
#pragma unroll
    for (int c = 0; c < CHUNK; ++c) {
      const int kt = k0 + c < k_tiles ? k0 + c : k_tiles - 1;     // clamped: the surplus is not used
#pragma unroll
      for (int j = 0; j < CT; ++j) {
        b[c][j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(bt + ((int64_t)j * k_tiles + kt) * BT + lane * 16));
        rs[c][j] = __builtin_nontemporal_load(br + ((int64_t)j * k_tiles + kt) * 64);
      }
      sb[c] = *reinterpret_cast<const uint32_t*>(bs + (int64_t)kt * 256) >> b_shift;
      sa[c] = *reinterpret_cast<const uint32_t*>(a_sc + (int64_t)kt * 256 + lane * 4);
#pragma unroll
      for (int i = 0; i < TMR; ++i) {
        const uint8_t* ta = a_el + ((int64_t)i * k_tiles + kt) * AT;
        u32x4 alo = {0, 0, 0, 0}, ahi = {0, 0, 0, 0};
        if (32 * i + (lane & 31) < M) {
          alo = *reinterpret_cast<const u32x4*>(ta + lane * 16);
          if (AT == kTileBytes) {
            const u32x2 h2 = *reinterpret_cast<const u32x2*>(ta + 1024 + lane * 8);
            ahi.x = h2.x;
            ahi.y = h2.y;
          } else {
            ahi = *reinterpret_cast<const u32x4*>(ta + 1024 + lane * 16);
          }
        }
        a[c][i] = (v8i){(int)alo.x, (int)alo.y, (int)alo.z, (int)alo.w, (int)ahi.x, (int)ahi.y, (int)ahi.z, (int)ahi.w};
      }
    }
#pragma unroll
    for (int c = 0; c < CHUNK; ++c) {
      if (k0 + c < k_tiles) {
        uint32_t sbm = sb[c];                                   // XM: the scale bytes of the first MFMA, each lowered by its delta
        if (XM) {
#pragma unroll
          for (int j = 0; j < CT; ++j) sbm -= (rs[c][j] >> 5) << (8 * j);
        }
#pragma unroll
        for (int j = 0; j < CT; ++j) {
          const uint32_t r = rs[c][j];
          v8i bv, lv;
          if (!XM) {
            bv = (v8i){(int)b[c][j].x, (int)b[c][j].y, (int)b[c][j].z, (int)b[c][j].w, 0, 0, 0, 0};
            // the tile of BM_L codes: sign | 0 m1 m0 at the block's BM position, zeros elsewhere (no BM: residual byte 0)
            const uint32_t word = (((r >> 5) & 3u) | ((r >> 4) & 8u)) << (4u * (r & 7u));
            const uint32_t piece = (r >> 3) & 3u;
            lv = (v8i){(int)(piece == 0u ? word : 0u), (int)(piece == 1u ? word : 0u), (int)(piece == 2u ? word : 0u),
                       (int)(piece == 3u ? word : 0u), 0, 0, 0, 0};
          } else {
            const uint32_t sw = (sb[c] >> (8 * j)) & 255u;
            const bool live = sw != 0u && sw != 255u;             // all-zero, absent and NaN blocks have no BM
            const uint32_t idx = r & 31u, piece = idx >> 3, in8 = idx & 7u, sh4 = 4u * in8;
            uint32_t w[4] = {b[c][j].x, b[c][j].y, b[c][j].z, b[c][j].w};
            const uint32_t nib = ((piece == 0u ? w[0] : piece == 1u ? w[1] : piece == 2u ? w[2] : w[3]) >> sh4) & 15u;
            const uint32_t out4 = live ? nib << sh4 : 0u;         // xor takes the BM's nibble out of its dword
#pragma unroll
            for (int p4 = 0; p4 < 4; ++p4) w[p4] ^= piece == (uint32_t)p4 ? out4 : 0u;
            bv = (v8i){(int)w[0], (int)w[1], (int)w[2], (int)w[3], 0, 0, 0, 0};
            // the BM as an E2M3 code at element idx of a 32 x 6-bit string: 8 elements are 48 bits, so group `piece` starts at
            // bit 0 or 16 of dword 3 (piece / 2) and the code, shifted to its place in the group, spans at most two dwords
            const uint32_t code = live ? (((nib & 8u) << 2) | 0x18u | (nib & 7u)) : 0u;
            const uint64_t v48 = (uint64_t)code << (6u * in8);
            const uint32_t lo = (uint32_t)v48, hi = (uint32_t)(v48 >> 32);
            const bool odd = (piece & 1u) != 0u, upper = piece >= 2u;
            const uint32_t t0 = odd ? 0u : lo, t1 = odd ? lo << 16 : hi, t2 = odd ? __builtin_amdgcn_alignbit(hi, lo, 16) : 0u;
            const uint32_t e[6] = {upper ? 0u : t0, upper ? 0u : t1, upper ? 0u : t2, upper ? t0 : 0u, upper ? t1 : 0u, upper ? t2 : 0u};
            lv = (v8i){(int)e[0], (int)e[1], (int)e[2], (int)e[3], (int)e[4], (int)e[5], 0, 0};
          }
          constexpr int FL = XM ? kFmtE2M3 : kFmtE2M1;
#pragma unroll
          for (int i = 0; i < TMR; ++i)
            switch (i * 4 + j) {
#define MXP_RES_MFMA(I, J)                                                                                        \
  acc[i][j] = mfma<I, J, kFmtE2M1, FA>(a[c][i], bv, acc[i][j], (int)sa[c], (int)sbm);                             \
  acc[i][j] = mfma<I, J, FL, FA>(a[c][i], lv, acc[i][j], (int)sa[c], (int)sb[c]);                                 \
  break
              case 0: MXP_RES_MFMA(0, 0);
              case 1: MXP_RES_MFMA(0, 1);
              case 2: MXP_RES_MFMA(0, 2);
              case 3: MXP_RES_MFMA(0, 3);
              case 4: MXP_RES_MFMA(1, 0);
              case 5: MXP_RES_MFMA(1, 1);
              case 6: MXP_RES_MFMA(1, 2);
              case 7: MXP_RES_MFMA(1, 3);
              case 8: MXP_RES_MFMA(2, 0);
              case 9: MXP_RES_MFMA(2, 1);
              case 12: MXP_RES_MFMA(3, 0);
              default: MXP_RES_MFMA(3, 1);
#undef MXP_RES_MFMA
            }
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < TMR; ++i)
#pragma unroll
    for (int j = 0; j < CT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) part[wave][i * CT + j][r][lane] = acc[i][j][r];
  __syncthreads();
  for (int e = tid; e < TMR * CT * 16 * 64; e += 64 * WAVES) {
    const int l = e & 63, r = (e >> 6) & 15, ij = e >> 10;
    const int i = ij / CT, j = ij % CT;
    float v = 0.0f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) v += part[w][ij][r][l];
    const int64_t row = 32 * i + (l & 31);
    const int64_t col = 32 * (ct + j) + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
    if (row < M && col < N) {
      if (OUT_BF16) static_cast<uint16_t*>(Dv)[row * ldd + col] = (uint16_t)f32_to_bf16_rne(v);
      else static_cast<float*>(Dv)[row * ldd + col] = v;
    }
  }
}

template <int TMR, int CT, int WAVES, int AT, bool XM>
void launch_skinny_res_cfg(bool bf, int64_t n_ct, hipStream_t s, const uint8_t* ae, const uint8_t* as, const uint8_t* be,
                           const uint8_t* bs, const uint8_t* br, int kt, int64_t M, int64_t N, void* D, int64_t ldd) {
  constexpr int lds = WAVES * TMR * CT * 16 * 64 * 4;
  static_assert(lds <= 128 * 1024, "partial tiles must fit in LDS");
  const dim3 grid((unsigned)((n_ct + CT - 1) / CT));
  if (bf) {
    allow_dynamic_lds<&gemm_skinny_res_kernel<TMR, CT, true, WAVES, AT, XM>>((int)lds);
    hipLaunchKernelGGL((gemm_skinny_res_kernel<TMR, CT, true, WAVES, AT, XM>), grid, dim3(64 * WAVES), lds, s, ae, as, be, bs, br, kt, M, N, D, ldd);
  } else {
    allow_dynamic_lds<&gemm_skinny_res_kernel<TMR, CT, false, WAVES, AT, XM>>((int)lds);
    hipLaunchKernelGGL((gemm_skinny_res_kernel<TMR, CT, false, WAVES, AT, XM>), grid, dim3(64 * WAVES), lds, s, ae, as, be, bs, br, kt, M, N, D, ldd);
  }
}

// Launch shapes: those of launch_skinny (the entry points admit up to 64 rows).
template <int AT, bool XM>
int launch_skinny_res(const uint8_t* Ai, const uint8_t* Bi, int64_t M, int64_t N, int64_t K, void* D, int d_dtype, int64_t ldd,
                      hipStream_t s) {
  const ImageGeom ga = image_geom(M, K, AT), gb = image_geom(N, K, kTileBytesE2M1);
  const int64_t ct = (N + 31) / 32;
  if (ct > 2147483647LL || ga.k_tiles > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  const int kt = (int)ga.k_tiles;
  const uint8_t *ae = Ai, *as = Ai + ga.elem_bytes, *be = Bi, *bs = Bi + gb.elem_bytes, *br = bs + gb.scale_bytes;
  const bool bf = d_dtype == MXP_BF16, wide = kt >= 64;
  constexpr int64_t kEnough = 200;                          // workgroups
#define MXP_RES(TMR, CT, W) launch_skinny_res_cfg<TMR, CT, W, AT, XM>(bf, ct, s, ae, as, be, bs, br, kt, M, N, D, ldd)
  if (M <= 32) {
    if (ct / 4 >= kEnough) MXP_RES(1, 4, 8);
    else if (ct / 2 >= kEnough && wide) MXP_RES(1, 2, 16);
    else if (ct / 2 >= kEnough) MXP_RES(1, 2, 8);
    else if (wide) MXP_RES(1, 1, 16);
    else MXP_RES(1, 1, 8);
  } else {
    if (ct / 2 >= kEnough) MXP_RES(2, 2, 8);
    else if (wide && AT != kTileBytesE4M3) {                    // (E4M3 fragments: 16 wavefronts would spill)
      if constexpr (AT != kTileBytesE4M3) MXP_RES(2, 1, 16);
    } else MXP_RES(2, 1, 8);
  }
#undef MXP_RES
  return launch_status();
}

// ---- few rows against few weight rows: 16-column tiles ----------------------------------------------------------
// A layer with N = 4096 has only 128 column tiles of 32 -- half the compute units would read weights, and a compute unit
// draws about 27 GB/s whatever is in flight, so the product would run at half the HBM rate.  With up to 16 activation
// rows the 16x16x128 form of the block-scaled MFMA gives twice the workgroups from the same images: a workgroup owns 16
// weight rows (one half of a 32-row image tile), lane l supplies weight row l % 16 and K-block l / 16 of a 128-wide
// step (= the two K-blocks of two consecutive image k-tiles), and the two halves of a tile read disjoint 256-byte runs
// of it.  The activations come from rows 0..15 of their image's first row tile the same way.  The B tile goes in as the
// MFMA's first operand: accumulator register r of lane l is D[m = l % 16][n = 16 c + 4 (l / 16) + r].  K is split over
// the wavefronts and summed through LDS in a fixed order, as in gemm_skinny_kernel.  RES: 4-bit MXFP4+ weights with
// residual bytes (image kind E2M1R): BM_H in the FP4 operand, BM_L by a second MFMA (Eq. 3, Sec. 5.2).
typedef float v4f __attribute__((ext_vector_type(4)));

template <bool OUT_BF16, int BT, bool RES, int WAVES, int CHUNK>
__global__ void __launch_bounds__(64 * WAVES) gemm_skinny16_kernel(const uint8_t* __restrict__ a_el, const uint8_t* __restrict__ a_sc,
                                                                   const uint8_t* __restrict__ b_el, const uint8_t* __restrict__ b_sc,
                                                                   const uint8_t* __restrict__ b_res, int k_tiles, int64_t M,
                                                                   int64_t N, void* __restrict__ Dv, int64_t ldd) {
  static_assert(BT == kTileBytes || BT == kTileBytesE2M1, "weight image: E2M3 or E2M1");
  static_assert(!RES || BT == kTileBytesE2M1, "residual bytes go with 4-bit codes");
  constexpr int AT = kTileBytes;
  constexpr int FB = BT == kTileBytes ? kFmtE2M3 : kFmtE2M1;
  __shared__ float part[WAVES][4][64];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t c16 = blockIdx.x, T = c16 >> 1;              // 16-column tile, image row tile
  const int row16 = lane & 15, kq = lane >> 4;               // weight row in the tile, K-block of the 128-wide step
  const int slot_b = (kq & 1) * 32 + (int)(c16 & 1) * 16 + row16, slot_a = (kq & 1) * 32 + row16;
  const int kt_in_pair = kq >> 1;
  const uint8_t* bt = b_el + T * (int64_t)k_tiles * BT + slot_b * 16;
  const uint8_t* bth = b_el + T * (int64_t)k_tiles * BT + 1024 + slot_b * 8;
  const uint8_t* bs = b_sc + ((T >> 2) * (int64_t)k_tiles) * 256 + slot_b * 4;
  const uint8_t* br = RES ? b_res + T * (int64_t)k_tiles * 64 + slot_b : nullptr;
  const int b_shift = (int)(T & 3) * 8;
  const bool a_row = row16 < M;
  v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};

  const int n_pairs = k_tiles >> 1;                          // images are padded to K % 128 == 0: k_tiles is even
  const int n_chunks = (n_pairs + CHUNK - 1) / CHUNK;
  const int first = (int)((blockIdx.x * 5u) % (uint32_t)n_chunks);   // (workgroups start their walk at different chunks)
  for (int ci = wave; ci < n_chunks; ci += WAVES) {
    const int q = ci + first < n_chunks ? ci + first : ci + first - n_chunks;
    const int p0 = q * CHUNK;
    v8i b[CHUNK], a[CHUNK];
    uint32_t sb[CHUNK], sa[CHUNK], rs[CHUNK];
#pragma unroll
    for (int c = 0; c < CHUNK; ++c) {
      const int pr = p0 + c < n_pairs ? p0 + c : n_pairs - 1;       // clamped: the surplus is not used
      const int64_t kt = 2 * pr + kt_in_pair;
      const u32x4 lo = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(bt + kt * BT));
      u32x2 hi = {0, 0};
      if (BT == kTileBytes) hi = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(bth + kt * BT));
      b[c] = (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, 0, 0};
      rs[c] = RES ? (uint32_t)__builtin_nontemporal_load(br + kt * 64) : 0u;
      sb[c] = *reinterpret_cast<const uint32_t*>(bs + kt * 256) >> b_shift;
      sa[c] = *reinterpret_cast<const uint32_t*>(a_sc + kt * 256 + slot_a * 4);
      u32x4 alo = {0, 0, 0, 0};
      u32x2 ahi = {0, 0};
      if (a_row) {                                             // rows past M are the image's zero padding: not fetched
        alo = *reinterpret_cast<const u32x4*>(a_el + kt * AT + slot_a * 16);
        ahi = *reinterpret_cast<const u32x2*>(a_el + kt * AT + 1024 + slot_a * 8);
      }
      a[c] = (v8i){(int)alo.x, (int)alo.y, (int)alo.z, (int)alo.w, (int)ahi.x, (int)ahi.y, 0, 0};
    }
#pragma unroll
    for (int c = 0; c < CHUNK; ++c) {
      if (p0 + c < n_pairs) {
        acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b[c], a[c], acc, FB, kFmtE2M3, 0, (int)sb[c], 0, (int)sa[c]);
        if (RES) {
          // the tile of BM_L codes: sign | 0 m1 m0 at the block's BM position, zeros elsewhere (no BM: residual byte 0)
          const uint32_t r = rs[c];
          const uint32_t word = (((r >> 5) & 3u) | ((r >> 4) & 8u)) << (4u * (r & 7u));
          const uint32_t piece = (r >> 3) & 3u;
          const v8i lv = (v8i){(int)(piece == 0u ? word : 0u), (int)(piece == 1u ? word : 0u), (int)(piece == 2u ? word : 0u),
                               (int)(piece == 3u ? word : 0u), 0, 0, 0, 0};
          acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(lv, a[c], acc, kFmtE2M1, kFmtE2M3, 0, (int)sb[c], 0, (int)sa[c]);
        }
      }
    }
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) part[wave][r][lane] = acc[r];
  __syncthreads();
  if (tid < 256) {
    const int l = tid & 63, r = tid >> 6;
    float v = 0.0f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) v += part[w][r][l];
    const int64_t row = l & 15, col = 16 * c16 + 4 * (l >> 4) + r;
    if (row < M && col < N) {
      if (OUT_BF16) static_cast<uint16_t*>(Dv)[row * ldd + col] = (uint16_t)f32_to_bf16_rne(v);
      else static_cast<float*>(Dv)[row * ldd + col] = v;
    }
  }
}

// Takes M <= 16 when the 32-column kernels would launch fewer than one workgroup per compute unit.
inline bool skinny16_applies(int64_t M, int64_t N) { return M <= 16 && (N + 31) / 32 < kNumCU; }

template <int BT, bool RES>
int launch_skinny16(const uint8_t* Ai, const uint8_t* Bi, int64_t M, int64_t N, int64_t K, void* D, int d_dtype, int64_t ldd,
                    hipStream_t s) {
  const ImageGeom ga = image_geom(M, K, kTileBytes), gb = image_geom(N, K, BT);
  if (ga.k_tiles > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  const int kt = (int)ga.k_tiles;
  const uint8_t *ae = Ai, *as = Ai + ga.elem_bytes, *be = Bi, *bs = Bi + gb.elem_bytes, *br = bs + gb.scale_bytes;
  const dim3 grid((unsigned)((N + 15) / 16)), block(64 * 16);
  const bool bf = d_dtype == MXP_BF16;
  const int n_pairs = kt / 2;
#define MXP_S16(CH)                                                                                                               \
  do {                                                                                                                            \
    if (bf) hipLaunchKernelGGL((gemm_skinny16_kernel<true, BT, RES, 16, CH>), grid, block, 0, s, ae, as, be, bs, br, kt, M, N, D, ldd); \
    else hipLaunchKernelGGL((gemm_skinny16_kernel<false, BT, RES, 16, CH>), grid, block, 0, s, ae, as, be, bs, br, kt, M, N, D, ldd);   \
  } while (0)
  // k-steps in flight per wavefront: as many as give every one of the 16 wavefronts a chunk, at most 7 (128 registers per lane)
  if (n_pairs > 64) MXP_S16(7);
  else if (n_pairs == 64) MXP_S16(4);
  else if (n_pairs >= 32) MXP_S16(2);
  else MXP_S16(1);
#undef MXP_S16
  return launch_status();
}

// ---- block kernel with K split inside the workgroup (shapes with too few 256-wide tiles to fill the chip) ----------
// A shape like 2048 x 1024 gives the persistent kernel 64 half tiles for 256 compute units, and what one compute unit
// can draw from the L2 (about 100 GB/s) then sets the time: its 1.2 MB of operand panels.  Here a workgroup owns a
// 32 TMR x 32 CT block of the output (128 x 64: 256 workgroups for that shape, 0.6 MB of panels each) and its four
// wavefronts split K in interleaved chunks: every wavefront holds the whole block in its accumulators, loads its k-tiles
// of both operands straight from the images into MFMA operand registers (a tile is contiguous and in lane order: no
// LDS staging, no barrier in the loop, no operand fetched twice by a workgroup), two chunks in flight, and the four
// partial blocks are added through LDS in a fixed order.  The partial blocks lie in LDS as rows of the output (padded
// by 16 bytes against bank conflicts), so the summing pass reads and stores 16-byte pieces of full 128- or 256-byte rows.
// Two chunks of two k-tiles per wavefront in flight (147 KB per compute unit) are enough: with three the launch got slower.
// A 128 x 128 block (for shapes that would need a second round of 128 x 64 blocks) fills all 256 AGPRs of a wavefront
// and keeps two single k-tiles in flight.
// Workgroups are dealt to the XCDs like the persistent kernel's tiles, in bands of 8 block columns: 32 consecutive positions
// = 4 x 8 output blocks per XCD, i.e. 4 row panels and 8 (half as large) column panels, which its L2 then fetches once.
template <int TMR_, int CT_, int BT_, int AT_>
struct BlockCfg {
  static constexpr int WM = TMR_, WN = CT_;
  static constexpr int FB = BT_ == kTileBytes ? kFmtE2M3 : (BT_ == kTileBytesE4M3 ? kFmtE4M3 : kFmtE2M1);
  static constexpr int FA = AT_ == kTileBytes ? kFmtE2M3 : (AT_ == kTileBytesE4M3 ? kFmtE4M3 : kFmtE2M1);
};

// One lane's operand registers of a tile in global memory: 16 (E2M1), 24 (E2M3) or 32 (E4M3) bytes
template <int TB>
__device__ __forceinline__ v8i load_tile_global(const uint8_t* tile, int lane) {
  const u32x4 lo = *reinterpret_cast<const u32x4*>(tile + lane * 16);
  u32x4 hi = {0, 0, 0, 0};
  if (TB == kTileBytes) {
    const u32x2 h2 = *reinterpret_cast<const u32x2*>(tile + 1024 + lane * 8);
    hi.x = h2.x;
    hi.y = h2.y;
  } else if (TB == kTileBytesE4M3) {
    hi = *reinterpret_cast<const u32x4*>(tile + 1024 + lane * 16);
  }
  return (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
}

template <int TMR, int CT, bool OUT_BF16, int BT, int AT>
__global__ void __launch_bounds__(256) gemm_block_kernel(const uint8_t* __restrict__ a_el, const uint8_t* __restrict__ a_sc,
                                                         const uint8_t* __restrict__ b_el, const uint8_t* __restrict__ b_sc,
                                                         int k_tiles, int64_t M, int64_t N, void* __restrict__ Dv, int64_t ldd,
                                                         int n_rg, int n_cg) {
  static_assert((TMR == 2 || TMR == 4) && (CT == 2 || (CT == 4 && TMR == 4)), "blocks of 64 x 64, 128 x 64 or 128 x 128");
  using C = BlockCfg<TMR, CT, BT, AT>;
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  constexpr bool BIG = TMR * CT == 16;                                      // 128 x 128: the accumulators fill the AGPRs
  constexpr int WAVES = 4, CHUNK = BIG ? 1 : 2, NBUF = 2;                   // (a third k-tile in flight: 3 - 5 % slower)
  constexpr int ROWS = 32 * TMR, COLS = 32 * CT, STRIDE = COLS + 4;        // floats per row of a partial block
  extern __shared__ __attribute__((aligned(16))) uint8_t block_lds[];
  float* part = reinterpret_cast<float*>(block_lds);                        // [WAVES][ROWS][STRIDE]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // this workgroup's block: position in band order, one contiguous run of positions per XCD
  const int T = n_rg * n_cg, c = blockIdx.x;
  const int x = c & 7, j = c >> 3, base = T >> 3, rem = T & 7;
  int rg, cg;
  band_decode(x * base + (x < rem ? x : rem) + j, n_rg, n_cg, rg, cg, 8);
  const int64_t rt0 = (int64_t)rg * TMR, ct0 = (int64_t)cg * CT;           // first row tile of A, first column tile of B
  const uint8_t* at = a_el + rt0 * k_tiles * AT;
  const uint8_t* bt = b_el + ct0 * k_tiles * BT;
  const uint8_t* as = a_sc + ((rt0 >> 2) * k_tiles) * 256 + lane * 4;
  const uint8_t* bs = b_sc + ((ct0 >> 2) * k_tiles) * 256 + lane * 4;
  const int a_shift = (int)(rt0 & 3) * 8, b_shift = (int)(ct0 & 3) * 8;    // byte i of the shifted dword = tile i of the block

  v16f acc[TMR][CT];
#pragma unroll
  for (int i = 0; i < TMR; ++i)
#pragma unroll
    for (int jj = 0; jj < CT; ++jj)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][jj][r] = 0.0f;

  auto load_chunk = [&](int q, v8i (&a)[CHUNK][TMR], v8i (&b)[CHUNK][CT], uint32_t (&sa)[CHUNK][1], uint32_t (&sb)[CHUNK][1]) {
#pragma unroll
    for (int cc = 0; cc < CHUNK; ++cc) {
      const int kt = q * CHUNK + cc < k_tiles ? q * CHUNK + cc : k_tiles - 1;   // clamped: the surplus is not used
#pragma unroll
      for (int i = 0; i < TMR; ++i) a[cc][i] = load_tile_global<AT>(at + ((int64_t)i * k_tiles + kt) * AT, lane);
#pragma unroll
      for (int jj = 0; jj < CT; ++jj) b[cc][jj] = load_tile_global<BT>(bt + ((int64_t)jj * k_tiles + kt) * BT, lane);
      sa[cc][0] = *reinterpret_cast<const uint32_t*>(as + (int64_t)kt * 256) >> a_shift;
      sb[cc][0] = *reinterpret_cast<const uint32_t*>(bs + (int64_t)kt * 256) >> b_shift;
    }
  };
  auto mma_chunk = [&](int q, const v8i (&a)[CHUNK][TMR], const v8i (&b)[CHUNK][CT], const uint32_t (&sa)[CHUNK][1],
                       const uint32_t (&sb)[CHUNK][1]) {
#pragma unroll
    for (int cc = 0; cc < CHUNK; ++cc)
      if (q * CHUNK + cc < k_tiles) mma_all<C>(acc, a[cc], b[cc], sa[cc], sb[cc]);
  };
  const int n_chunks = (k_tiles + CHUNK - 1) / CHUNK;
  // NBUF chunks of this wavefront in flight: buffer n % NBUF holds its n-th chunk
  v8i a[NBUF][CHUNK][TMR], b[NBUF][CHUNK][CT];
  uint32_t sa[NBUF][CHUNK][1], sb[NBUF][CHUNK][1];
#pragma unroll
  for (int n = 0; n < NBUF - 1; ++n)
    if (wave + n * WAVES < n_chunks) load_chunk(wave + n * WAVES, a[n], b[n], sa[n], sb[n]);
  for (int q = wave; q < n_chunks; q += NBUF * WAVES) {
#pragma unroll
    for (int n = 0; n < NBUF; ++n) {
      const int qn = q + n * WAVES;                                         // chunk in buffer n
      if (qn < n_chunks) {
        constexpr int ahead = NBUF - 1;
        if (qn + ahead * WAVES < n_chunks) load_chunk(qn + ahead * WAVES, a[(n + ahead) % NBUF], b[(n + ahead) % NBUF], sa[(n + ahead) % NBUF], sb[(n + ahead) % NBUF]);
        mma_chunk(qn, a[n], b[n], sa[n], sb[n]);
      }
    }
  }
  // A 128 x 128 block has four partial blocks of 64 KiB, more than LDS holds: wavefronts 2 and 3 first hand theirs to
  // wavefronts 0 and 1 in the accumulators' own layout (lane-contiguous 16-byte pieces, no transposition), which add them
  // to their own; the two sums then go through the row layout like the four partials of the smaller blocks.
  constexpr int PARTS = BIG ? 2 : WAVES;                                    // partial blocks in the row layout
  if constexpr (BIG) {
    f32x4* stage = reinterpret_cast<f32x4*>(block_lds) + (size_t)(wave & 1) * (TMR * CT * 4 * 64) + lane;
    if (wave >= 2) {
#pragma unroll
      for (int i = 0; i < TMR; ++i)
#pragma unroll
        for (int jj = 0; jj < CT; ++jj)
#pragma unroll
          for (int g = 0; g < 4; ++g)
            stage[((i * CT + jj) * 4 + g) * 64] = (f32x4){acc[i][jj][4 * g], acc[i][jj][4 * g + 1], acc[i][jj][4 * g + 2], acc[i][jj][4 * g + 3]};
    }
    __syncthreads();
    if (wave < 2) {
#pragma unroll
      for (int i = 0; i < TMR; ++i)
#pragma unroll
        for (int jj = 0; jj < CT; ++jj)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const f32x4 o = stage[((i * CT + jj) * 4 + g) * 64];
            acc[i][jj][4 * g] += o[0]; acc[i][jj][4 * g + 1] += o[1]; acc[i][jj][4 * g + 2] += o[2]; acc[i][jj][4 * g + 3] += o[3];
          }
    }
    __syncthreads();                                                        // the staging area is read: it becomes the row layout
  }
  // partial blocks to LDS as output rows: accumulator quad g of lane l is row l % 32, columns 8 g + 4 (l / 32) .. + 3 of its tile
  if (wave < PARTS) {
    float* mine = part + (size_t)wave * ROWS * STRIDE;
#pragma unroll
    for (int i = 0; i < TMR; ++i)
#pragma unroll
      for (int jj = 0; jj < CT; ++jj)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 q4 = {acc[i][jj][4 * g], acc[i][jj][4 * g + 1], acc[i][jj][4 * g + 2], acc[i][jj][4 * g + 3]};
          *reinterpret_cast<f32x4*>(mine + (32 * i + (lane & 31)) * STRIDE + 32 * jj + 8 * g + 4 * (lane >> 5)) = q4;
        }
  }
  __syncthreads();
  const bool vec_ok = (ldd % 4 == 0) && ((reinterpret_cast<uintptr_t>(Dv) & 15u) == 0);
  constexpr int QUADS = COLS / 4;                                           // 16-byte pieces per row
  for (int e = tid; e < ROWS * QUADS; e += 256) {
    const int r = e / QUADS, q = e % QUADS;
    f32x4 v = *reinterpret_cast<const f32x4*>(part + r * STRIDE + 4 * q);
#pragma unroll
    for (int w = 1; w < PARTS; ++w) v += *reinterpret_cast<const f32x4*>(part + ((size_t)w * ROWS + r) * STRIDE + 4 * q);
    const int64_t row = rt0 * 32 + r, col = ct0 * 32 + 4 * q;
    if (row >= M || col >= N) continue;
    if (vec_ok && col + 3 < N) {
      if (OUT_BF16) {
        const u32x2 o = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
        __builtin_nontemporal_store(o, reinterpret_cast<u32x2*>(static_cast<uint16_t*>(Dv) + row * ldd + col));
      } else {
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(static_cast<float*>(Dv) + row * ldd + col));
      }
    } else {
#pragma unroll
      for (int t = 0; t < 4; ++t)
        if (col + t < N) {
          if (OUT_BF16) static_cast<uint16_t*>(Dv)[row * ldd + col + t] = (uint16_t)f32_to_bf16_rne(v[t]);
          else static_cast<float*>(Dv)[row * ldd + col + t] = v[t];
        }
    }
  }
}

// Which shapes take the block kernel: more rows than the few-row kernels take, and one round of workgroups on the chip's
// compute units with blocks of 128 x 128 at most.  Measured against the persistent kernel at K = 4096: 128 x 64 blocks in
// one round (2048 x 1024, 512 x 4096, 1024 x 2048) 11 - 13 us against 24; shapes of twice that size (1024 x 4096,
// 2048 x 2048, 512 x 8192) 22 - 23 us in two rounds of 128 x 64 blocks against 24.5, and in one round of 128 x 128 blocks
// as launched now; four rounds of 128 x 64 (2048 x 4096) 44 us and two rounds of 128 x 128 blocks 40 - 41 us against 29 --
// there every compute unit already has a half tile of its own.  Blocks are 64 x 64 when 128 x 64 ones would leave more
// than half of the chip idle.
inline bool block_kernel_applies(int64_t M, int64_t N) {
  return M > 128 && ((M + 127) / 128) * ((N + 127) / 128) <= kNumCU;
}

template <int BT, int AT>
int launch_block(const uint8_t* Ai, const uint8_t* Bi, int64_t M, int64_t N, int64_t K, void* D, int d_dtype, int64_t ldd,
                 hipStream_t s) {
  const ImageGeom ga = image_geom(M, K, AT), gb = image_geom(N, K, BT);
  if (ga.k_tiles > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  const int kt = (int)ga.k_tiles;
  const uint8_t *ae = Ai, *as = Ai + ga.elem_bytes, *be = Bi, *bs = Bi + gb.elem_bytes;
  const bool bf = d_dtype == MXP_BF16;
  const int64_t rg128 = (M + 127) / 128, cg64 = (N + 63) / 64;
  const bool big = rg128 * cg64 > kNumCU;                                    // 128 x 64 blocks would need a second round
  const bool tall = rg128 * cg64 >= kNumCU / 2;
  const int64_t n_cg = big ? (N + 127) / 128 : cg64;
  const int64_t n_rg = (big || tall) ? rg128 : (M + 63) / 64;
#define MXP_BLOCK(TMRV, CTV, BFV)                                                                                                 \
  do {                                                                                                                            \
    constexpr int rows_l = (CTV == 4 ? 2 : 4) * 32 * TMRV * (32 * CTV + 4) * 4, stage_l = CTV == 4 ? 2 * 16 * 4 * 64 * 16 : 0;    \
    constexpr int lds = rows_l > stage_l ? rows_l : stage_l;                                                                      \
    static_assert(lds <= 160 * 1024, "partial blocks must fit in LDS");                                                           \
    allow_dynamic_lds<&gemm_block_kernel<TMRV, CTV, BFV, BT, AT>>((int)lds);                                                    \
    hipLaunchKernelGGL((gemm_block_kernel<TMRV, CTV, BFV, BT, AT>), dim3((unsigned)(n_rg * n_cg)), dim3(256), lds, s, ae, as, be, \
                       bs, kt, M, N, D, ldd, (int)n_rg, (int)n_cg);                                                               \
  } while (0)
  if (big) {
    if (bf) MXP_BLOCK(4, 4, true);
    else MXP_BLOCK(4, 4, false);
  } else if (tall) {
    if (bf) MXP_BLOCK(4, 2, true);
    else MXP_BLOCK(4, 2, false);
  } else {
    if (bf) MXP_BLOCK(2, 2, true);
    else MXP_BLOCK(2, 2, false);
  }
#undef MXP_BLOCK
  return launch_status();
}

// ---- skinny-M kernel on canonical weights -----------------------------------------------------------------------
// The decode stage is bound by the weight bytes (Sec. 7.2).  This kernel reads the canonical arrays as they are: per
// chunk of 4 k-tiles a wavefront loads, for each of its column tiles, 32 rows x 128 contiguous bytes (8 blocks per row:
// full lines) and passes them through a private LDS patch into operand order (lane l gets the block of row l % 32,
// half l / 32); scale and index bytes come as one 8-byte load per row.  The 4-bit codes are the FP4 MFMA's operand;
// an MXFP4+ block gets the BM split of Eq. 3 in registers (BM_H in place, BM_L in a second MFMA), as in
// gemm_skinny_res_kernel.  Everything else -- A from its image, K split over the wavefronts, rotated walk, reduction
// through LDS -- as above.
constexpr int kCanonPatchStride = 144;                        // bytes per patch row: 128 + 16 against bank conflicts
constexpr int kCanonPatchBytes = 32 * kCanonPatchStride;

template <int TMR, int CT, bool OUT_BF16, bool PLUS, int AT, int WAVES>
__global__ void __launch_bounds__(64 * WAVES) gemm_skinny_canon_kernel(const uint8_t* __restrict__ a_el, const uint8_t* __restrict__ a_sc,
                                                                       const u32x4* __restrict__ w_el, const uint8_t* __restrict__ w_sc,
                                                                       const uint8_t* __restrict__ w_ix, int64_t nbk, int k_tiles,
                                                                       int64_t M, int64_t N, void* __restrict__ Dv, int64_t ldd) {
  constexpr int CHUNK = 4;                                    // k-tiles per chunk = 8 blocks = 128 bytes of a weight row
  extern __shared__ __attribute__((aligned(16))) uint8_t skinny_lds[];
  float (*part)[TMR * CT][16][64] = reinterpret_cast<float (*)[TMR * CT][16][64]>(skinny_lds);   // after the K loop
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  uint8_t* patch = skinny_lds + wave * kCanonPatchBytes;      // during the K loop
  const int64_t ct = (int64_t)blockIdx.x * CT;
  constexpr int FB = kFmtE2M1, FA = AT == kTileBytes ? kFmtE2M3 : kFmtE2M1;
  const int n_in = lane & 31, h = lane >> 5;                  // operand role of this lane: row of the tile, half of the k-tile
  const int ld_row = lane >> 3, ld_piece = lane & 7;          // load role: row (+ 8 r) and 16-byte piece of the 128-byte run
  v16f acc[TMR][CT];
#pragma unroll
  for (int i = 0; i < TMR; ++i)
#pragma unroll
    for (int j = 0; j < CT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const int n_chunks = (k_tiles + CHUNK - 1) / CHUNK;
  const int first = (int)((blockIdx.x * 5u) % (uint32_t)n_chunks);
  for (int ci = wave; ci < n_chunks; ci += WAVES) {
    const int q = ci + first < n_chunks ? ci + first : ci + first - n_chunks;
    const int64_t kb0 = (int64_t)q * 8;                       // first block of the chunk
    u32x4 raw[CT][4];
    u32x2 s8[CT], i8[CT];
#pragma unroll
    for (int j = 0; j < CT; ++j) {
      const int64_t row0 = 32 * (ct + j);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int64_t row = row0 + 8 * r + ld_row;
        raw[j][r] = (u32x4){0, 0, 0, 0};
        if (row < N && kb0 + ld_piece < nbk) raw[j][r] = __builtin_nontemporal_load(w_el + row * nbk + kb0 + ld_piece);
      }
      const int64_t orow = row0 + n_in;
      s8[j] = (u32x2){0, 0};
      i8[j] = (u32x2){0, 0};
      if (orow < N) {                                         // nbk % 8 == 0: the 8 bytes exist and are aligned
        s8[j] = *reinterpret_cast<const u32x2*>(w_sc + orow * nbk + kb0);
        if (PLUS) i8[j] = *reinterpret_cast<const u32x2*>(w_ix + orow * nbk + kb0);
      }
    }
    v8i a[CHUNK][TMR];
    uint32_t sa[CHUNK];
#pragma unroll
    for (int c = 0; c < CHUNK; ++c) {
      const int kt = q * CHUNK + c < k_tiles ? q * CHUNK + c : k_tiles - 1;
      sa[c] = *reinterpret_cast<const uint32_t*>(a_sc + (int64_t)kt * 256 + lane * 4);
#pragma unroll
      for (int i = 0; i < TMR; ++i) {
        const uint8_t* ta = a_el + ((int64_t)i * k_tiles + kt) * AT;
        u32x4 alo = {0, 0, 0, 0};
        u32x2 ahi = {0, 0};
        if (32 * i + (lane & 31) < M) {
          alo = *reinterpret_cast<const u32x4*>(ta + lane * 16);
          if (AT == kTileBytes) ahi = *reinterpret_cast<const u32x2*>(ta + 1024 + lane * 8);
        }
        a[c][i] = (v8i){(int)alo.x, (int)alo.y, (int)alo.z, (int)alo.w, (int)ahi.x, (int)ahi.y, 0, 0};
      }
    }
#pragma unroll
    for (int j = 0; j < CT; ++j) {
      // memory order -> operand order through the wavefront's patch (LDS operations of one wavefront run in order)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        *reinterpret_cast<u32x4*>(patch + (8 * r + ld_row) * kCanonPatchStride + ld_piece * 16) = raw[j][r];
#pragma unroll
      for (int c = 0; c < CHUNK; ++c) {
        const u32x4 nib = *reinterpret_cast<const u32x4*>(patch + n_in * kCanonPatchStride + (2 * c + h) * 16);
        const uint32_t byte_sh = (uint32_t)((2 * c + h) & 3) * 8u;
        uint32_t sbyte = ((2 * c + h) < 4 ? s8[j].x : s8[j].y) >> byte_sh & 0xFFu;
        uint32_t bm = 64u;
        if (PLUS) bm = (((2 * c + h) < 4 ? i8[j].x : i8[j].y) >> byte_sh) & 31u;
        // MXFP4+: the BM split of Eq. 3 as in gemm_skinny_res_kernel -- the BM's nibble becomes the E2M1 code of BM_H
        // (sign | 11 | m2) and BM_L (sign | 0 m1 m0, an E2M1 number too) goes into a second operand that is zero elsewhere
        uint32_t w[4] = {nib.x, nib.y, nib.z, nib.w}, l[4] = {0u, 0u, 0u, 0u};
        if (PLUS) {
          const bool live = sbyte != 0u && sbyte != 255u;
          const uint32_t sh = 4u * (bm & 7u), piece = bm >> 3;
          const uint32_t n4 = ((piece == 0u ? w[0] : piece == 1u ? w[1] : piece == 2u ? w[2] : w[3]) >> sh) & 15u;
          // s m2 m1 m0 -> s 1 1 m2 by xor; s 0 m1 m0 beside it
          const uint32_t flip = live ? (n4 ^ ((n4 & 8u) | 6u | ((n4 >> 2) & 1u))) << sh : 0u;
          const uint32_t low = live ? (n4 & 11u) << sh : 0u;
#pragma unroll
          for (int p = 0; p < 4; ++p) {
            w[p] ^= piece == (uint32_t)p ? flip : 0u;
            l[p] = piece == (uint32_t)p ? low : 0u;
          }
        }
        v8i b = {(int)w[0], (int)w[1], (int)w[2], (int)w[3], 0, 0, 0, 0};
        const v8i lv = {(int)l[0], (int)l[1], (int)l[2], (int)l[3], 0, 0, 0, 0};
        if (sbyte == 0u) {                                    // flushed (or absent) block: zeros, whatever the nibbles say
          b = (v8i){0, 0, 0, 0, 0, 0, 0, 0};
          sbyte = 127u;
        }
        if (q * CHUNK + c < k_tiles) {
#pragma unroll
          for (int i = 0; i < TMR; ++i)
            switch (i) {
#define MXP_CANON_MFMA(I)                                                                               \
  acc[i][j] = mfma<I, 0, FB, FA>(a[c][i], b, acc[i][j], (int)sa[c], (int)sbyte);                         \
  if (PLUS) acc[i][j] = mfma<I, 0, FB, FA>(a[c][i], lv, acc[i][j], (int)sa[c], (int)sbyte);              \
  break
              case 0: MXP_CANON_MFMA(0);
              case 1: MXP_CANON_MFMA(1);
              case 2: MXP_CANON_MFMA(2);
              default: MXP_CANON_MFMA(3);
#undef MXP_CANON_MFMA
            }
        }
      }
    }
  }
  __syncthreads();                                            // the patches make room for the partial tiles
#pragma unroll
  for (int i = 0; i < TMR; ++i)
#pragma unroll
    for (int j = 0; j < CT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) part[wave][i * CT + j][r][lane] = acc[i][j][r];
  __syncthreads();
  for (int e = tid; e < TMR * CT * 16 * 64; e += 64 * WAVES) {
    const int l = e & 63, r = (e >> 6) & 15, ij = e >> 10;
    const int i = ij / CT, j = ij % CT;
    float v = 0.0f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) v += part[w][ij][r][l];
    const int64_t row = 32 * i + (l & 31);
    const int64_t col = 32 * (ct + j) + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
    if (row < M && col < N) {
      if (OUT_BF16) static_cast<uint16_t*>(Dv)[row * ldd + col] = (uint16_t)f32_to_bf16_rne(v);
      else static_cast<float*>(Dv)[row * ldd + col] = v;
    }
  }
}

template <int TMR, int CT, bool PLUS, int WAVES>
void launch_canon_cfg(bool bf, int64_t n_ct, hipStream_t s, const uint8_t* ae, const uint8_t* as, const uint8_t* we, const uint8_t* ws,
                      const uint8_t* wi, int64_t nbk, int kt, int64_t M, int64_t N, void* D, int64_t ldd) {
  constexpr int part_bytes = WAVES * TMR * CT * 16 * 64 * 4, patch_bytes = WAVES * kCanonPatchBytes;
  constexpr int lds = part_bytes > patch_bytes ? part_bytes : patch_bytes;
  static_assert(lds <= 128 * 1024, "partial tiles must fit in LDS");
  const dim3 grid((unsigned)((n_ct + CT - 1) / CT));
  const u32x4* we4 = reinterpret_cast<const u32x4*>(we);
  if (bf) {
    allow_dynamic_lds<&gemm_skinny_canon_kernel<TMR, CT, true, PLUS, kTileBytes, WAVES>>((int)lds);
    hipLaunchKernelGGL((gemm_skinny_canon_kernel<TMR, CT, true, PLUS, kTileBytes, WAVES>), grid, dim3(64 * WAVES), lds, s, ae, as, we4, ws, wi,
                       nbk, kt, M, N, D, ldd);
  } else {
    allow_dynamic_lds<&gemm_skinny_canon_kernel<TMR, CT, false, PLUS, kTileBytes, WAVES>>((int)lds);
    hipLaunchKernelGGL((gemm_skinny_canon_kernel<TMR, CT, false, PLUS, kTileBytes, WAVES>), grid, dim3(64 * WAVES), lds, s, ae, as, we4, ws, wi,
                       nbk, kt, M, N, D, ldd);
  }
}

// A: E2M3 image of M <= 64 rows; W: canonical MXFP4 (PLUS = false) or MXFP4+ arrays, K % 256 == 0.
template <bool PLUS>
int launch_canon(const uint8_t* Ai, const uint8_t* we, const uint8_t* ws, const uint8_t* wi, int64_t M, int64_t N, int64_t K, void* D,
                 int d_dtype, int64_t ldd, hipStream_t s) {
  const ImageGeom ga = image_geom(M, K);
  const int64_t ct = (N + 31) / 32, nbk = K / kBlock;
  if (ct > 2147483647LL || ga.k_tiles > 2147483647LL) return MXP_ERR_UNSUPPORTED;
  const int kt = (int)ga.k_tiles;
  const uint8_t *ae = Ai, *as = Ai + ga.elem_bytes;
  const bool bf = d_dtype == MXP_BF16, wide = kt >= 64;
  constexpr int64_t kEnough = 200;
  if (M <= 32) {
    if (ct / 4 >= kEnough) launch_canon_cfg<1, 4, PLUS, 8>(bf, ct, s, ae, as, we, ws, wi, nbk, kt, M, N, D, ldd);
    else if (ct / 2 >= kEnough) launch_canon_cfg<1, 2, PLUS, 8>(bf, ct, s, ae, as, we, ws, wi, nbk, kt, M, N, D, ldd);
    else if (wide) launch_canon_cfg<1, 1, PLUS, 16>(bf, ct, s, ae, as, we, ws, wi, nbk, kt, M, N, D, ldd);
    else launch_canon_cfg<1, 1, PLUS, 8>(bf, ct, s, ae, as, we, ws, wi, nbk, kt, M, N, D, ldd);
  } else {
    if (ct / 2 >= kEnough) launch_canon_cfg<2, 2, PLUS, 8>(bf, ct, s, ae, as, we, ws, wi, nbk, kt, M, N, D, ldd);
    else launch_canon_cfg<2, 1, PLUS, 8>(bf, ct, s, ae, as, we, ws, wi, nbk, kt, M, N, D, ldd);   // 16 wavefronts would spill
  }
  return launch_status();
}

#ifndef MXP_RING
#define MXP_RING 4   // ring depth; 4 x 25.6 KB + 36 KB of epilogue patches = 136 KB of the 160 KB LDS (E4M3: 4 x 33 KB + 3 KB)
#endif
template <int BT, int AT>
int gemm_images_kind(const uint8_t* Ai, const uint8_t* Bi, int64_t M, int64_t N, int64_t K, void* D, int d_dtype, int64_t ldd,
                     hipStream_t s) {
  // few rows: bound by reading the weights once.  Up to 128 rows when the tiled kernel would get fewer than 64 tile columns
  // (it then leaves most of the chip idle).
  if constexpr (AT == kTileBytes && (BT == kTileBytes || BT == kTileBytesE2M1)) {
    if (skinny16_applies(M, N)) return launch_skinny16<BT, false>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
  }
  if (M <= 64 || (M <= 128 && (N + 255) / 256 < 64)) return launch_skinny<BT, AT>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
  if (block_kernel_applies(M, N)) return launch_block<BT, AT>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
  // the pipelined kernel needs at least 4 k-tiles (prologue of 3 stages + peeled tail) and a whole MI355X (its work
  // lists are cut for 256 compute units in 8 XCDs)
  if (image_geom(M, K).k_tiles < 4 || !chip().whole_mi355x()) return launch_cfg<Cfg<4, 4, 2, 2, BT, AT>>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
  return launch_dma<Cfg<4, 4, 2, 2, BT, AT>, MXP_RING>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
}

// Image kinds per operand: E2M3, or E2M1 for a plain MXFP4 operand.  E2M1 A with E2M3 B is not instantiated (a plain
// MXFP4 A next to MXFP4+ weights is simply widened); the entry points reject that combination.
int gemm_images(const void* A_image, int a_kind, const void* B_image, int b_kind, int64_t M, int64_t N, int64_t K, void* D,
                int d_dtype, int64_t ldd, hipStream_t s) {
  const uint8_t* Ai = static_cast<const uint8_t*>(A_image);
  const uint8_t* Bi = static_cast<const uint8_t*>(B_image);
  // E4M3 images (the MXFP4++ product, Sec. 4.3): the pipelined kernel, or the two-stage one for few rows / short K
  if (b_kind == MXP_IMAGE_E2M1R || b_kind == MXP_IMAGE_E2M1X) {      // decode-only images: 4-bit MX+ weights with residual bytes
    if (a_kind == MXP_IMAGE_E2M1 || M > 64) return MXP_ERR_UNSUPPORTED;
    if (b_kind == MXP_IMAGE_E2M1X) {
      if (a_kind == MXP_IMAGE_E4M3) return launch_skinny_res<kTileBytesE4M3, true>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
      return launch_skinny_res<kTileBytes, true>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
    }
    if (a_kind == MXP_IMAGE_E4M3) return launch_skinny_res<kTileBytesE4M3, false>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
    if (skinny16_applies(M, N)) return launch_skinny16<kTileBytesE2M1, true>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
    return launch_skinny_res<kTileBytes, false>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
  }
  if (a_kind == MXP_IMAGE_E4M3 && b_kind == MXP_IMAGE_E2M1) {   // MXFP4++ activations x plain MXFP4 weights, few rows
    if (M > 64) return MXP_ERR_UNSUPPORTED;
    return launch_skinny<kTileBytesE2M1, kTileBytesE4M3>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
  }
  if (a_kind == MXP_IMAGE_E4M3) {
    using C8 = Cfg<4, 4, 2, 2, kTileBytesE4M3, kTileBytesE4M3>;
    if (M <= 64) return launch_skinny<kTileBytesE4M3, kTileBytesE4M3>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
    if (block_kernel_applies(M, N)) return launch_block<kTileBytesE4M3, kTileBytesE4M3>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
    if (M <= 128 || image_geom(M, K).k_tiles < 4 || !chip().whole_mi355x()) return launch_cfg<C8>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
    return launch_dma<C8, 4>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);   // (4 x 33 KiB: a fifth slot does not fit)
  }
  if (a_kind == MXP_IMAGE_E2M1) return gemm_images_kind<kTileBytesE2M1, kTileBytesE2M1>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
  if (b_kind == MXP_IMAGE_E2M1) return gemm_images_kind<kTileBytesE2M1, kTileBytes>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
  return gemm_images_kind<kTileBytes, kTileBytes>(Ai, Bi, M, N, K, D, d_dtype, ldd, s);
}

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

extern "C" size_t mxp_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K) {
  if (M < 0 || N < 0 || K < 0) return 0;
  return align_up((size_t)mxp::image_geom(M, K).total()) + align_up((size_t)mxp::image_geom(N, K).total());
}

extern "C" size_t mxp_gemm_workspace_bytes_e4m3(int64_t M, int64_t N, int64_t K) {
  if (M < 0 || N < 0 || K < 0) return 0;
  return align_up((size_t)mxp::image_geom(M, K, mxp::kTileBytesE4M3).total()) + align_up((size_t)mxp::image_geom(N, K, mxp::kTileBytesE4M3).total());
}

// Six-bit operands (Sec. 4.2): K segments per image and which of them hold the BM residual.  A+ x B: A = [p | r],
// B = [p | p];  A x B+: A = [p | p], B = [p | r];  A+ x B+: A = [p | r | p | r], B = [p | p | r | r].
namespace {
struct Fp6Plan {
  int n_seg;
  uint32_t mask_a, mask_b;
};
Fp6Plan fp6_plan(int fmtA, int fmtB) {
  const bool pa = fmtA == MXP_FMT_MXFP6P, pb = fmtB == MXP_FMT_MXFP6P;
  if (pa && pb) return {4, 0xAu, 0xCu};
  if (pa) return {2, 0x2u, 0x0u};
  if (pb) return {2, 0x0u, 0x2u};
  return {1, 0u, 0u};
}
bool is_fp6(int fmt) { return fmt == MXP_FMT_MXFP6 || fmt == MXP_FMT_MXFP6P; }
}  // namespace

extern "C" size_t mxp_gemm_workspace_bytes_fmt(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB) {
  if (M < 0 || N < 0 || K < 0) return 0;
  {
    // pairs that are multiplied from de-converted operands: room for A as bf16 (optional, see mxp_gemm)
    const bool valid = fmtA >= MXP_FMT_MXFP4 && fmtA <= MXP_FMT_MXFP8P && fmtB >= MXP_FMT_MXFP4 && fmtB <= MXP_FMT_MXFP8P;
    const bool eight = fmtA == MXP_FMT_MXFP8 || fmtA == MXP_FMT_MXFP8P || fmtB == MXP_FMT_MXFP8 || fmtB == MXP_FMT_MXFP8P;
    const bool six_pp = (is_fp6(fmtA) && fmtB == MXP_FMT_MXFP4PP) || (fmtA == MXP_FMT_MXFP4PP && is_fp6(fmtB));
    if (valid && (eight || six_pp)) return align_up((size_t)M * (size_t)K * 2);
  }
  if (is_fp6(fmtA) && is_fp6(fmtB)) {
    const int n = fp6_plan(fmtA, fmtB).n_seg;
    return align_up(mxp_image_bytes_fp6(M, K, n)) + align_up(mxp_image_bytes_fp6(N, K, n));
  }
  {
    const bool fa = fmtA == MXP_FMT_MXFP4 || fmtA == MXP_FMT_MXFP4P, fb = fmtB == MXP_FMT_MXFP4 || fmtB == MXP_FMT_MXFP4P;
    if ((fmtA == MXP_FMT_MXFP6 && fb) || (fa && fmtB == MXP_FMT_MXFP6)) return mxp_gemm_workspace_bytes(M, N, K);
    if ((fmtA == MXP_FMT_MXFP6P && fb) || (fa && fmtB == MXP_FMT_MXFP6P))
      return align_up(mxp_image_bytes_fp6(M, K, 2)) + align_up(mxp_image_bytes_fp6(N, K, 2));
  }
  const bool a4 = fmtA == MXP_FMT_MXFP4 || fmtA == MXP_FMT_MXFP4P || fmtA == MXP_FMT_MXFP4PP;
  const bool b4 = fmtB == MXP_FMT_MXFP4 || fmtB == MXP_FMT_MXFP4P || fmtB == MXP_FMT_MXFP4PP;
  if (!a4 || !b4) return 0;
  if (fmtA == MXP_FMT_MXFP4PP && fmtB == MXP_FMT_MXFP4PP) return mxp_gemm_workspace_bytes_e4m3(M, N, K);
  if (fmtA == MXP_FMT_MXFP4PP || fmtB == MXP_FMT_MXFP4PP)      // one-sided MXFP4++: two K segments per image
    return align_up(mxp_image_bytes_fp6(M, K, 2)) + align_up(mxp_image_bytes_fp6(N, K, 2));
  return mxp_gemm_workspace_bytes(M, N, K);
}

extern "C" size_t mxp_gemm_workspace_size(int64_t M, int64_t N, int64_t K, int fmtA, int fmtB) {
  return mxp_gemm_workspace_bytes_fmt(M, N, K, fmtA, fmtB);
}

extern "C" int mxp_gemm_prepacked(int64_t M, int64_t N, int64_t K, const void* A_image, int a_kind, const void* B_image,
                                  int b_kind, void* D, int d_dtype, int64_t ldd, void* stream) {
  if (b_kind != MXP_IMAGE_E2M3 && b_kind != MXP_IMAGE_E2M1 && b_kind != MXP_IMAGE_E4M3 && b_kind != MXP_IMAGE_E2M1R && b_kind != MXP_IMAGE_E2M1X) return MXP_ERR_FORMAT;
  if (a_kind != MXP_IMAGE_E2M3 && a_kind != MXP_IMAGE_E2M1 && a_kind != MXP_IMAGE_E4M3) return MXP_ERR_FORMAT;
  if (a_kind == MXP_IMAGE_E2M1 && b_kind != MXP_IMAGE_E2M1) return MXP_ERR_UNSUPPORTED;
  const bool b_res = b_kind == MXP_IMAGE_E2M1R || b_kind == MXP_IMAGE_E2M1X;
  if (b_res && (a_kind == MXP_IMAGE_E2M1 || M > 64)) return MXP_ERR_UNSUPPORTED;
  // E4M3 images pair with each other; few rows of E4M3 activations (MXFP4++) also with the 4-bit weight images
  const bool b_four = b_kind == MXP_IMAGE_E2M1 || b_res;
  if ((a_kind == MXP_IMAGE_E4M3) != (b_kind == MXP_IMAGE_E4M3) && !(a_kind == MXP_IMAGE_E4M3 && b_four && M <= 64)) return MXP_ERR_UNSUPPORTED;
  int rc = check_gemm(M, N, K, D, d_dtype, ldd, 4 * kMaxGemmK);   // K of the images: up to four K segments
  if (rc != MXP_OK || M == 0 || N == 0) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (K == 0) return zero_output(D, d_dtype, M, N, ldd, s);
  if (!A_image || !B_image) return MXP_ERR_NULL;
  if (!mxp::aligned16(A_image) || !mxp::aligned16(B_image)) return MXP_ERR_ALIGN;
  return gemm_images(A_image, a_kind, B_image, b_kind, M, N, K, D, d_dtype, ldd, s);
}

extern "C" int mxp_gemm(int64_t M, int64_t N, int64_t K, const uint8_t* A_elems, const uint8_t* A_scales, const uint8_t* A_idx,
                        int fmtA, const uint8_t* B_elems, const uint8_t* B_scales, const uint8_t* B_idx, int fmtB, void* D,
                        int d_dtype, int64_t ldd, void* workspace, size_t workspace_bytes, void* stream) {
  using namespace mxp;
  const bool pp = fmtA == MXP_FMT_MXFP4PP || fmtB == MXP_FMT_MXFP4PP;
  const bool six = is_fp6(fmtA) || is_fp6(fmtB), eight = fmtA == MXP_FMT_MXFP8 || fmtB == MXP_FMT_MXFP8;   // (eight: mixed with a narrower format)
  const bool eight_plus = fmtA == MXP_FMT_MXFP8P || fmtB == MXP_FMT_MXFP8P;
  if (eight_plus || eight || (six && pp)) {
    // an E4M7 BM fits no block-scaled MFMA element: the product of the de-converted operands on the bf16 MFMA (exact
    // products: every value is a bf16 number), at least one operand eight-bit, the other of any format; no workspace.  A
    // six-bit format next to MXFP4++ goes the same way (two scales per block on one side, a six-bit BM split on the other).
    // Plain MXFP8 x MXFP8 takes this route too: the FP8 MFMA aligns the 64 products of a k-tile to the largest and drops
    // what falls below its adder width, which the stated error bound of this entry point does not admit (that faster route
    // remains available through mxp_prepack_fp8 + mxp_gemm_prepacked, with its own bound).
    if (fmtA < MXP_FMT_MXFP4 || fmtA > MXP_FMT_MXFP8P || fmtB < MXP_FMT_MXFP4 || fmtB > MXP_FMT_MXFP8P) return MXP_ERR_FORMAT;
    int rc8 = check_gemm(M, N, K, D, d_dtype, ldd);
    if (rc8 != MXP_OK || M == 0 || N == 0) return rc8;
    hipStream_t s8 = static_cast<hipStream_t>(stream);
    if (K == 0) return zero_output(D, d_dtype, M, N, ldd, s8);
    const bool ix_a = fmtA != MXP_FMT_MXFP4 && !plain_wide_format(fmtA), ix_b = fmtB != MXP_FMT_MXFP4 && !plain_wide_format(fmtB);
    if (!A_elems || !A_scales || !B_elems || !B_scales || (ix_a && !A_idx) || (ix_b && !B_idx)) return MXP_ERR_NULL;
    if (!aligned16(A_elems) || !aligned16(A_scales) || !aligned16(B_elems) || !aligned16(B_scales) || (A_idx && !aligned16(A_idx)) ||
        (B_idx && !aligned16(B_idx)))
      return MXP_ERR_ALIGN;
    // With a workspace for A as bf16 (2 M K bytes) A is de-converted once, by the de-conversion kernel, and the product runs
    // as the conversion-based one (bf16 rows x quantized B): the same bf16 values are multiplied (in the tiled kernel, which
    // takes more than 128 rows, by the same MFMAs in the same order: identical bits), and A is no longer de-converted again
    // for every tile column (1.3 - 1.65x faster).
    // Without it, both operands are de-converted inside the kernel.
    const size_t a_bf16 = align_up((size_t)M * (size_t)K * 2);
    if (workspace && aligned16(workspace) && workspace_bytes >= a_bf16) {
      rc8 = mxp_dequantize(A_elems, A_scales, A_idx, fmtA, M, K, workspace, MXP_BF16, K, stream);
      if (rc8 != MXP_OK) return rc8;
      return mxp_gemm_w4a16(M, N, K, workspace, MXP_BF16, K, B_elems, B_scales, B_idx, fmtB, D, d_dtype, ldd, stream);
    }
    return deconv_gemm_launch(M, N, K, A_elems, A_scales, A_idx, fmtA, B_elems, B_scales, B_idx, fmtB, D, d_dtype, ldd, s8);
  }
  if (six) {
    if (fmtA < MXP_FMT_MXFP4 || fmtA > MXP_FMT_MXFP8P || fmtB < MXP_FMT_MXFP4 || fmtB > MXP_FMT_MXFP8P) return MXP_ERR_FORMAT;
    // both operands six-bit, or a six-bit operand with MXFP4 / MXFP4+ (plain MXFP6: one segment, the
    // same E2M3 / E2M1 images as ever; MXFP6+: its two K segments, primary and BM residual, against the four-bit operand's
    // E2M3 image laid out twice)
    const bool four_a = fmtA == MXP_FMT_MXFP4 || fmtA == MXP_FMT_MXFP4P, four_b = fmtB == MXP_FMT_MXFP4 || fmtB == MXP_FMT_MXFP4P;
    const bool mixed64 = (is_fp6(fmtA) && four_b) || (four_a && is_fp6(fmtB));
    if (!(is_fp6(fmtA) && is_fp6(fmtB)) && !mixed64) return MXP_ERR_UNSUPPORTED;
  } else if ((fmtA != MXP_FMT_MXFP4 && fmtA != MXP_FMT_MXFP4P && fmtA != MXP_FMT_MXFP4PP) ||
             (fmtB != MXP_FMT_MXFP4 && fmtB != MXP_FMT_MXFP4P && fmtB != MXP_FMT_MXFP4PP)) {
    return MXP_ERR_FORMAT;
  }
  int rc = check_gemm(M, N, K, D, d_dtype, ldd);
  if (rc != MXP_OK || M == 0 || N == 0) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (K == 0) return zero_output(D, d_dtype, M, N, ldd, s);
  const bool idx_a = fmtA != MXP_FMT_MXFP4 && !plain_wide_format(fmtA), idx_b = fmtB != MXP_FMT_MXFP4 && !plain_wide_format(fmtB);
  if (!A_elems || !A_scales || !B_elems || !B_scales || (idx_a && !A_idx) || (idx_b && !B_idx) || !workspace)
    return MXP_ERR_NULL;
  if (!aligned16(A_elems) || !aligned16(A_scales) || !aligned16(B_elems) || !aligned16(B_scales) || !aligned16(workspace) ||
      (A_idx && !aligned16(A_idx)) || (B_idx && !aligned16(B_idx)))
    return MXP_ERR_ALIGN;
  if (six && !(is_fp6(fmtA) && is_fp6(fmtB)) && (fmtA == MXP_FMT_MXFP6P || fmtB == MXP_FMT_MXFP6P)) {
    // MXFP6+ with a four-bit operand (Sec. 5: the approach carries over to MXFP6+): two K segments
    if (workspace_bytes < mxp_gemm_workspace_bytes_fmt(M, N, K, fmtA, fmtB)) return MXP_ERR_WORKSPACE;
    uint8_t* wa2 = static_cast<uint8_t*>(workspace);
    uint8_t* wb2 = wa2 + align_up(mxp_image_bytes_fp6(M, K, 2));
    rc = is_fp6(fmtA) ? prepack_fp6_launch(A_elems, A_scales, A_idx, fmtA, M, K, 2, 0x2u, wa2, s)
                      : prepack_seg_launch(A_elems, A_scales, A_idx, fmtA, M, K, 2, 0u, wa2, s);
    if (rc != MXP_OK) return rc;
    rc = is_fp6(fmtB) ? prepack_fp6_launch(B_elems, B_scales, B_idx, fmtB, N, K, 2, 0x2u, wb2, s)
                      : prepack_seg_launch(B_elems, B_scales, B_idx, fmtB, N, K, 2, 0u, wb2, s);
    if (rc != MXP_OK) return rc;
    return gemm_images(wa2, MXP_IMAGE_E2M3, wb2, MXP_IMAGE_E2M3, M, N, image_geom(M, K).K_p * 2, D, d_dtype, ldd, s);
  }
  if (six && !(is_fp6(fmtA) && is_fp6(fmtB))) {
    // plain MXFP6 with a four-bit operand: one E2M3 image each (a plain MXFP4 B stays in four-bit codes)
    if (workspace_bytes < mxp_gemm_workspace_bytes(M, N, K)) return MXP_ERR_WORKSPACE;
    uint8_t* wa = static_cast<uint8_t*>(workspace);
    uint8_t* wb = wa + align_up((size_t)image_geom(M, K).total());
    rc = is_fp6(fmtA) ? prepack_fp6_launch(A_elems, A_scales, nullptr, fmtA, M, K, 1, 0u, wa, s)
                      : prepack_launch(A_elems, A_scales, A_idx, fmtA, M, K, wa, s);
    if (rc != MXP_OK) return rc;
    const bool b4 = fmtB == MXP_FMT_MXFP4;
    rc = is_fp6(fmtB) ? prepack_fp6_launch(B_elems, B_scales, nullptr, fmtB, N, K, 1, 0u, wb, s)
         : b4         ? prepack_e2m1_launch(B_elems, B_scales, nullptr, N, K, wb, s, 0)
                      : prepack_launch(B_elems, B_scales, B_idx, fmtB, N, K, wb, s);
    if (rc != MXP_OK) return rc;
    return gemm_images(wa, MXP_IMAGE_E2M3, wb, b4 ? MXP_IMAGE_E2M1 : MXP_IMAGE_E2M3, M, N, K, D, d_dtype, ldd, s);
  }
  if (six) {
    const Fp6Plan plan = fp6_plan(fmtA, fmtB);
    if (workspace_bytes < mxp_gemm_workspace_bytes_fmt(M, N, K, fmtA, fmtB)) return MXP_ERR_WORKSPACE;
    uint8_t* wa6 = static_cast<uint8_t*>(workspace);
    uint8_t* wb6 = wa6 + align_up(mxp_image_bytes_fp6(M, K, plan.n_seg));
    rc = prepack_fp6_launch(A_elems, A_scales, A_idx, fmtA, M, K, plan.n_seg, plan.mask_a, wa6, s);
    if (rc != MXP_OK) return rc;
    rc = prepack_fp6_launch(B_elems, B_scales, B_idx, fmtB, N, K, plan.n_seg, plan.mask_b, wb6, s);
    if (rc != MXP_OK) return rc;
    return gemm_images(wa6, MXP_IMAGE_E2M3, wb6, MXP_IMAGE_E2M3, M, N, image_geom(M, K).K_p * plan.n_seg, D, d_dtype, ldd, s);
  }
  if (pp && (fmtA == MXP_FMT_MXFP4PP) != (fmtB == MXP_FMT_MXFP4PP)) {
    // one MXFP4++ operand (Sec. 4.3; Sec. 7.1: MX++ activations on MXFP4 / MXFP4+ weights): the exact product over two K
    // segments -- the MXFP4++ operand as [elements without the BM, scale lowered by delta | the BM alone, own scale], the
    // other operand as its E2M3 image twice
    if (workspace_bytes < mxp_gemm_workspace_bytes_fmt(M, N, K, fmtA, fmtB)) return MXP_ERR_WORKSPACE;
    constexpr uint32_t kSplit = 1u | (2u << 2), kTwice = 0u;
    uint8_t* wa2 = static_cast<uint8_t*>(workspace);
    uint8_t* wb2 = wa2 + align_up(mxp_image_bytes_fp6(M, K, 2));
    rc = prepack_seg_launch(A_elems, A_scales, A_idx, fmtA, M, K, 2, fmtA == MXP_FMT_MXFP4PP ? kSplit : kTwice, wa2, s);
    if (rc != MXP_OK) return rc;
    rc = prepack_seg_launch(B_elems, B_scales, B_idx, fmtB, N, K, 2, fmtB == MXP_FMT_MXFP4PP ? kSplit : kTwice, wb2, s);
    if (rc != MXP_OK) return rc;
    return gemm_images(wa2, MXP_IMAGE_E2M3, wb2, MXP_IMAGE_E2M3, M, N, image_geom(M, K).K_p * 2, D, d_dtype, ldd, s);
  }
  if (pp) {
    // both operands MXFP4++: E4M3 images (Sec. 4.3), FP8 MFMAs
    if (workspace_bytes < mxp_gemm_workspace_bytes_e4m3(M, N, K)) return MXP_ERR_WORKSPACE;
    uint8_t* wa8 = static_cast<uint8_t*>(workspace);
    uint8_t* wb8 = wa8 + align_up((size_t)image_geom(M, K, kTileBytesE4M3).total());
    rc = prepack_e4m3_launch(A_elems, A_scales, A_idx, fmtA, M, K, wa8, s);
    if (rc != MXP_OK) return rc;
    rc = prepack_e4m3_launch(B_elems, B_scales, B_idx, fmtB, N, K, wb8, s);
    if (rc != MXP_OK) return rc;
    return gemm_images(wa8, MXP_IMAGE_E4M3, wb8, MXP_IMAGE_E4M3, M, N, K, D, d_dtype, ldd, s);
  }
  if (workspace_bytes < mxp_gemm_workspace_bytes(M, N, K)) return MXP_ERR_WORKSPACE;
  uint8_t* wa = static_cast<uint8_t*>(workspace);
  uint8_t* wb = wa + align_up((size_t)image_geom(M, K).total());
  if (M <= 64 && fmtB == MXP_FMT_MXFP4P) {
    // few rows (the decode stage, Sec. 7.2): the product is bound by the weight bytes, so MXFP4+ weights go into the 4-bit
    // image with residual bytes (BM_H in place, BM_L by a second MFMA: Eq. 3, Sec. 5.2) instead of the wider E2M3 one --
    // fewer bytes to write here and fewer to read in the product
    rc = prepack_launch(A_elems, A_scales, A_idx, fmtA, M, K, wa, s);
    if (rc != MXP_OK) return rc;
    rc = prepack_e2m1_launch(B_elems, B_scales, B_idx, N, K, wb, s, 1);
    if (rc != MXP_OK) return rc;
    return gemm_images(wa, MXP_IMAGE_E2M3, wb, MXP_IMAGE_E2M1R, M, N, K, D, d_dtype, ldd, s);
  }
  // a plain MXFP4 B operand stays in 4-bit codes (smaller image, less operand traffic in the product); so does A
  // when both operands are plain MXFP4
  const bool b4 = fmtB == MXP_FMT_MXFP4, a4 = b4 && fmtA == MXP_FMT_MXFP4;
  rc = a4 ? prepack_e2m1_launch(A_elems, A_scales, nullptr, M, K, wa, s, 0) : prepack_launch(A_elems, A_scales, A_idx, fmtA, M, K, wa, s);
  if (rc != MXP_OK) return rc;
  rc = b4 ? prepack_e2m1_launch(B_elems, B_scales, nullptr, N, K, wb, s, 0) : prepack_launch(B_elems, B_scales, B_idx, fmtB, N, K, wb, s);
  if (rc != MXP_OK) return rc;
  return gemm_images(wa, a4 ? MXP_IMAGE_E2M1 : MXP_IMAGE_E2M3, wb, b4 ? MXP_IMAGE_E2M1 : MXP_IMAGE_E2M3, M, N, K, D, d_dtype, ldd, s);
}

// ---- mxp_gemm without a caller workspace ------------------------------------------------------------------------
// For callers that cannot allocate (HIP graph capture, serving loops that forbid hipMalloc): the two operand images go
// to a file-scope device array instead of a workspace argument.  Every GPU the library runs on holds its own copy of
// the array at its own address until the process ends; host code never uses the array's name as a pointer (it is only
// a stand-in on the host) but the address hipGetSymbolAddress returns, asked once per device with that device current.
namespace {
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) uint8_t scratch[kStaticScratchBytes];

int static_scratch(void** out) {
  constexpr int kMaxDev = 64;
  static std::mutex mu;
  static void* ptr[kMaxDev] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return MXP_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return MXP_ERR_HIP;
    }
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return MXP_OK;
}
}  // namespace

extern "C" size_t mxp_gemm_static_capacity(void) { return kStaticScratchBytes; }

extern "C" int mxp_gemm_static(int64_t M, int64_t N, int64_t K, const uint8_t* A_elems, const uint8_t* A_scales, const uint8_t* A_idx,
                               int fmtA, const uint8_t* B_elems, const uint8_t* B_scales, const uint8_t* B_idx, int fmtB, void* D,
                               int d_dtype, int64_t ldd, void* stream) {
  if (fmtA < MXP_FMT_MXFP4 || fmtA > MXP_FMT_MXFP8P || fmtB < MXP_FMT_MXFP4 || fmtB > MXP_FMT_MXFP8P) return MXP_ERR_FORMAT;
  if (M < 0 || N < 0 || K < 0) return MXP_ERR_SHAPE;
  // (the size functions saturate nowhere near these limits: image bytes of 2^31 x 2^21 elements still fit a size_t)
  if (M > ((int64_t)1 << 31) || N > ((int64_t)1 << 31) || K > mxp::kMaxGemmK) return MXP_ERR_SCRATCH;
  // pairs multiplied from de-converted operands use the workspace only as an option (A as bf16): too large a product of
  // that kind runs without it instead of being refused
  const bool optional_ws = fmtA >= MXP_FMT_MXFP8 || fmtB >= MXP_FMT_MXFP8 || (is_fp6(fmtA) && fmtB == MXP_FMT_MXFP4PP) ||
                           (fmtA == MXP_FMT_MXFP4PP && is_fp6(fmtB));
  const bool fits = mxp_gemm_workspace_bytes_fmt(M, N, K, fmtA, fmtB) <= kStaticScratchBytes;
  if (!fits && !optional_ws) return MXP_ERR_SCRATCH;
  void* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != MXP_OK) return rc;
  return mxp_gemm(M, N, K, A_elems, A_scales, A_idx, fmtA, B_elems, B_scales, B_idx, fmtB, D, d_dtype, ldd, ws, fits ? kStaticScratchBytes : 0,
                  stream);
}

extern "C" size_t mxp_gemm_bf16a_workspace_bytes(int64_t M, int64_t K) {
  if (M < 0 || K < 0) return 0;
  return align_up((size_t)mxp::image_geom(M, K).total());
}

extern "C" int mxp_gemm_bf16a(int64_t M, int64_t N, int64_t K, const void* A, int a_dtype, int64_t lda, int fmtA,
                              const void* B_image, int b_kind, void* D, int d_dtype, int64_t ldd, void* workspace,
                              size_t workspace_bytes, void* stream) {
  using namespace mxp;
  if (fmtA != MXP_FMT_MXFP4 && fmtA != MXP_FMT_MXFP4P && fmtA != MXP_FMT_MXFP4PP) return MXP_ERR_FORMAT;
  if (b_kind != MXP_IMAGE_E2M3 && b_kind != MXP_IMAGE_E2M1 && b_kind != MXP_IMAGE_E4M3 && b_kind != MXP_IMAGE_E2M1R && b_kind != MXP_IMAGE_E2M1X) return MXP_ERR_FORMAT;
  const bool fp8 = fmtA == MXP_FMT_MXFP4PP;
  const bool b_res = b_kind == MXP_IMAGE_E2M1R || b_kind == MXP_IMAGE_E2M1X, b_four = b_kind == MXP_IMAGE_E2M1 || b_res;
  if (fp8 != (b_kind == MXP_IMAGE_E4M3) && !(fp8 && b_four && M <= 64)) return MXP_ERR_UNSUPPORTED;
  if (b_res && M > 64) return MXP_ERR_UNSUPPORTED;
  if (a_dtype != MXP_F32 && a_dtype != MXP_BF16) return MXP_ERR_DTYPE;
  int rc = check_gemm(M, N, K, D, d_dtype, ldd);
  if (rc != MXP_OK || M == 0 || N == 0) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (K == 0) return zero_output(D, d_dtype, M, N, ldd, s);
  if (!A || !B_image || !workspace) return MXP_ERR_NULL;
  if (lda < K) return MXP_ERR_SHAPE;
  if (!aligned16(A) || !aligned16(B_image) || !aligned16(workspace) || (lda * (a_dtype == MXP_BF16 ? 2 : 4)) % 16 != 0)
    return MXP_ERR_ALIGN;
  if (workspace_bytes < (fp8 ? mxp_image_bytes_e4m3(M, K) : mxp_gemm_bf16a_workspace_bytes(M, K))) return MXP_ERR_WORKSPACE;
  uint8_t* img = static_cast<uint8_t*>(workspace);
  rc = quantize_image_launch(A, a_dtype, M, K, lda, fmtA, nullptr, nullptr, nullptr, img, s, /*skip_padding_tiles=*/M <= 64);   // (M <= 64: the few-row kernels read only the tiles that hold rows)
  if (rc != MXP_OK) return rc;
  return gemm_images(img, fp8 ? MXP_IMAGE_E4M3 : MXP_IMAGE_E2M3, B_image, b_kind, M, N, K, D, d_dtype, ldd, s);
}

// Few activation rows against weights in canonical storage (the decode stage, Sec. 7.2).
extern "C" int mxp_gemm_decode(int64_t M, int64_t N, int64_t K, const void* A_image, const uint8_t* W_elems,
                               const uint8_t* W_scales, const uint8_t* W_idx, int fmtW, void* D, int d_dtype, int64_t ldd,
                               void* stream) {
  using namespace mxp;
  if (fmtW == MXP_FMT_MXFP4PP) return MXP_ERR_UNSUPPORTED;
  if (fmtW != MXP_FMT_MXFP4 && fmtW != MXP_FMT_MXFP4P) return MXP_ERR_FORMAT;
  int rc = check_gemm(M, N, K, D, d_dtype, ldd);
  if (rc != MXP_OK || M == 0 || N == 0) return rc;
  if (M > 64 || K % 256 != 0) return MXP_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (K == 0) return zero_output(D, d_dtype, M, N, ldd, s);
  if (!A_image || !W_elems || !W_scales || (fmtW == MXP_FMT_MXFP4P && !W_idx)) return MXP_ERR_NULL;
  if (!aligned16(A_image) || !aligned16(W_elems) || !aligned16(W_scales) || (W_idx && !aligned16(W_idx))) return MXP_ERR_ALIGN;
  const uint8_t* Ai = static_cast<const uint8_t*>(A_image);
  if (fmtW == MXP_FMT_MXFP4P) return launch_canon<true>(Ai, W_elems, W_scales, W_idx, M, N, K, D, d_dtype, ldd, s);
  return launch_canon<false>(Ai, W_elems, W_scales, W_idx, M, N, K, D, d_dtype, ldd, s);
}

extern "C" int mxp_gemm_decode_bf16a(int64_t M, int64_t N, int64_t K, const void* A, int a_dtype, int64_t lda, int fmtA,
                                     const uint8_t* W_elems, const uint8_t* W_scales, const uint8_t* W_idx, int fmtW, void* D,
                                     int d_dtype, int64_t ldd, void* workspace, size_t workspace_bytes, void* stream) {
  using namespace mxp;
  if (fmtA == MXP_FMT_MXFP4PP) return MXP_ERR_UNSUPPORTED;
  if (fmtA != MXP_FMT_MXFP4 && fmtA != MXP_FMT_MXFP4P) return MXP_ERR_FORMAT;
  if (a_dtype != MXP_F32 && a_dtype != MXP_BF16) return MXP_ERR_DTYPE;
  if (fmtW == MXP_FMT_MXFP4PP) return MXP_ERR_UNSUPPORTED;
  if (fmtW != MXP_FMT_MXFP4 && fmtW != MXP_FMT_MXFP4P) return MXP_ERR_FORMAT;
  int rc = check_gemm(M, N, K, D, d_dtype, ldd);
  if (rc != MXP_OK || M == 0 || N == 0) return rc;
  if (M > 64 || K % 256 != 0) return MXP_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (K == 0) return zero_output(D, d_dtype, M, N, ldd, s);
  if (!A || !workspace) return MXP_ERR_NULL;
  if (lda < K) return MXP_ERR_SHAPE;
  if (!aligned16(A) || !aligned16(workspace) || (lda * (a_dtype == MXP_BF16 ? 2 : 4)) % 16 != 0) return MXP_ERR_ALIGN;
  if (workspace_bytes < mxp_gemm_bf16a_workspace_bytes(M, K)) return MXP_ERR_WORKSPACE;
  uint8_t* img = static_cast<uint8_t*>(workspace);
  rc = quantize_image_launch(A, a_dtype, M, K, lda, fmtA, nullptr, nullptr, nullptr, img, s, /*skip_padding_tiles=*/M <= 64);   // (M <= 64: the few-row kernels read only the tiles that hold rows)
  if (rc != MXP_OK) return rc;
  return mxp_gemm_decode(M, N, K, img, W_elems, W_scales, W_idx, fmtW, D, d_dtype, ldd, stream);
}

extern "C" const char* mxp_status_string(int status) {
  switch (status) {
    case MXP_OK: return "ok";
    case MXP_ERR_NULL: return "null pointer";
    case MXP_ERR_SHAPE: return "bad shape (negative size, K not a multiple of 32, or leading dimension too small)";
    case MXP_ERR_ALIGN: return "pointer or leading dimension not 16-byte aligned";
    case MXP_ERR_DTYPE: return "unknown dtype";
    case MXP_ERR_FORMAT: return "unknown block format";
    case MXP_ERR_WORKSPACE: return "workspace or image buffer too small";
    case MXP_ERR_HIP: return "HIP launch error";
    case MXP_ERR_UNSUPPORTED: return "request not supported by this build";
    case MXP_ERR_SCRATCH: return "operand images exceed the built-in scratch array of mxp_gemm_static (mxp_gemm_static_capacity bytes)";
    default: return "unknown status";
  }
}

extern "C" int mxp_version(void) { return 100; }
