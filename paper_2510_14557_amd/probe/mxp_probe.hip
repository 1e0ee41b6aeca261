// Measurement aid (own library, not part of libmxp): the matrix pipes alone.
// One workgroup per compute unit, one wavefront per SIMD, 16 independent accumulator tiles per wavefront (the shape of
// the product kernel's inner loop), operands resident in registers.  What this reaches is what the chip's power limit
// leaves of the nominal MFMA rate for these operand formats and bits.
#include "mxp_probe.h"
#include "mxp_common.h"

namespace {
using namespace mxp;
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kFmtE2M3 = 2, kFmtE4M3 = 0, kFmtE2M1 = 4;   // cbsz / blgp codes of the f8f6f4 MFMA

template <int FA, int FB>
__device__ __forceinline__ void probe_loop(const v8i (&a)[4], const v8i (&b)[4], int sa, int sb, int iters, float* sink) {
  v16f acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[j], a[i], acc[i][j], FB, FA, 0, sb, 0, sa);
  }
  float x = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) x += acc[i][j][r];
  sink[blockIdx.x * 256 + threadIdx.x] = x;
}

template <int FA, int FB>
__global__ void __launch_bounds__(256) mfma_probe_kernel(float* __restrict__ sink, int iters, uint32_t seed) {
  v8i a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a[j][i] = (int)((threadIdx.x * 2654435761u + (8 * j + i) * 40503u + blockIdx.x) * seed);
      b[j][i] = (int)((threadIdx.x * 2246822519u + (8 * j + i) * 3266489917u + blockIdx.x) * seed);
    }
  probe_loop<FA, FB>(a, b, 0x7F7F7F7F, 0x7F7F7F7F, iters, sink);
}

// one lane's operand of image tile `t` (tile_bytes 1024 / 1536 / 2048: 16, 24 or 32 bytes per lane)
__device__ __forceinline__ v8i load_operand(const uint8_t* tile, int tile_bytes, int lane) {
  const u32x4 lo = *reinterpret_cast<const u32x4*>(tile + lane * 16);
  u32x4 hi = {0, 0, 0, 0};
  if (tile_bytes == kTileBytes) {
    const u32x2 h = *reinterpret_cast<const u32x2*>(tile + 1024 + lane * 8);
    hi.x = h.x;
    hi.y = h.y;
  } else if (tile_bytes == kTileBytesE4M3) {
    hi = *reinterpret_cast<const u32x4*>(tile + 1024 + lane * 16);
  }
  return (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
}

template <int FA, int FB, int AT, int BT>
__global__ void __launch_bounds__(256) mfma_probe_images_kernel(const uint8_t* __restrict__ a_img, int64_t a_tiles, int64_t a_sc_off,
                                                                const uint8_t* __restrict__ b_img, int64_t b_tiles, int64_t b_sc_off,
                                                                int64_t k_tiles, float* __restrict__ sink, int iters) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t id = (uint64_t)blockIdx.x * 4 + wave;
  v8i a[4], b[4];
  // four tiles of each operand, spread over the image (all indices < number of tiles: no access leaves the image)
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int64_t ta = (int64_t)((id * 4 + j) * 2654435761ull % (uint64_t)a_tiles);
    const int64_t tb = (int64_t)((id * 4 + j) * 2246822519ull % (uint64_t)b_tiles);
    a[j] = load_operand(a_img + ta * AT, AT, lane);
    b[j] = load_operand(b_img + tb * BT, BT, lane);
  }
  // scale dwords of the first tile's row-tile group and k-tile (tile t = row_tile * k_tiles + k_tile)
  const int64_t ta0 = (int64_t)((id * 4) * 2654435761ull % (uint64_t)a_tiles), tb0 = (int64_t)((id * 4) * 2246822519ull % (uint64_t)b_tiles);
  const int sa = *reinterpret_cast<const int*>(a_img + a_sc_off + (((ta0 / k_tiles) >> 2) * k_tiles + ta0 % k_tiles) * 256 + lane * 4);
  const int sb = *reinterpret_cast<const int*>(b_img + b_sc_off + (((tb0 / k_tiles) >> 2) * k_tiles + tb0 % k_tiles) * 256 + lane * 4);
  probe_loop<FA, FB>(a, b, sa, sb, iters, sink);
}

int tile_bytes_of(int kind) {
  return kind == MXP_IMAGE_E2M3 ? kTileBytes : kind == MXP_IMAGE_E2M1 ? kTileBytesE2M1 : kind == MXP_IMAGE_E4M3 ? kTileBytesE4M3 : 0;
}
}  // namespace

extern "C" int mxp_probe_mfma(int a_kind, int b_kind, int iters, uint32_t seed, float* sink, void* stream) {
  const bool fp8 = a_kind == MXP_IMAGE_E4M3 && b_kind == MXP_IMAGE_E4M3;
  if (!fp8 && ((a_kind != MXP_IMAGE_E2M3 && a_kind != MXP_IMAGE_E2M1) || (b_kind != MXP_IMAGE_E2M3 && b_kind != MXP_IMAGE_E2M1))) return MXP_ERR_FORMAT;
  if (iters < 0 || iters > (1 << 24)) return MXP_ERR_SHAPE;
  if (!sink) return MXP_ERR_NULL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid(256), block(256);
  if (fp8) hipLaunchKernelGGL((mfma_probe_kernel<kFmtE4M3, kFmtE4M3>), grid, block, 0, s, sink, iters, seed);
  else if (a_kind == MXP_IMAGE_E2M3 && b_kind == MXP_IMAGE_E2M3) hipLaunchKernelGGL((mfma_probe_kernel<kFmtE2M3, kFmtE2M3>), grid, block, 0, s, sink, iters, seed);
  else if (a_kind == MXP_IMAGE_E2M3) hipLaunchKernelGGL((mfma_probe_kernel<kFmtE2M3, kFmtE2M1>), grid, block, 0, s, sink, iters, seed);
  else if (b_kind == MXP_IMAGE_E2M3) hipLaunchKernelGGL((mfma_probe_kernel<kFmtE2M1, kFmtE2M3>), grid, block, 0, s, sink, iters, seed);
  else hipLaunchKernelGGL((mfma_probe_kernel<kFmtE2M1, kFmtE2M1>), grid, block, 0, s, sink, iters, seed);
  return mxp::launch_status();
}

extern "C" int mxp_probe_mfma_images(const void* a_image, int a_kind, int64_t rows_a, const void* b_image, int b_kind, int64_t rows_b,
                                     int64_t K, int iters, float* sink, void* stream) {
  const int at = tile_bytes_of(a_kind), bt = tile_bytes_of(b_kind);
  if (!at || !bt) return MXP_ERR_FORMAT;
  if ((a_kind == MXP_IMAGE_E4M3) != (b_kind == MXP_IMAGE_E4M3)) return MXP_ERR_UNSUPPORTED;
  if (a_kind == MXP_IMAGE_E2M1 && b_kind == MXP_IMAGE_E2M3) return MXP_ERR_UNSUPPORTED;
  if (iters < 0 || iters > (1 << 24) || rows_a <= 0 || rows_b <= 0 || K <= 0 || K % 32 != 0) return MXP_ERR_SHAPE;
  if (!sink || !a_image || !b_image) return MXP_ERR_NULL;
  if (!mxp::aligned16(a_image) || !mxp::aligned16(b_image)) return MXP_ERR_ALIGN;
  const ImageGeom ga = image_geom(rows_a, K, at), gb = image_geom(rows_b, K, bt);
  const uint8_t* A = static_cast<const uint8_t*>(a_image);
  const uint8_t* B = static_cast<const uint8_t*>(b_image);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid(256), block(256);
  const int64_t na = ga.row_tiles * ga.k_tiles, nb = gb.row_tiles * gb.k_tiles;
#define MXP_PROBE_LAUNCH(FA, FB, AT, BT) \
  hipLaunchKernelGGL((mfma_probe_images_kernel<FA, FB, AT, BT>), grid, block, 0, s, A, na, ga.elem_bytes, B, nb, gb.elem_bytes, ga.k_tiles, sink, iters)
  if (a_kind == MXP_IMAGE_E4M3) MXP_PROBE_LAUNCH(kFmtE4M3, kFmtE4M3, kTileBytesE4M3, kTileBytesE4M3);
  else if (a_kind == MXP_IMAGE_E2M3 && b_kind == MXP_IMAGE_E2M3) MXP_PROBE_LAUNCH(kFmtE2M3, kFmtE2M3, kTileBytes, kTileBytes);
  else if (a_kind == MXP_IMAGE_E2M3) MXP_PROBE_LAUNCH(kFmtE2M3, kFmtE2M1, kTileBytes, kTileBytesE2M1);
  else MXP_PROBE_LAUNCH(kFmtE2M1, kFmtE2M1, kTileBytesE2M1, kTileBytesE2M1);
#undef MXP_PROBE_LAUNCH
  return mxp::launch_status();
}
