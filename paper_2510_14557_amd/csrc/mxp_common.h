// Internal helpers shared by the HIP translation units of libmxp (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include "mxp.h"

namespace mxp {

constexpr int kBlock = 32;    // elements per MX block (Sec. 2)
constexpr int kNumCU = 256;   // MI355X compute units (whole device): what the persistent launches are laid out for
constexpr int kNumXCD = 8;    // ... in 8 XCDs, each with its own L2; the hardware deals workgroups to them round-robin

// Shape of the current device, asked of the runtime once per device: compute units and XCDs.  The XCD-aware work lists of
// the tiled product are laid out for kNumCU / kNumXCD; on any other shape (a partitioned device) the entry points take
// the plain, non-persistent kernel instead.  The grid caps of the streaming kernels only use kNumCU as a size hint.
struct Chip {
  int cus, xcds;
  bool whole_mi355x() const { return cus == kNumCU && xcds == kNumXCD; }
};
Chip chip();

// Image stores are ordinary (cached) stores, not streaming ones: the GEMM reads the image right after it is written,
// and measured 10 % faster behind image kernels that store this way.
#define MXP_IMAGE_STORE(v, p) (*(p) = (v))

// six- and eight-bit formats (mxp_wide.hip)
bool is_wide_format(int fmt);
inline bool plain_wide_format(int fmt) { return fmt == MXP_FMT_MXFP6 || fmt == MXP_FMT_MXFP8; }   // no index byte
int wide_quantize_launch(const void* src, int src_dtype, int64_t rows, int64_t K, int64_t ld_src, int fmt, uint8_t* elems,
                         uint8_t* scales, uint8_t* bm_idx, hipStream_t stream);
int wide_dequantize_launch(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows,
                           int64_t K, void* dst, int dst_dtype, int64_t ld_dst, hipStream_t stream);

int prepack_fp6_launch(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows, int64_t K,
                       int n_seg, uint32_t res_mask, void* image, hipStream_t stream);
int prepack_seg_launch(const uint8_t* elems, const uint8_t* scales, const uint8_t* bm_idx, int fmt, int64_t rows, int64_t K, int n_seg,
                       uint32_t roles, void* image, hipStream_t stream);
int prepack_fp8_launch(const uint8_t* elems, const uint8_t* scales, int64_t rows, int64_t K, void* image, hipStream_t stream);

// the bf16-MFMA product of two quantized operands de-converted inside the kernel (mxp_w4a16.hip): pairs with an eight-bit
// format, and a six-bit format next to MXFP4++
int deconv_gemm_launch(int64_t M, int64_t N, int64_t K, const uint8_t* ae, const uint8_t* as, const uint8_t* ai, int fmtA,
                       const uint8_t* be, const uint8_t* bs, const uint8_t* bi, int fmtB, void* D, int d_dtype, int64_t ldd,
                       hipStream_t s);

// Longest reduction the product entry points take: the tiled kernel addresses an 8-tile run of an operand image with a
// 32-bit lane offset, and a six-bit + product lays up to four K segments side by side.
constexpr int64_t kMaxGemmK = (int64_t)1 << 21;
// Checks shared by every mxp_gemm* entry point: dtype, shape, K limit, D non-null and aligned to its element type.
int check_gemm(int64_t M, int64_t N, int64_t K, const void* D, int d_dtype, int64_t ldd, int64_t max_k = kMaxGemmK);
// D[M][N] = 0 (the product over an empty K).
int zero_output(void* D, int d_dtype, int64_t M, int64_t N, int64_t ldd, hipStream_t s);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// A kernel that takes more than 64 KiB of dynamic LDS has to be told so through its function attribute, on every device it
// is launched on: done at the first launch per device (one bit per device in a word of the kernel's own; threads that get
// there together set the same attribute twice).
template <auto Kernel>
inline void allow_dynamic_lds(int bytes) {
  static std::atomic<uint64_t> done{0};
  int dev = 0;
  const bool known = hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64;
  const uint64_t bit = known ? (uint64_t)1 << dev : 0;
  if (known && (done.load(std::memory_order_relaxed) & bit)) return;
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (known) done.fetch_or(bit, std::memory_order_relaxed);
}

inline int launch_status() {
  return hipGetLastError() == hipSuccess ? MXP_OK : MXP_ERR_HIP;
}

// ---- MFMA-ready image geometry --------------------------------------------------------------------------------
// Unit tile = 32 rows x 64 K = 64 blocks, one per lane of a 32x32x64 block-scaled MFMA operand
// (lane l <-> row l % 32, K-block l / 32).  A tile stores, for its 64 lanes, first the low 16 bytes of every
// lane's 24-byte E2M3 block, then the high 8 bytes:  [64 x 16 B][64 x 8 B] = 1536 B.
// Tiles are ordered [row_tile][k_tile]; rows are padded to a multiple of 256 and K to a multiple of 128.
// Scales follow the element tiles: for each group of 4 row tiles (128 rows) and each k_tile, 64 dwords, lane l's
// dword holding the E8M0 bytes of its block in row tiles 4g+0..3 (byte j = row tile 4g+j).
constexpr int kTileRows = 32;
constexpr int kTileK = 64;
constexpr int kTileBytes = 1536;
// A plain MXFP4 operand (no BM) can stay in 4-bit codes: the MFMA takes E2M1 for one operand and E2M3 for the other at
// the same rate.  Its tile is the 64 lanes' 16-byte canonical blocks, [64 x 16 B] = 1024 B; everything else is the same.
constexpr int kTileBytesE2M1 = 1024;
// An MXFP4++ operand (Sec. 4.3) has two scales per block, 2^delta apart.  In units of 2^(shared_exp - delta + 2) every
// one of its elements is an FP8 E4M3 number (ordinary elements 0.125 ... 1.5, the BM up to 1.875 * 2^7), so an image of
// E4M3 codes, 32 bytes per lane = [64 x 16 B][64 x 16 B] = 2048 B per tile, carries the block exactly.
constexpr int kTileBytesE4M3 = 2048;
constexpr int kRowPad = 256;
constexpr int kKPad = 128;

struct ImageGeom {
  int64_t rows_p, K_p;      // padded sizes
  int64_t row_tiles, k_tiles;
  int64_t elem_bytes;       // bytes of the element part
  int64_t scale_bytes;      // bytes of the scale part
  __host__ __device__ int64_t total() const { return elem_bytes + scale_bytes; }
};

__host__ __device__ inline ImageGeom image_geom(int64_t rows, int64_t K, int tile_bytes = kTileBytes) {
  ImageGeom g;
  g.rows_p = (rows + kRowPad - 1) / kRowPad * kRowPad;
  g.K_p = (K + kKPad - 1) / kKPad * kKPad;
  g.row_tiles = g.rows_p / kTileRows;
  g.k_tiles = g.K_p / kTileK;
  g.elem_bytes = g.row_tiles * g.k_tiles * (int64_t)tile_bytes;
  g.scale_bytes = (g.row_tiles / 4) * g.k_tiles * 256;
  return g;
}

// Workgroup -> (row tile, group of 4 k-tiles) for the kernels that write an image.  The hardware deals workgroups
// round-robin to the 8 XCDs (each with its own L2), so workgroup c runs on XCD c % 8.  All patches of four consecutive
// row tiles (128 rows: the rows whose scale bytes share the image's scale dwords, and whose canonical scale / index
// bytes share cache lines along K) go to one XCD, close together in launch order, so that those partially written or
// partially read lines are merged in one L2 instead of being moved once per XCD.
struct PatchMap {
  int64_t rt, kg;
  bool valid;
};
__device__ inline PatchMap patch_of_workgroup(uint32_t c, uint32_t k_groups, uint32_t row_tile_groups) {
  const uint32_t x = c & 7u, j = c >> 3;
  const uint32_t per = 4u * k_groups;
  const uint32_t gi = (j / per) * 8u + x, rem = j % per;
  PatchMap m;
  m.rt = (int64_t)gi * 4 + rem / k_groups;
  m.kg = rem % k_groups;
  m.valid = gi < row_tile_groups;
  return m;
}
inline int64_t patch_grid(int64_t k_groups, int64_t row_tile_groups) {
  return 8 * 4 * k_groups * ((row_tile_groups + 7) / 8);
}

// E4M3 image codes (Sec. 4.3): an E2M1 magnitude m stands in the image as m / 4, an FP8 E4M3 number.
constexpr uint64_t kE2M1QuarterAsE4M3 = 0x3C3834302C282000ull;   // byte m = E4M3 code of (E2M1 magnitude m) / 4

__device__ __forceinline__ uint32_t nibbles4_to_e4m3(uint32_t h) {   // low 16 bits: 4 nibbles -> 4 bytes
  uint32_t out = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t n = (h >> (4 * i)) & 15u;
    const uint32_t code = (uint32_t)(kE2M1QuarterAsE4M3 >> (8u * (n & 7u))) & 0xFFu;
    out |= (code | ((n & 8u) << 4)) << (8 * i);
  }
  return out;
}

}  // namespace mxp
