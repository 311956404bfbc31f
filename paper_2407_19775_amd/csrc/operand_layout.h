// Geometry of the packed int8 operands shared by the pre-quantization, packing and GEMM kernels.
//
// Both GEMM operands (activation codes Xq [M][K] and transposed weight codes Wt [N][K]) live in
// HBM in the order in which the kernels consume them.  Rows are grouped into panels of 256, K
// into slabs of 64 bytes; one (panel, slab) block of 256 rows x 64 bytes = 16 KB is contiguous,
// and a panel's blocks follow each other along K, so a workgroup streams one contiguous run per
// operand.  Inside a block, each group of 32 rows (2 KB) is stored fragment-major: first the
// 32 x 32-byte half slab of k-step 0, then that of k-step 1, each as the 64 sixteen-byte pieces
// that the 64 lanes of a v_mfma_i32_32x32x32_i8 operand hold (lane = 32 (piece of the half slab)
// + row).  The LDS image of a block is the block verbatim, a wave's fragment read is 1 KB of
// consecutive addresses (no bank conflicts, no swizzle), and a kernel that feeds the MFMA straight
// from HBM (decode shapes) reads 1 KB contiguous per instruction.
// Rows are padded to a multiple of 256 and K to a multiple of 128; weight padding is zero.
#pragma once
#include "common.h"

namespace mmd8 {

constexpr uint32_t kPackedLayoutTag = 0x6d6d0003u;   // panels of 256 rows x slabs of 64 B, fragment-major groups of 32 rows
constexpr int kPackK = 128;                           // K padded to a multiple of this many bytes
constexpr int kPackN = 256;                           // N (weights) and M (activations) padded to this many rows
constexpr int kPanelRows = 256;
constexpr int kSlabBytes = 64;
constexpr int kBlockBytes = kPanelRows * kSlabBytes;  // 16 KB

__host__ __device__ constexpr inline int packed_k(int K) { return round_up(K, kPackK); }
__host__ __device__ constexpr inline int packed_n(int N) { return round_up(N, kPackN); }

// byte offset of the 16-byte piece that holds bytes [16 c, 16 c + 16) of slab `slab` of row `row`
__host__ __device__ constexpr inline size_t packed_chunk_offset(int row, int slab, int c, int n_slabs) {
  return ((size_t)(row >> 8) * n_slabs + slab) * kBlockBytes + (size_t)((row & 255) >> 5) * 2048 + (size_t)(c >> 1) * 1024 +
         (size_t)(((c & 1) << 5) | (row & 31)) * 16;
}
// byte offset of element (row, k)
__host__ __device__ constexpr inline size_t packed_offset(int row, int k, int n_slabs) {
  return packed_chunk_offset(row, k >> 6, (k & 63) >> 4, n_slabs) + (k & 15);
}

}  // namespace mmd8
