// Geometry of the packed int8 operands shared by the pre-quantization, packing and GEMM kernels.
//
// Both GEMM operands (activation codes Xq [M][K] and transposed weight codes Wt [N][K]) live in
// HBM in the order in which a GEMM workgroup pulls them into LDS: rows are grouped into panels of
// 256, K into slabs of 64 bytes, and one (panel, slab) block of 256 rows x 64 bytes = 16 KB is
// contiguous.  A panel's blocks follow each other along K, so a workgroup streams one contiguous
// run per operand.  Inside a 64-byte row the four 16-byte chunks are stored XOR-swizzled with a
// function of the row: the LDS image of a block is the block verbatim, and the fragment reads
// of the MFMA lanes (one 16-byte chunk per lane, 32 consecutive rows) are free of bank conflicts.
// Rows are padded to a multiple of 256 and K to a multiple of 128; weight padding is zero.
#pragma once
#include "common.h"

namespace mmd8 {

constexpr uint32_t kPackedLayoutTag = 0x6d6d0002u;   // panels of 256 rows x slabs of 64 B, swizzled chunks
constexpr int kPackK = 128;                           // K padded to a multiple of this many bytes
constexpr int kPackN = 256;                           // N (weights) and M (activations) padded to this many rows
constexpr int kPanelRows = 256;
constexpr int kSlabBytes = 64;
constexpr int kBlockBytes = kPanelRows * kSlabBytes;  // 16 KB

__host__ __device__ constexpr inline int packed_k(int K) { return round_up(K, kPackK); }
__host__ __device__ constexpr inline int packed_n(int N) { return round_up(N, kPackN); }

// chunk swizzle: distinct for rows {r, r+2, r+4, r+6} and for rows {r, r+4, r+8, r+12}
__host__ __device__ constexpr inline int chunk_swizzle(int r) {
  return (((r >> 1) ^ (r >> 3)) & 1) | (((r >> 2) & 1) << 1);
}
// byte offset of the 16-byte chunk that holds bytes [16 c, 16 c + 16) of slab `slab` of row `row`
__host__ __device__ constexpr inline size_t packed_chunk_offset(int row, int slab, int c, int n_slabs) {
  return ((size_t)(row >> 8) * n_slabs + slab) * kBlockBytes + (size_t)(row & 255) * kSlabBytes +
         ((c ^ chunk_swizzle(row)) << 4);
}
// byte offset of element (row, k)
__host__ __device__ constexpr inline size_t packed_offset(int row, int k, int n_slabs) {
  return packed_chunk_offset(row, k >> 6, (k & 63) >> 4, n_slabs) + (k & 15);
}

}  // namespace mmd8
