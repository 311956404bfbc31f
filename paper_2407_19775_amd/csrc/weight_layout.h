// Geometry of the packed operands shared by the pre-quantization, packing and GEMM kernels.
#pragma once
#include "common.h"

namespace mmd8 {

constexpr uint32_t kPackedLayoutTag = 0x6d6d0001u;   // transposed [Npad][Kpad], zero padded
constexpr int kPackK = 128;                           // K padded to a multiple of this many bytes
constexpr int kPackN = 256;                           // N (weights) and M (activations) padded to this many rows

__host__ __device__ constexpr inline int packed_k(int K) { return round_up(K, kPackK); }
__host__ __device__ constexpr inline int packed_n(int N) { return round_up(N, kPackN); }

}  // namespace mmd8
