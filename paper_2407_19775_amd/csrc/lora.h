// Low-rank adapter on top of the int8 layer (see lora_kernels.hip).
#pragma once
#include "common.h"

namespace mmd8 {

// The low-rank operands travel through the GEMM's slab ring as fp16 slabs of 32 columns behind the slabs of the
// critical columns; the rank limit bounds the workspace (two slabs per row of both operands).
constexpr int kLoraMaxRank = MMD8_MAX_LORA_RANK;
__host__ __device__ constexpr inline int lora_slabs(int r) { return ceil_div(r, 32); }

struct LoraArgs {
  const uint16_t* X;     // [M][ldx] fp16
  int M, K, ldx;
  const uint16_t* A;     // [r][K] fp16
  const uint16_t* B;     // [N][r] fp16
  int r, N;
  uint16_t* T;           // [M][kLoraMaxRank] fp16, columns >= r zero: T = f16(X A^T)
  uint16_t* T_user;      // [M][r] or null
  uint16_t* Xo;          // fp16 slabs of the GEMM's activation side (slabs 0 .. crit_slabs - 1: critical columns), or null
  uint16_t* Wo;          // likewise, weight side
  int f_slabs;           // slabs per panel in Xo / Wo: crit_slabs + lora_slabs(r)
  int crit_slabs;        // slabs of the critical columns in front of the adapter's
};
// how K is split between workgroups for this shape (depends on the device's CU count)
struct LoraPlan {
  int splits, steps_per_split;   // ranges of K, each this many 64-column steps
  size_t partial_bytes;          // fp32 [splits][M][kLoraMaxRank] when splits > 1
};
LoraPlan plan_lora(int M, int K);
// T for every row (and, where Xo is given, T and B in the GEMM's slab layout)
hipError_t launch_lora_down(const LoraArgs& a, const LoraPlan& plan, float* partial, hipStream_t stream);

}  // namespace mmd8
