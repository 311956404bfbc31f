// Arguments and launcher of the decode-shaped (at most 64 rows) GEMM, see skinny_kernels.hip.
#pragma once
#include "common.h"
#include "gemm.h"

namespace mmd8 {

constexpr int kSkinnyMaxM = 64;

struct SkinnyPlan {
  int n_slabs, tiles_n, splits, slabs_per_split;
  size_t partial_bytes;    // fp32 [splits][M][N] when splits > 1
};
// how the K range is split between workgroups for this shape (depends on the device's CU count)
SkinnyPlan plan_skinny(int M, int K, int N);

struct SkinnyArgs {
  const int8_t* Xq;       // activation codes, blocked layout, rows 0..63 of panel 0
  const int8_t* Wt;       // weight codes, blocked layout
  const uint16_t* Xf;     // [64][Kpad] fp16: X with the non-critical columns (and the K padding) zeroed
  const uint8_t* mask;    // [Kpad] 1 = critical column
  int M, N, Kpad;
  const float* r;         // [>= 64]
  const float* c;         // [N]
  const uint16_t* bias;   // [N] or null
  uint16_t* Y;
  int ldy;
  float* partial;         // workspace for split K
  int32_t* tap_acc;       // [M][N] or null
  uint8_t* flag_reset;    // [Kpad] column flags of the scan: zeroed again by workgroup 0
  int n_slabs, tiles_n, slabs_per_split;   // filled by the launcher
};

hipError_t launch_gemm_skinny(SkinnyArgs a, const SkinnyPlan& plan, hipStream_t stream);

}  // namespace mmd8
