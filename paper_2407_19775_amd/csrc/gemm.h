// Arguments and launcher of the fused int8 GEMM (see gemm_kernels.hip).
#pragma once
#include "common.h"

namespace mmd8 {

struct GemmArgs {
  const int8_t* Xq;      // [Mpad][Kpad]
  const int8_t* Wt;      // [Npad][Kpad]
  int M, N, Kpad;
  const float* r;        // [M]
  const float* c;        // [N]
  const uint16_t* bias;  // [N] or null
  const uint16_t* X;     // [M][ldx] fp16 (critical columns are read from here)
  int ldx;
  const int32_t* idx;    // ascending critical columns
  const int32_t* n_out;  // their count
  uint16_t* Y;
  int ldy;
  int32_t* tap_acc;      // [M][N] or null
  int tiles_m, tiles_n;
};


// variant selects a tile configuration; every variant computes the same result.
hipError_t launch_gemm_mixed(const GemmArgs& a, int variant, hipStream_t stream);

}  // namespace mmd8
