// Arguments and launcher of the fused int8 GEMM (see gemm_kernels.hip).
#pragma once
#include "common.h"

namespace mmd8 {

// Critical columns handled on the fast path: they travel as extra 64-byte K-slabs of fp16 operands, 32 columns
// each, prepared once per call by the pack kernels; they ride through the GEMM's slab ring behind the codes.
// Columns beyond 32 kCriticalSlabs (inputs where a large share of the dimensions is critical) are multiplied 64
// at a time after the ring has drained: fp16 activations straight from X, weight codes converted in registers.
constexpr int kOutlierSlab = 32;
constexpr int kCriticalSlabs = 8;
// Whether a call takes the dense path for its critical columns: more of them than the slabs hold, and at least twelve
// per 64-column slab of K on average (below that, gathering the columns beyond the slabs one by one is cheaper than
// a pass over every slab: 0.44 us per column against 3.7 us per slab on a 2048 x 4096 x 12288 call, which meet at
// 800 columns of 4096).  Then no fp16 slab is prepared or read at all.  The same decision in the kernel that
// prepares the slabs and in the GEMM, from the count that both read; never with original 16-bit weight rows (the
// dense path multiplies the weight codes).
__host__ __device__ constexpr inline bool dense_critical_path(int n_out, int crit_slabs, int n_slabs, bool master_rows) {
  return !master_rows && n_out > kOutlierSlab * crit_slabs && n_out >= 12 * n_slabs;
}

struct GemmArgs {
  const int8_t* Xq;      // activation codes, blocked layout (operand_layout.h), Mpad x Kpad
  const int8_t* Wt;      // weight codes, blocked layout, Npad x Kpad
  int M, N, Kpad;
  const float* r;        // [Mpad + 256]
  const float* c;        // [N]
  const uint16_t* bias;  // [N] or null
  const uint16_t* X;     // [M][ldx] fp16 (critical columns beyond the slab are read from here)
  int ldx;
  const int32_t* idx;    // ascending critical columns
  const int32_t* n_out;  // their count
  const uint8_t* mask;   // [Kpad] 1 = critical column (the copy of the flags that the compaction publishes)
  const uint16_t* Xo;    // f_slabs slabs of fp16 per row, each blocked like a slab of codes: X[m, O_j], zero for j >= n_out
  const uint16_t* Wo;    // likewise: f16(Wt[n, O_j] c[n] / 127), zero for j >= n_out
  int f_slabs;           // fp16 slabs per panel in Xo / Wo: crit_slabs for the critical columns, then those of a low-rank
                         // adapter (at most 2), whose operands are multiplied in the same way
  int crit_slabs;        // slabs set aside for critical columns (1 .. kCriticalSlabs); ceil(min(n_out, 32 crit_slabs) / 32) are in use
  uint16_t* Y;           // may be null when `codes` is given (only the coded form of the output is wanted)
  int ldy;
  // The output leaving in coded form (the shard's last linear): H = Y, or f16(Y + residual) when a residual is
  // given; H is what Y receives and what is encoded blockwise, the blocks running over the flattened [M][code_ld]
  // tensor.  Blocks of 64, 128 or 256 elements that divide N and the tile width, so that no block leaves a tile.
  const uint16_t* residual;   // [M][ldr] fp16 or null
  int ldr;
  int gelu;              // 1: Y := f16(gelu(Y)) (exact, erf-based), before a residual is added
  uint8_t* codes;        // [M][code_ld] or null
  float* code_absmax;    // [M code_ld / block]
  int code_ld;           // elements per row of the coded tensor
  int code_log_block;    // 6, 7 or 8
  int32_t* tap_acc;      // [M][tap_ld] or null
  int tap_ld;
  int tiles_m, tiles_n;
  uint8_t* flag_reset;   // [Kpad] column flags of the scan: zeroed again by workgroup 0
  // Alternative reading: the 16-bit weights of the critical dimensions are the rows of the original fp16 matrix
  // W[k * ldw_master + n] (null: they are re-created from the codes).  Wo was then gathered from it as well.
  const uint16_t* W_master;
  int ldw_master;
};

// Workgroup 0 of the kernel that ends a call puts the scan's column flags back to zero (the next
// call's scan is ordered after it on the stream).
__device__ inline void reset_column_flags(uint8_t* flags, int Kpad) {
  if (blockIdx.x != 0 || flags == nullptr) return;
  v4u* p = reinterpret_cast<v4u*>(flags);
  const int n = Kpad / 16;
  for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = v4u{0, 0, 0, 0};
}

// variant selects a tile configuration, 0..5 (anything else: automatic); every variant computes the same result.
hipError_t launch_gemm_mixed(const GemmArgs& a, int variant, hipStream_t stream);
// sets the LDS attribute of every GEMM kernel on the current device (otherwise done by a kernel's first launch,
// which must then not happen while a stream is being captured)
hipError_t prepare_gemm_kernels();

}  // namespace mmd8
