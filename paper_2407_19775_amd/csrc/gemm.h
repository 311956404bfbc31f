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
// Critical columns beyond those slabs.  Gathering them column by column in the GEMM's epilogue (gather_outlier_columns)
// costs 0.44 us per column on a 2048 x 4096 x 12288 call: a 2-byte element of a column of X pulls a whole line,
// a weight code a quarter of one, and every tile does it again.  So the kernel that lists the critical columns
// gathers them once into further slabs of the same layout, Xg / Wg (g_slabs of them per panel, up to kGatherMax
// columns, fewer where the weight side would exceed kGatherWeightBytesMax), and the GEMM takes those through its
// ring behind the first crit_slabs: 1.5 us per slab of 32 columns on that call.  Only columns beyond both are
// gathered in the epilogue, and from dense_from critical columns on the GEMM makes a second, fp16 pass over K
// instead (dense_critical_columns in gemm_kernels.hip, 3.7 us per 64-column slab of K on that call): where that is
// cheaper, the measured costs applied as ratios.
constexpr int kGatherMax = 2048;
constexpr size_t kGatherWeightBytesMax = (size_t)96 << 20;
struct CriticalPlan {
  int g_slabs;      // further slabs of 32 critical columns in Xg / Wg, 0: none
  int dense_from;   // critical columns from which a call takes the dense pass
};
inline CriticalPlan plan_critical_columns(int n_slabs, size_t Npad, bool further_slabs) {
  const double dense = 3.7 * n_slabs, per_slab_column = 1.5 / kOutlierSlab, per_gathered_column = 0.44;
  CriticalPlan p = {0, 0};
  if (further_slabs) {
    size_t cols = (size_t)n_slabs * 32;                              // half of the columns at most
    if (cols > (size_t)kGatherMax) cols = kGatherMax;
    const size_t fit = kGatherWeightBytesMax / (Npad * 2);
    if (cols > fit) cols = fit;
    p.g_slabs = (int)(cols / kOutlierSlab);
  }
  const int in_slabs = kOutlierSlab * (kCriticalSlabs + p.g_slabs);
  const double left = dense - in_slabs * per_slab_column;
  p.dense_from = in_slabs + (left > 0 ? (int)(left / per_gathered_column) : 0);
  return p;
}
// Whether a call takes the dense pass for its critical columns.  Then no fp16 slab is prepared or read at all.  The
// same decision in the kernel that prepares the slabs and in the GEMM, from the count that both read; never with
// original 16-bit weight rows (the dense pass multiplies the weight codes).
__host__ __device__ constexpr inline bool dense_critical_path(int n_out, int crit_slabs, int dense_from, bool master_rows) {
  return !master_rows && n_out > kOutlierSlab * crit_slabs && n_out >= dense_from;
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
  const uint16_t* Xg;    // further fp16 slabs of critical columns, laid out like Xo with g_slabs per panel, or null
  const uint16_t* Wg;    // likewise for the weight side (both or neither)
  int g_slabs;
  int dense_from;        // critical columns from which the call takes the dense pass (plan_critical_columns)
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
