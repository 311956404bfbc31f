// Arguments and launcher of the decode-shaped (at most 64 rows) GEMM, see skinny_kernels.hip.
#pragma once
#include "common.h"
#include "gemm.h"

namespace mmd8 {

constexpr int kSkinnyMaxM = 64;

// Xf, the 16-bit operand of the decode kernels, is stored per 64-column slab as 8 KB =
// [32-row group 0..1][piece p = 2 (k-step) + t][lane = 32 (lane group) + row % 32] x 8 halves, which is
// the order in which the lanes of v_mfma_f32_32x32x16_f16 take them next to the int8 fragments
// (lane group g of k-step ks holds columns 32 ks + 16 g + 8 t .. + 8 in piece t).  Byte offset of the
// 8 halves that start at column k (a multiple of 8) of row m:
__host__ __device__ constexpr inline size_t xf_group_offset(int m, int k) {
  return (size_t)(k >> 6) * 8192 + (size_t)(m >> 5) * 4096 + (size_t)(2 * ((k >> 5) & 1) + ((k >> 3) & 1)) * 1024 +
         (size_t)(32 * ((k >> 4) & 1) + (m & 31)) * 16;
}

struct SkinnyPlan {
  int waves;               // 0: 32-column tiles (up to 16 rows); 4 or 8: panel kernel with that many waves per workgroup
  int n_slabs, tiles_n, splits, slabs_per_split;
  size_t partial_bytes;    // fp32 [splits][M][N] when splits > 1
};
// how the K range is split between workgroups for this shape (depends on the device's CU count)
SkinnyPlan plan_skinny(int M, int K, int N);

struct SkinnyArgs {
  const int8_t* Xq;       // activation codes, blocked layout, rows 0..63 of panel 0
  const int8_t* Wt;       // weight codes, blocked layout
  const uint16_t* Xf;     // fp16 X with the non-critical columns (and the K padding) zeroed, blocked: xf_group_offset
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
  uint8_t* flag_reset_late;   // likewise, by the kernel that sums the splits: for calls whose `mask` is the flags themselves
  const uint16_t* lora_T; // low-rank term T B^T added to the output: T [M][lora_ldt] fp16, B [N][lora_r] fp16
  const uint16_t* lora_B;
  int lora_ldt, lora_r;   // lora_r == 0: none
  // The output with a residual added, H = f16(Y + residual), and / or leaving in blockwise-coded form (the rows
  // of this call as one flattened tensor of M N elements; Y, where given, is then contiguous: ldy == N).
  const uint16_t* residual;   // [M][ldr] fp16 or null
  int ldr;
  int gelu;               // 1: Y := f16(gelu(Y)) before a residual is added
  uint8_t* codes;         // [M N] or null
  float* code_absmax;     // [ceil(M N / code_block)]
  int code_block;         // a multiple of 64, at most 4096
  // A few rows: the panel kernel prepares its activation operands itself (no scan and pack kernels before it):
  // every workgroup finds the row scales from X, and the codes / critical columns of its own K range.
  // Then Xq, Xf, mask and r are not read.
  const uint16_t* X;      // [M][ldx] fp16, or null: operands prepared by the pack kernel
  int ldx, K;
  uint32_t th;            // fp16 pattern of the threshold
  int n_slabs, tiles_n, slabs_per_split;   // filled by the launcher
};
constexpr int kPanelPrepMaxM = 8;          // rows up to which the panel kernel can prepare its own operands
constexpr int kPanelPrepMaxSlabs = 128;    // ... slabs per workgroup (one flag per column in LDS)
constexpr int kPanelPrepMaxRowSlabs = 256; // ... and rows x slabs per workgroup (its columns of X are held in LDS: 32 KB)
// whether launch_gemm_skinny may be given X instead of packed operands for this plan
inline bool panel_prep_fits(int M, const SkinnyPlan& plan) {
  return M <= kPanelPrepMaxM && plan.waves != 0 && plan.slabs_per_split <= kPanelPrepMaxSlabs &&
         M * plan.slabs_per_split <= kPanelPrepMaxRowSlabs;
}

hipError_t launch_gemm_skinny(SkinnyArgs a, const SkinnyPlan& plan, hipStream_t stream);

// One or two rows, whole layer in one kernel (k_gemm_rows): a workgroup owns 32 output columns and its eight
// waves share out the K range, so nothing is split between workgroups and no second kernel adds partial
// outputs.  The rows' codes and fp16 critical columns for the whole of K live in LDS (3 bytes per element).
// Needs a.X (the kernel prepares its operands); takes bias, the low-rank term of an adapter, GELU and a residual;
// no coded output (the encoder follows it).
constexpr int kRowsMaxM = 2;   // (the kernel is written for any small number; measured with 4: 78.8 us per 7B layer at four rows against 76 with the split-K kernels)
constexpr int kRowsMaxOperandBytes = 66 * 1024;   // two rows of K = 11008; two workgroups per compute unit still fit
inline bool rows_kernel_fits(int M, int Kpad) { return M <= kRowsMaxM && 3 * M * Kpad <= kRowsMaxOperandBytes; }
hipError_t launch_gemm_rows(SkinnyArgs a, hipStream_t stream);
hipError_t prepare_rows_kernels();   // its LDS attribute on the current device (else set by the first launch)

}  // namespace mmd8
