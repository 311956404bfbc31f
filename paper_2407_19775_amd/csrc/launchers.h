// Host-side entry points of the kernel files, as the ABI layer (api.hip) calls them, and the argument
// blocks they share.  Each launcher is defined next to its kernels.
#pragma once
#include "common.h"

namespace mmd8 {

// ---- codec_kernels.hip
const float* code_table_host();        // the 256 code values, ascending
const float* code_midpoints_host();    // the 255 decision thresholds between neighbouring code values
hipError_t launch_quantize_blockwise(const uint16_t* x, size_t n, int block, uint8_t* codes, float* absmax,
                                     hipStream_t stream);
hipError_t launch_dequantize_blockwise(const uint8_t* codes, const float* absmax, size_t n, int block, uint16_t* out,
                                       hipStream_t stream);

// the same with the block scales stored as the fp16 numbers they are (2 bytes per block)
hipError_t launch_quantize_blockwise_h(const uint16_t* x, size_t n, int block, uint8_t* codes, uint16_t* absmax,
                                       hipStream_t stream);
hipError_t launch_dequantize_blockwise_h(const uint8_t* codes, const uint16_t* absmax, size_t n, int block, uint16_t* out,
                                         hipStream_t stream);

// ---- weight_kernels.hip
hipError_t launch_col_absmax(const uint16_t* W, int K, int N, int ldw, float* c, hipStream_t stream);
hipError_t launch_weight_quant_pack(const uint16_t* W, int K, int N, int ldw, const float* c, int8_t* Wt,
                                    hipStream_t stream);
hipError_t launch_weight_unpack(const int8_t* Wt, int K, int N, int8_t* Wq, hipStream_t stream);

// ---- activation_kernels.hip
struct PackOutliers {   // the critical columns: compaction outputs and the operands of their fp16 slab
  int32_t* idx;          // ascending critical columns
  int32_t* n_out;        // [1]
  uint8_t* mask;         // [Kpad] 1 = critical column (padding 0)
  uint8_t* tap_mask;     // [K] or null
  int32_t* tap_idx;      // or null
  int32_t* tap_n;        // or null
  const int8_t* Wt;
  const float* c;
  int N;
  uint16_t* Xo;
  uint16_t* Wo;
  int f_slabs;           // fp16 slabs per panel in Xo / Wo
  int crit_slabs;        // ... of which the first crit_slabs are for critical columns, 32 each (the rest: an adapter's)
  // Alternative reading of where the 16-bit weights of the critical dimensions come from: null (re-created from
  // the codes, f16(Wt c / 127)), or the original fp16 weights W[k * ldw + n], whose rows are then used as they are.
  const uint16_t* W_master;
  int ldw;
  uint16_t* Xg;          // further slabs of critical columns (gemm.h), laid out like Xo with g_slabs per panel, or null
  uint16_t* Wg;          // likewise for the weight side
  int g_slabs;
  int dense_from;        // critical columns from which the GEMM takes the dense pass (no slab is prepared then)
};
struct CodedInput {     // activations in their blockwise-coded form
  const uint8_t* codes;
  const float* absmax;
  int block;
};
hipError_t launch_fill_u32(uint32_t* p, uint32_t v, int n, hipStream_t stream);
hipError_t launch_scan(const uint16_t* X, int M, int K, int ldx, uint32_t th, int Kpad, uint8_t* flag, float* r,
                       hipStream_t stream);
// Alternative reading of the row scale: r[m] = max |X[m,k]| over the columns that are not critical (flag 0); needs
// the flags of all rows, i.e. runs after launch_scan.  Overwrites the scan's r.
hipError_t launch_row_absmax_noncritical(const uint16_t* X, int M, int K, int ldx, const uint8_t* flag, float* r,
                                         hipStream_t stream);
hipError_t launch_pack(const uint16_t* X, int M, int K, int ldx, const uint8_t* flag, const float* r, int8_t* Xq,
                       int Kpad, int8_t* tap_xq, uint16_t* Xf, const PackOutliers& o, hipStream_t stream,
                       bool list_columns = true);   // false (with Xf): codes and fp16 copy only, nothing of `o` is written
// One-pass preparation for inputs taller than the decode kernels take; prep_fits is false when K is too
// large for a row to be held in the registers of one workgroup (the caller then uses scan + pack).
bool prep_fits(int K);
bool prep_from_codes_fits(int K);   // likewise for launch_prep with coded activations (a smaller bound)
// coded: null, or the blockwise-coded form of the activations (X is then written, not read).
hipError_t launch_prep(uint16_t* X, int M, int K, int ldx, uint32_t th, int Kpad, uint8_t* flag, float* r,
                       int8_t* Xq, int8_t* tap_xq, const PackOutliers& o, const CodedInput* coded, void* event_mid,
                       hipStream_t stream);   // event_mid: null, or a hipEvent_t recorded between the two kernels

}  // namespace mmd8
