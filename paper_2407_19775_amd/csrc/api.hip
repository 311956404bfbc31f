// C ABI of the mmd8 library: argument checks, workspace carving, kernel sequencing.
#include <math.h>
#include <string.h>

#include <mutex>

#include "common.h"
#include "gemm.h"
#include "launchers.h"
#include "lora.h"
#include "operand_layout.h"
#include "skinny.h"

namespace mmd8 {

int device_cu_count() {
  static std::mutex mu;
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  std::lock_guard<std::mutex> lock(mu);
  if (cached[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    cached[dev] = cus;
  }
  return cached[dev];
}

// smallest fp16 bit pattern (non-negative) whose value is >= tau; 0x7c00 (+inf) if none is finite
static uint32_t threshold_pattern(float tau) {
  if (!(tau > 0.0f)) return 0;
  if (tau > 65504.0f) return 0x7c00u;
  // walk the exponent/mantissa of tau into an fp16 pattern rounded towards +inf
  uint32_t fb;
  memcpy(&fb, &tau, 4);
  const int exp = (int)((fb >> 23) & 0xff) - 127;
  const uint32_t man = fb & 0x7fffffu;
  if (exp < -24) return 1u;                                        // below the smallest subnormal
  if (exp < -14) {                                                 // subnormal range: value = m * 2^-24
    const uint64_t sig = (uint64_t)(0x800000u | man);              // tau = sig * 2^(exp - 23)
    const int drop = -exp - 1;                                     // tau / 2^-24 = sig >> drop, drop = 14..23
    uint32_t m = (uint32_t)(sig >> drop);
    if (sig & ((1ull << drop) - 1)) m += 1;                        // round up
    return m;                                                      // may reach 0x400 = smallest normal: still correct
  }
  uint32_t h = ((uint32_t)(exp + 15) << 10) | (man >> 13);
  if (man & 0x1fffu) h += 1;                                       // round up; a carry moves into the exponent correctly
  return h;
}

static inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

static int check_lora_rank(int r) { return (r >= 8 && r <= kLoraMaxRank && (r % 8) == 0) ? MMD8_OK : MMD8_E_SHAPE; }
static int check_linear_shape(int K, int N) {
  if (K < 16 || K > MMD8_MAX_K || (K % 16) != 0 || N < 8 || (N % 8) != 0) return MMD8_E_SHAPE;
  return MMD8_OK;
}

// Workspace layout.  The head (counters and the column flags, sized for the largest K so that
// its place does not depend on the shape) is standing state: zero between calls.
constexpr int kSkinnyChunkedMaxM = 2 * kSkinnyMaxM;   // most rows the decode kernels are used for (in passes of kSkinnyMaxM)
constexpr size_t kHeadCounters = 256;
constexpr size_t kHeadBytes = kHeadCounters + MMD8_MAX_K;
struct Workspace {
  int32_t* n_out;      // [1]
  uint8_t* flag;       // [Kpad] inside a region sized for the largest K: standing state
  uint8_t* mask;       // [Kpad]
  int32_t* idx;        // [Kpad]
  float* r;            // [Mpad + 256]
  uint16_t* xo;        // [Mpad][kOutlierSlab] per fp16 slab, blocked like the codes
  uint16_t* wo;        // [Npad][kOutlierSlab] per fp16 slab
  uint16_t* xg;        // further fp16 slabs of critical columns (tiled GEMM only): [Mpad][32] per slab, blocked like xo, or null
  uint16_t* wg;        // likewise [Npad][32] per slab
  int g_slabs;
  int dense_from;      // critical columns from which the tiled GEMM takes its dense pass
  int f_slabs;         // fp16 slabs: crit_slabs for the critical columns, then the low-rank operands of an adapter of rank r
  int crit_slabs;      // 32 critical columns each: kCriticalSlabs where the tiled GEMM is the usual path, else 1
  uint16_t* lora_t;    // adapter only: [M][kLoraMaxRank] fp16
  float* lora_part;    // adapter only: partial sums of the down-projection when K is split between workgroups
  int8_t* xq;          // Mpad x Kpad codes, blocked layout
  uint16_t* xf;        // decode path only: [64][Kpad] fp16
  float* partial;      // decode path only: split-K partial outputs
  uint16_t* h;         // coded output only, where the encoder runs as a kernel of its own: [M][N] fp16
  size_t bytes;
};
// r: rank of an adapter (0: none).  exit_block: block size of a coded output (0: plain output).
static bool exit_fuses(int M, int K, int N, int block);
// gathered_rows: room for further slabs of critical columns (not in the fixed-size static workspace)
static Workspace carve(void* base, int M, int K, int N, int r = 0, int exit_block = 0, bool gathered_rows = true) {
  const size_t Kpad = packed_k(K), Mpad = packed_n(M), Npad = packed_n(N);
  Workspace w;
  size_t off = 0;
  auto take = [&](size_t n) {
    uint8_t* p = base ? static_cast<uint8_t*>(base) + off : nullptr;
    off += round_up_sz(n, 256);
    return p;
  };
  uint8_t* counters = take(kHeadCounters);
  w.n_out = reinterpret_cast<int32_t*>(counters);
  w.flag = take(MMD8_MAX_K);
  w.mask = take(Kpad);
  w.idx = reinterpret_cast<int32_t*>(take(Kpad * 4));
  w.r = reinterpret_cast<float*>(take((Mpad + 256) * 4));
  // (up to 128 rows the decode kernels do the work and these slabs are not used, except by calls that force the
  // tiled GEMM: one slab, further critical columns through its gather loop)
  w.crit_slabs = M > kSkinnyChunkedMaxM ? kCriticalSlabs : 1;
  w.f_slabs = w.crit_slabs + lora_slabs(r);
  w.xo = reinterpret_cast<uint16_t*>(take(Mpad * kOutlierSlab * 2 * w.f_slabs));
  w.wo = reinterpret_cast<uint16_t*>(take(Npad * kOutlierSlab * 2 * w.f_slabs));
  // (the same count decides for the dense pass with and without the further slabs, so that a call gives the same
  // bits whichever workspace it runs in; a workspace without them gathers tile by tile up to that count)
  const CriticalPlan cp = plan_critical_columns((int)(Kpad / kSlabBytes), Npad, w.crit_slabs == kCriticalSlabs);
  w.g_slabs = gathered_rows ? cp.g_slabs : 0;
  w.dense_from = cp.dense_from;
  w.xg = w.g_slabs > 0 ? reinterpret_cast<uint16_t*>(take(Mpad * kOutlierSlab * 2 * w.g_slabs)) : nullptr;
  w.wg = w.g_slabs > 0 ? reinterpret_cast<uint16_t*>(take(Npad * kOutlierSlab * 2 * w.g_slabs)) : nullptr;
  if (!base) w.xg = w.wg = nullptr;
  w.xq = reinterpret_cast<int8_t*>(take(Mpad * Kpad));
  w.xf = nullptr;
  w.partial = nullptr;
  if (M > 0 && M <= kSkinnyChunkedMaxM) {
    const int Mc = M < kSkinnyMaxM ? M : kSkinnyMaxM;              // rows per pass of the decode kernels
    w.xf = reinterpret_cast<uint16_t*>(take((size_t)kSkinnyMaxM * Kpad * 2));
    size_t pb = plan_skinny(Mc, K, N).partial_bytes;
    // a low-rank term is added, an activation applied and a coded output encoded where the partial outputs are
    // summed: room for one partial output even when K is not split
    if (pb == 0) pb = (size_t)Mc * N * sizeof(float);
    if (pb) w.partial = reinterpret_cast<float*>(take(pb));
  }
  w.lora_t = r > 0 ? reinterpret_cast<uint16_t*>(take((size_t)M * kLoraMaxRank * 2)) : nullptr;
  w.lora_part = nullptr;
  if (r > 0 && M > 0) {
    const size_t lb = plan_lora(M, K).partial_bytes;
    if (lb) w.lora_part = reinterpret_cast<float*>(take(lb));
  }
  w.h = nullptr;
  if (exit_block > 0 && M > 0 && !exit_fuses(M, K, N, exit_block)) w.h = reinterpret_cast<uint16_t*>(take((size_t)M * N * 2));
  w.bytes = off;
  return w;
}
// A coded output is produced by the kernel that ends the layer when no block of it is shared between
// workgroups: the tiled GEMM needs blocks inside its 256-column tiles; the decode path encodes where it sums
// its partial outputs, any block size, as long as its second pass of 64 rows starts on a block boundary.  The
// first few rows are a single kernel with 32 columns per workgroup and nothing to sum afterwards: the encoder follows it.
static bool exit_fuses(int M, int K, int N, int block) {
  if (rows_kernel_fits(M, packed_k(K))) return false;
  if (M <= kSkinnyChunkedMaxM) return M <= kSkinnyMaxM || ((size_t)kSkinnyMaxM * N) % block == 0;
  return (block == 64 || block == 128 || block == 256) && N % block == 0;
}

// byte ranges [a, a + na) and [b, b + nb) share a byte
static inline bool ranges_overlap(const void* a, size_t na, const void* b, size_t nb) {
  const uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
  return pa < pb + nb && pb < pa + na;
}
// bytes from the first to one past the last element of a [rows][ld] fp16 matrix of `cols` columns
static inline size_t span_bytes(int rows, int cols, int ld) { return rows > 0 ? ((size_t)(rows - 1) * ld + cols) * 2 : 0; }

}  // namespace mmd8

using namespace mmd8;

extern "C" {

const char* mmd8_status_string(int status) {
  switch (status) {
    case MMD8_OK: return "ok";
    case MMD8_E_ARG: return "invalid argument (null, negative, misaligned, leading dimension, NaN threshold)";
    case MMD8_E_SHAPE: return "unsupported shape or block size";
    case MMD8_E_WORKSPACE: return "workspace too small";
    case MMD8_E_HIP: return "HIP runtime or launch error";
    case MMD8_E_VERSION: return "packed weights written under another layout version";
    default: return "unknown status";
  }
}

const float* mmd8_code_table(void) { return code_table_host(); }
const float* mmd8_code_midpoints(void) { return code_midpoints_host(); }

static int check_block(int block) { return (block >= 64 && block <= 4096 && block % 64 == 0) ? MMD8_OK : MMD8_E_SHAPE; }

int mmd8_quantize_blockwise(const mmd8_half* x, size_t n, int block, uint8_t* codes, float* absmax, void* stream) {
  if (check_block(block) != MMD8_OK) return MMD8_E_SHAPE;
  if (n == 0) return MMD8_OK;
  if (!x || !codes || !absmax || !aligned(x, 16) || !aligned(codes, 8) || !aligned(absmax, 4)) return MMD8_E_ARG;
  return launch_quantize_blockwise(x, n, block, codes, absmax, static_cast<hipStream_t>(stream)) == hipSuccess
             ? MMD8_OK
             : MMD8_E_HIP;
}

int mmd8_dequantize_blockwise(const uint8_t* codes, const float* absmax, size_t n, int block, mmd8_half* out,
                              void* stream) {
  if (check_block(block) != MMD8_OK) return MMD8_E_SHAPE;
  if (n == 0) return MMD8_OK;
  if (!codes || !absmax || !out || !aligned(out, 16) || !aligned(codes, 8) || !aligned(absmax, 4)) return MMD8_E_ARG;
  return launch_dequantize_blockwise(codes, absmax, n, block, out, static_cast<hipStream_t>(stream)) == hipSuccess
             ? MMD8_OK
             : MMD8_E_HIP;
}

int mmd8_quantize_blockwise_h(const mmd8_half* x, size_t n, int block, uint8_t* codes, mmd8_half* absmax, void* stream) {
  if (check_block(block) != MMD8_OK) return MMD8_E_SHAPE;
  if (n == 0) return MMD8_OK;
  if (!x || !codes || !absmax || !aligned(x, 16) || !aligned(codes, 8) || !aligned(absmax, 2)) return MMD8_E_ARG;
  return launch_quantize_blockwise_h(x, n, block, codes, absmax, static_cast<hipStream_t>(stream)) == hipSuccess
             ? MMD8_OK
             : MMD8_E_HIP;
}

int mmd8_dequantize_blockwise_h(const uint8_t* codes, const mmd8_half* absmax, size_t n, int block, mmd8_half* out,
                                void* stream) {
  if (check_block(block) != MMD8_OK) return MMD8_E_SHAPE;
  if (n == 0) return MMD8_OK;
  if (!codes || !absmax || !out || !aligned(out, 16) || !aligned(codes, 8) || !aligned(absmax, 2)) return MMD8_E_ARG;
  return launch_dequantize_blockwise_h(codes, absmax, n, block, out, static_cast<hipStream_t>(stream)) == hipSuccess
             ? MMD8_OK
             : MMD8_E_HIP;
}

uint32_t mmd8_packed_weight_layout(void) { return kPackedLayoutTag; }

size_t mmd8_packed_weight_bytes(int K, int N) {
  if (check_linear_shape(K, N) != MMD8_OK) return 0;
  return (size_t)packed_k(K) * (size_t)packed_n(N);
}

int mmd8_prequantize_weight(const mmd8_half* W, int K, int N, int ldw, int8_t* Wq_packed, float* col_absmax,
                            void* stream) {
  if (int s = check_linear_shape(K, N)) return s;
  if (!W || !Wq_packed || !col_absmax || ldw < N || (ldw % 8) != 0 || !aligned(W, 16) || !aligned(Wq_packed, 256) ||
      !aligned(col_absmax, 4))
    return MMD8_E_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (launch_fill_u32(reinterpret_cast<uint32_t*>(col_absmax), 0u, N, st) != hipSuccess) return MMD8_E_HIP;
  if (launch_col_absmax(W, K, N, ldw, col_absmax, st) != hipSuccess) return MMD8_E_HIP;
  if (launch_weight_quant_pack(W, K, N, ldw, col_absmax, Wq_packed, st) != hipSuccess) return MMD8_E_HIP;
  return MMD8_OK;
}

int mmd8_unpack_weight(const int8_t* Wq_packed, uint32_t Wq_layout, int K, int N, int8_t* Wq_rowmajor, void* stream) {
  if (int s = check_linear_shape(K, N)) return s;
  if (Wq_layout != kPackedLayoutTag) return MMD8_E_VERSION;
  if (!Wq_packed || !Wq_rowmajor) return MMD8_E_ARG;
  return launch_weight_unpack(Wq_packed, K, N, Wq_rowmajor, static_cast<hipStream_t>(stream)) == hipSuccess
             ? MMD8_OK
             : MMD8_E_HIP;
}

size_t mmd8_linear_workspace_bytes(int M, int K, int N) {
  if (M < 0 || check_linear_shape(K, N) != MMD8_OK) return 0;
  return carve(nullptr, M, K, N).bytes;
}
size_t mmd8_linear_lora_workspace_bytes(int M, int K, int N, int r) {
  if (M < 0 || check_linear_shape(K, N) != MMD8_OK || check_lora_rank(r) != MMD8_OK) return 0;
  return carve(nullptr, M, K, N, r).bytes;
}

int mmd8_linear_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace || !aligned(workspace, 256)) return MMD8_E_ARG;
  if (workspace_bytes < kHeadBytes) return MMD8_E_WORKSPACE;
  // kernel attributes of this device, so that no later call has to set one (a call may be under stream capture)
  if (prepare_gemm_kernels() != hipSuccess || prepare_rows_kernels() != hipSuccess) return MMD8_E_HIP;
  return launch_fill_u32(static_cast<uint32_t*>(workspace), 0u, (int)(kHeadBytes / 4),
                         static_cast<hipStream_t>(stream)) == hipSuccess
             ? MMD8_OK
             : MMD8_E_HIP;
}

struct CodedExit {   // a residual added to the output and / or the output leaving in blockwise-coded form
  const mmd8_half* residual;   // [M][ldr] or null
  int ldr;
  int block;                   // 0: the output is not encoded (codes and absmax unused)
  uint8_t* codes;              // [M N]
  float* absmax;               // [ceil(M N / block)]
};

struct Readings {   // alternative readings of the method (mmd8_readings), checked
  bool non_critical_scale;
  const mmd8_half* W_master;   // [K][ldw] or null
  int ldw;
};

struct Adapter {   // low-rank factors of W' = W + B A
  const mmd8_half* A;   // [r][K]
  const mmd8_half* B;   // [N][r]
  int r;
  mmd8_half* T_out;     // [M][r] or null
};

// The layer.  coded: null, or the blockwise-coded form of the activations, in which case X is the
// buffer that receives the decoded activations (ldx == K) before the layer reads them.
// lora: null, or the adapter whose term is added to the output.
// exit: null, or where the coded form of the output goes; Y (contiguous, ldy == N) then receives the tensor that
// is encoded and may be null.
static int run_linear(mmd8_half* X, int M, int K, int ldx, const int8_t* Wq_packed, uint32_t Wq_layout, const float* col_absmax, int N,
                      const mmd8_half* bias, float tau, mmd8_half* Y, int ldy, void* workspace, size_t workspace_bytes,
                      const mmd8_debug_taps* taps, const CodedInput* coded, const Adapter* lora, const CodedExit* exit,
                      void* stream, bool gelu = false, const Readings* readings = nullptr, bool gathered_rows = true) {
  if (M < 0) return MMD8_E_ARG;
  if (int s = check_linear_shape(K, N)) return s;
  if (isnan(tau)) return MMD8_E_ARG;
  if (Wq_layout != kPackedLayoutTag) return MMD8_E_VERSION;
  if (M == 0) return MMD8_OK;
  if (!X || !Wq_packed || !col_absmax || (!Y && !exit) || !workspace) return MMD8_E_ARG;
  if (ldx < K || ldy < N || (ldx % 8) != 0 || (ldy % 8) != 0) return MMD8_E_ARG;
  if (exit && exit->block > 0 &&
      (!exit->codes || !exit->absmax || !aligned(exit->codes, 16) || !aligned(exit->absmax, 4) || ldy != N))
    return MMD8_E_ARG;
  if (exit && ((exit->block == 0 && (!exit->residual || !Y)) ||
               (exit->residual && (exit->ldr < N || (exit->ldr % 8) != 0 || !aligned(exit->residual, 16)))))
    return MMD8_E_ARG;
  if (!aligned(X, 16) || !aligned(Y, 16) || !aligned(Wq_packed, 256) || !aligned(workspace, 256) ||
      !aligned(col_absmax, 4) || (bias && !aligned(bias, 2)))
    return MMD8_E_ARG;
  if (Y && ranges_overlap(X, span_bytes(M, K, ldx), Y, span_bytes(M, N, ldy))) return MMD8_E_ARG;
  if (lora && (!lora->A || !lora->B || !aligned(lora->A, 16) || !aligned(lora->B, 16) ||
               (lora->T_out && !aligned(lora->T_out, 16))))
    return MMD8_E_ARG;
  const Workspace ws = carve(workspace, M, K, N, lora ? lora->r : 0, exit ? exit->block : 0, gathered_rows);
  if (workspace_bytes < ws.bytes) return MMD8_E_WORKSPACE;
  // a coded output is written by the layer's last kernel where that is possible, otherwise by the encoder after it
  const bool encodes = exit && exit->block > 0;
  const bool exit_fused = encodes && exit_fuses(M, K, N, exit->block);
  if (encodes && !exit_fused && !Y) Y = ws.h;

  hipStream_t st = static_cast<hipStream_t>(stream);
  const int Kpad = packed_k(K);
  const mmd8_debug_taps none = {};
  const mmd8_debug_taps& t = taps ? *taps : none;

  auto record = [&](void* ev) {
    return !ev || hipEventRecord(static_cast<hipEvent_t>(ev), st) == hipSuccess;
  };
  if (!record(t.event_begin)) return MMD8_E_HIP;
  const PackOutliers po = {ws.idx, ws.n_out, ws.mask, t.outlier_mask, t.outlier_idx, t.n_outliers,
                           Wq_packed, col_absmax, N, ws.xo, ws.wo, ws.f_slabs, ws.crit_slabs,
                           readings ? readings->W_master : nullptr, readings ? readings->ldw : 0, ws.xg, ws.wg, ws.g_slabs, ws.dense_from};
  // Up to 128 rows go through the decode kernels, 64 rows at a time (the weights are streamed twice for more
  // than 64): for activations with few critical columns that costs what the tiled GEMM costs at this size, and
  // with heavy-tailed activations (hundreds of critical columns) it is ten times faster.
  // (the decode kernels multiply the critical columns with the weight codes themselves: original 16-bit rows go
  // through the tiled GEMM whatever the number of rows)
  const bool skinny = M <= kSkinnyChunkedMaxM && !(readings && readings->W_master);
  // A few rows (at most kPanelPrepMaxM): the decode GEMM kernel prepares its own operands (scales, codes, critical
  // columns) from X, and the scan and pack kernels are left out.  Not when their outputs are asked for through the taps.
  const bool wants_prep_taps = t.outlier_mask || t.row_absmax || t.xq || t.n_outliers || t.outlier_idx;
  // One or two rows (while their operands fit in LDS): the whole layer is one kernel (k_gemm_rows).  When the taps of the
  // preparation are asked for, the scan and pack kernels run ahead of it for their sake only.
  // (alternative readings: always the separate scan and pack kernels, which is where they differ)
  const bool may_own_prep = !(t.tuning & MMD8_TUNE_SEPARATE_PREP) && !readings;
  const bool rows_path = may_own_prep && !(t.tuning & MMD8_TUNE_NO_ROWS_KERNEL) && rows_kernel_fits(M, Kpad);
  const bool own_prep = skinny && !rows_path && !wants_prep_taps && may_own_prep && panel_prep_fits(M, plan_skinny(M, K, N));
  // coded activations are decoded by the one-pass preparation kernel itself where that kernel runs
  // (element offsets are held in 32 bits there); otherwise by the decoder, ahead of the usual kernels
  const bool one_pass = !skinny && prep_fits(K) && !readings;
  // Decode kernels after the scan and pack kernels, nobody asking for the list of critical columns: the pack kernel
  // leaves the list out (its longest part at these sizes) and the decode kernel reads the column flags themselves as
  // its mask.  Every workgroup reads them, so they are put back to zero by the kernel after it, the one that sums
  // the splits: only calls that have one.
  bool lean_pack = false;
  if (skinny && !rows_path && !own_prep && !wants_prep_taps) {
    const SkinnyPlan plan = plan_skinny(M < kSkinnyMaxM ? M : kSkinnyMaxM, K, N);
    lean_pack = plan.splits > 1 || lora || gelu || (exit && (exit->residual || exit_fused));
  }
  const bool fused_decode = coded && one_pass && prep_from_codes_fits(K) && (size_t)M * K < ((size_t)1 << 31);
  if (coded && !fused_decode &&
      launch_dequantize_blockwise(coded->codes, coded->absmax, (size_t)M * K, coded->block, X, st) != hipSuccess)
    return MMD8_E_HIP;
  if (one_pass) {
    // one pass over X: scales, flags and codes together, then the critical columns are cleared
    if (launch_prep(X, M, K, ldx, threshold_pattern(tau), Kpad, ws.flag, ws.r, ws.xq, t.xq, po, fused_decode ? coded : nullptr,
                    t.event_prep_mid, st) != hipSuccess)
      return MMD8_E_HIP;
  } else if (!own_prep && (!rows_path || wants_prep_taps)) {
    if (launch_scan(X, M, K, ldx, threshold_pattern(tau), Kpad, ws.flag, ws.r, st) != hipSuccess) return MMD8_E_HIP;
    if (!record(t.event_prep_mid)) return MMD8_E_HIP;
    // the row scale over the non-critical columns only: needs the flags of every row, hence a pass of its own
    if (readings && readings->non_critical_scale &&
        launch_row_absmax_noncritical(X, M, K, ldx, ws.flag, ws.r, st) != hipSuccess)
      return MMD8_E_HIP;
    // (the decode kernels' operands are packed 64 rows at a time, below)
    if (!skinny && launch_pack(X, M, K, ldx, ws.flag, ws.r, ws.xq, Kpad, t.xq, nullptr, po, st) != hipSuccess)
      return MMD8_E_HIP;
  }
  if (t.row_absmax &&
      hipMemcpyAsync(t.row_absmax, ws.r, (size_t)M * 4, hipMemcpyDeviceToDevice, st) != hipSuccess)
    return MMD8_E_HIP;

  if (lora) {
    // T = f16(X A^T); for the tiled GEMM T and B also go into the fp16 slabs behind the critical columns
    LoraArgs l = {};
    l.X = X;
    l.M = M;
    l.K = K;
    l.ldx = ldx;
    l.A = lora->A;
    l.B = lora->B;
    l.r = lora->r;
    l.N = N;
    l.T = ws.lora_t;
    l.T_user = lora->T_out;
    l.Xo = skinny ? nullptr : ws.xo;
    l.Wo = skinny ? nullptr : ws.wo;
    l.f_slabs = ws.f_slabs;
    l.crit_slabs = ws.crit_slabs;
    if (launch_lora_down(l, plan_lora(M, K), ws.lora_part, st) != hipSuccess) return MMD8_E_HIP;
  }

  if (rows_path) {   // (a coded output: the encoder follows)
    if (wants_prep_taps &&
        launch_pack(X, M, K, ldx, ws.flag, ws.r, ws.xq, Kpad, t.xq, ws.xf, po, st) != hipSuccess)
      return MMD8_E_HIP;
    if (!record(t.event_gemm_begin)) return MMD8_E_HIP;
    SkinnyArgs g = {};
    g.flag_reset = wants_prep_taps ? ws.flag : nullptr;               // the scan set them
    g.Wt = Wq_packed;
    g.M = M;
    g.N = N;
    g.Kpad = Kpad;
    g.c = col_absmax;
    g.bias = bias;
    g.Y = Y;
    g.ldy = ldy;
    g.tap_acc = t.acc;
    g.gelu = gelu ? 1 : 0;
    if (exit) {
      g.residual = exit->residual;
      g.ldr = exit->ldr;
    }
    if (lora) {
      g.lora_T = ws.lora_t;
      g.lora_ldt = kLoraMaxRank;
      g.lora_B = lora->B;
      g.lora_r = lora->r;
    }
    g.X = X;
    g.ldx = ldx;
    g.K = K;
    g.th = threshold_pattern(tau);
    if (launch_gemm_rows(g, st) != hipSuccess) return MMD8_E_HIP;
  } else if (skinny) {
    const SkinnyPlan plan = plan_skinny(M < kSkinnyMaxM ? M : kSkinnyMaxM, K, N);
    for (int row0 = 0; row0 < M; row0 += kSkinnyMaxM) {
      const int Mc = M - row0 < kSkinnyMaxM ? M - row0 : kSkinnyMaxM;
      // codes and the fp16 copy of these rows, masked with the flags of all M rows; the list of critical columns is
      // published again with every pass (the same list)
      if (!own_prep && launch_pack(X + (size_t)row0 * ldx, Mc, K, ldx, ws.flag, ws.r + row0, ws.xq, Kpad,
                                   t.xq ? t.xq + (size_t)row0 * K : nullptr, ws.xf, po, st, !lean_pack) != hipSuccess)
        return MMD8_E_HIP;
      if (row0 == 0 && !record(t.event_gemm_begin)) return MMD8_E_HIP;
      SkinnyArgs g = {};
      g.Xq = ws.xq;
      g.Wt = Wq_packed;
      g.Xf = ws.xf;
      g.mask = ws.mask;
      g.M = Mc;
      g.N = N;
      g.Kpad = Kpad;
      g.r = ws.r + row0;
      g.c = col_absmax;
      g.bias = bias;
      g.Y = Y ? Y + (size_t)row0 * ldy : nullptr;
      g.ldy = ldy;
      if (exit) {
        g.residual = exit->residual ? exit->residual + (size_t)row0 * exit->ldr : nullptr;
        g.ldr = exit->ldr;
        if (exit_fused) {
          g.codes = exit->codes + (size_t)row0 * N;
          g.code_absmax = exit->absmax + (size_t)row0 * N / exit->block;
          g.code_block = exit->block;
        }
      }
      g.gelu = gelu ? 1 : 0;
      g.partial = ws.partial;
      g.tap_acc = t.acc ? t.acc + (size_t)row0 * N : nullptr;
      g.flag_reset = (!own_prep && row0 + kSkinnyMaxM >= M) ? ws.flag : nullptr;   // the last pass zeroes the column flags again
      if (lean_pack) {
        g.mask = ws.flag;
        g.flag_reset_late = g.flag_reset;
        g.flag_reset = nullptr;
      }
      if (own_prep) {
        g.X = X;
        g.ldx = ldx;
        g.K = K;
        g.th = threshold_pattern(tau);
      }
      if (lora) {
        g.lora_T = ws.lora_t + (size_t)row0 * kLoraMaxRank;
        g.lora_ldt = kLoraMaxRank;
        g.lora_B = lora->B;
        g.lora_r = lora->r;
      }
      if (launch_gemm_skinny(g, plan, st) != hipSuccess) return MMD8_E_HIP;
    }
  } else {
    if (!record(t.event_gemm_begin)) return MMD8_E_HIP;
    GemmArgs g = {};
    g.Xq = ws.xq;
    g.Wt = Wq_packed;
    g.M = M;
    g.N = N;
    g.Kpad = Kpad;
    g.r = ws.r;
    g.c = col_absmax;
    g.bias = bias;
    g.X = X;
    g.ldx = ldx;
    g.idx = ws.idx;
    g.n_out = ws.n_out;
    g.mask = ws.mask;
    g.Xo = ws.xo;
    g.Wo = ws.wo;
    g.f_slabs = ws.f_slabs;
    g.crit_slabs = ws.crit_slabs;
    g.Y = Y;
    g.ldy = ldy;
    g.tap_acc = t.acc;
    g.tap_ld = N;
    g.tiles_m = g.tiles_n = 0;
    g.flag_reset = ws.flag;
    g.gelu = gelu ? 1 : 0;
    g.Xg = ws.xg;
    g.Wg = ws.wg;
    g.g_slabs = ws.g_slabs;
    g.dense_from = ws.dense_from;
    if (readings) {
      g.W_master = readings->W_master;
      g.ldw_master = readings->ldw;
    }
    if (exit) {
      g.residual = exit->residual;
      g.ldr = exit->ldr;
      if (exit_fused) {
        g.codes = exit->codes;
        g.code_absmax = exit->absmax;
        g.code_ld = N;
        g.code_log_block = exit->block == 64 ? 6 : exit->block == 128 ? 7 : 8;
      }
    }
    if (launch_gemm_mixed(g, (int)(t.tuning & 0xfu) - 1, st) != hipSuccess) return MMD8_E_HIP;
  }
  if (encodes && !exit_fused &&
      launch_quantize_blockwise(Y, (size_t)M * N, exit->block, exit->codes, exit->absmax, st) != hipSuccess)
    return MMD8_E_HIP;
  if (!record(t.event_gemm_end)) return MMD8_E_HIP;
  return MMD8_OK;
}

int mmd8_mixed_int8_linear(const mmd8_half* X, int M, int K, int ldx, const int8_t* Wq_packed,
                           uint32_t Wq_layout, const float* col_absmax, int N, const mmd8_half* bias, float tau, mmd8_half* Y, int ldy,
                           void* workspace, size_t workspace_bytes, const mmd8_debug_taps* taps, void* stream) {
  // X is only read on this path
  return run_linear(const_cast<mmd8_half*>(X), M, K, ldx, Wq_packed, Wq_layout, col_absmax, N, bias, tau, Y, ldy, workspace,
                    workspace_bytes, taps, nullptr, nullptr, nullptr, stream);
}

// ---- The layer for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops):
// the workspace is a file-scope device array instead of an argument.  Host code never uses the array's name as an
// address: the device address is asked for once per device (hipGetSymbolAddress, with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[MMD8_STATIC_WORKSPACE_BYTES];
namespace {
struct StaticWorkspace {
  void* ptr;       // device address of `scratch` on this device; null until the first call on it
  bool head_zero;  // the head (counters, column flags) holds zeros: true between calls that succeeded
};
StaticWorkspace g_static_ws[64];
std::mutex g_static_mu;
}  // namespace

int mmd8_mixed_int8_linear_static(const mmd8_half* X, int M, int K, int ldx, const int8_t* Wq_packed, uint32_t Wq_layout,
                                  const float* col_absmax, int N, const mmd8_half* bias, float tau, mmd8_half* Y, int ldy,
                                  const mmd8_debug_taps* taps, void* stream) {
  if (M < 0) return MMD8_E_ARG;
  if (int s = check_linear_shape(K, N)) return s;
  // (the array is small: the further slabs of critical columns only where they fit, else the GEMM gathers those
  // columns tile by tile)
  const bool further_slabs = carve(nullptr, M, K, N, 0, 0, true).bytes <= (size_t)MMD8_STATIC_WORKSPACE_BYTES;
  if (!further_slabs && carve(nullptr, M, K, N, 0, 0, false).bytes > (size_t)MMD8_STATIC_WORKSPACE_BYTES)
    return MMD8_E_WORKSPACE;   // too large for the array
  if (Wq_layout != kPackedLayoutTag) return MMD8_E_VERSION;
  if (M == 0) return isnan(tau) ? MMD8_E_ARG : MMD8_OK;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MMD8_E_HIP;
  void* ws = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_static_mu);
    StaticWorkspace& w = g_static_ws[dev];
    if (!w.ptr) {   // first call on this device: every GPU holds its own copy of the array at its own address
      void* p = nullptr;
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MMD8_E_HIP;
      if (prepare_gemm_kernels() != hipSuccess || prepare_rows_kernels() != hipSuccess) return MMD8_E_HIP;
      w.ptr = p;
      w.head_zero = false;
    }
    if (!w.head_zero) {
      // a fill kernel, not a memset: the call may be recorded into a graph
      if (launch_fill_u32(static_cast<uint32_t*>(w.ptr), 0u, (int)(kHeadBytes / 4), static_cast<hipStream_t>(stream)) != hipSuccess)
        return MMD8_E_HIP;
      w.head_zero = true;
    }
    ws = w.ptr;
  }
  const int s = run_linear(const_cast<mmd8_half*>(X), M, K, ldx, Wq_packed, Wq_layout, col_absmax, N, bias, tau, Y, ldy, ws,
                           MMD8_STATIC_WORKSPACE_BYTES, taps, nullptr, nullptr, nullptr, stream, false, nullptr, further_slabs);
  if (s == MMD8_E_HIP) {   // some kernels of the call may have run: the head is cleared again before the next call
    std::lock_guard<std::mutex> lock(g_static_mu);
    g_static_ws[dev].head_zero = false;
  }
  return s;
}

int mmd8_mixed_int8_linear_readings(const mmd8_half* X, int M, int K, int ldx, const int8_t* Wq_packed, uint32_t Wq_layout,
                                    const float* col_absmax, int N, const mmd8_half* bias, float tau,
                                    const mmd8_readings* readings, mmd8_half* Y, int ldy, void* workspace,
                                    size_t workspace_bytes, const mmd8_debug_taps* taps, void* stream) {
  if (!readings) return MMD8_E_ARG;
  if (readings->row_scale != MMD8_ROW_SCALE_SUB_THRESHOLD && readings->row_scale != MMD8_ROW_SCALE_NON_CRITICAL)
    return MMD8_E_ARG;
  if (readings->W_master && (readings->ldw < N || (readings->ldw % 8) != 0 || !aligned(readings->W_master, 16)))
    return MMD8_E_ARG;
  const Readings rd = {readings->row_scale == MMD8_ROW_SCALE_NON_CRITICAL, readings->W_master, readings->ldw};
  return run_linear(const_cast<mmd8_half*>(X), M, K, ldx, Wq_packed, Wq_layout, col_absmax, N, bias, tau, Y, ldy, workspace,
                    workspace_bytes, taps, nullptr, nullptr, nullptr, stream, false, &rd);
}

int mmd8_mixed_int8_linear_gelu(const mmd8_half* X, int M, int K, int ldx, const int8_t* Wq_packed,
                                uint32_t Wq_layout, const float* col_absmax, int N, const mmd8_half* bias, float tau, mmd8_half* Y, int ldy,
                                void* workspace, size_t workspace_bytes, const mmd8_debug_taps* taps, void* stream) {
  return run_linear(const_cast<mmd8_half*>(X), M, K, ldx, Wq_packed, Wq_layout, col_absmax, N, bias, tau, Y, ldy, workspace,
                    workspace_bytes, taps, nullptr, nullptr, nullptr, stream, true);
}

int mmd8_mixed_int8_linear_residual(const mmd8_half* X, int M, int K, int ldx, const int8_t* Wq_packed,
                                    uint32_t Wq_layout, const float* col_absmax, int N, const mmd8_half* bias, float tau,
                                    const mmd8_half* residual, int ldr, mmd8_half* Y, int ldy, void* workspace,
                                    size_t workspace_bytes, const mmd8_debug_taps* taps, void* stream) {
  const CodedExit exit = {residual, ldr, 0, nullptr, nullptr};
  return run_linear(const_cast<mmd8_half*>(X), M, K, ldx, Wq_packed, Wq_layout, col_absmax, N, bias, tau, Y, ldy, workspace,
                    workspace_bytes, taps, nullptr, nullptr, &exit, stream);
}

size_t mmd8_linear_to_codes_workspace_bytes(int M, int K, int N, int block) {
  if (M < 0 || check_linear_shape(K, N) != MMD8_OK || check_block(block) != MMD8_OK) return 0;
  return carve(nullptr, M, K, N, 0, block).bytes;
}

int mmd8_mixed_int8_linear_to_codes(const mmd8_half* X, int M, int K, int ldx, const int8_t* Wq_packed,
                                    uint32_t Wq_layout, const float* col_absmax, int N, const mmd8_half* bias, float tau,
                                    const mmd8_half* residual, int ldr, int block, uint8_t* codes, float* absmax,
                                    mmd8_half* H, void* workspace, size_t workspace_bytes,
                                    const mmd8_debug_taps* taps, void* stream) {
  if (check_block(block) != MMD8_OK) return MMD8_E_SHAPE;
  const CodedExit exit = {residual, ldr, block, codes, absmax};
  return run_linear(const_cast<mmd8_half*>(X), M, K, ldx, Wq_packed, Wq_layout, col_absmax, N, bias, tau, H, N, workspace,
                    workspace_bytes, taps, nullptr, nullptr, &exit, stream);
}

int mmd8_mixed_int8_linear_lora(const mmd8_half* X, int M, int K, int ldx, const int8_t* Wq_packed,
                                uint32_t Wq_layout, const float* col_absmax, int N, const mmd8_half* bias, float tau,
                                const mmd8_half* lora_A, const mmd8_half* lora_B, int r, mmd8_half* lora_T,
                                mmd8_half* Y, int ldy, void* workspace, size_t workspace_bytes,
                                const mmd8_debug_taps* taps, void* stream) {
  if (check_lora_rank(r) != MMD8_OK) return MMD8_E_SHAPE;
  const Adapter lora = {lora_A, lora_B, r, lora_T};
  return run_linear(const_cast<mmd8_half*>(X), M, K, ldx, Wq_packed, Wq_layout, col_absmax, N, bias, tau, Y, ldy, workspace,
                    workspace_bytes, taps, nullptr, &lora, nullptr, stream);
}

int mmd8_mixed_int8_linear_from_codes(const uint8_t* codes, const float* absmax, int block, int M, int K,
                                      mmd8_half* X_decoded, const int8_t* Wq_packed, uint32_t Wq_layout, const float* col_absmax, int N,
                                      const mmd8_half* bias, float tau, mmd8_half* Y, int ldy, void* workspace,
                                      size_t workspace_bytes, const mmd8_debug_taps* taps, void* stream) {
  if (check_block(block) != MMD8_OK) return MMD8_E_SHAPE;
  if (M > 0 && (!codes || !absmax || !aligned(codes, 16) || !aligned(absmax, 4))) return MMD8_E_ARG;
  const CodedInput coded = {codes, absmax, block};
  return run_linear(X_decoded, M, K, K, Wq_packed, Wq_layout, col_absmax, N, bias, tau, Y, ldy, workspace, workspace_bytes, taps,
                    &coded, nullptr, nullptr, stream);
}

uint32_t mmd8_threshold_fp16_pattern(float tau) { return threshold_pattern(tau); }

}  // extern "C"
