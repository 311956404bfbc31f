/* mmd8 -- mixed-matrix-decomposition int8 linear layer and dynamic blockwise 8-bit codec
 * for AMD Instinct MI355X (gfx950).  C ABI.
 *
 * The two operations are the compression techniques of the paper's section "Compression
 * techniques": item 1 (dynamic blockwise quantization of the hidden states sent from one shard
 * to the next) and item 2 (mixed matrix decomposition: 8-bit weights and activations with a
 * small 16-bit part for the critical feature dimensions).
 *
 * Conventions for every entry point
 *   - Pointers marked DEVICE are device memory owned by the caller; the library never
 *     allocates, frees or copies to the host.  HOST pointers returned by the library point at
 *     static read-only data.
 *   - fp16 data are IEEE binary16 bit patterns (mmd8_half).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream) and
 *     the call returns without synchronising.  Calls on one stream are ordered.
 *   - Return value: MMD8_OK, or a negative status.  MMD8_E_ARG, MMD8_E_SHAPE, MMD8_E_WORKSPACE and
 *     MMD8_E_VERSION are found before anything is launched: nothing has been enqueued.  MMD8_E_HIP
 *     (a launch failed) can come after some of a call's kernels were enqueued: outputs are then
 *     unspecified and a workspace of the layer must be set up again before it is reused.
 *   - Zero-sized problems (M == 0, n == 0) are valid and enqueue nothing.
 *   - Inputs are assumed finite; NaN/Inf give unspecified values but never a fault.
 */
#ifndef MMD8_H
#define MMD8_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t mmd8_half;

enum {
  MMD8_OK          = 0,
  MMD8_E_ARG       = -1,  /* null pointer, negative size, leading dimension too small, misaligned, NaN tau */
  MMD8_E_SHAPE     = -2,  /* unsupported shape: K % 16, N % 8, K above MMD8_MAX_K, bad block size          */
  MMD8_E_WORKSPACE = -3,  /* workspace smaller than mmd8_linear_workspace_bytes()                           */
  MMD8_E_HIP       = -4,  /* a HIP call or kernel launch failed                                             */
  MMD8_E_VERSION   = -5   /* packed weights written under another layout than mmd8_packed_weight_layout()   */
};

/* Largest supported K.  K * 127^2 must stay below 2^31 so that the int32 accumulators of the
 * integer product cannot overflow (that alone allows 133144); column indices are also held in
 * 16 bits inside the kernels. */
#define MMD8_MAX_K 65536

/* Human-readable text for a status code (HOST, static). */
const char* mmd8_status_string(int status);

/* ------------------------------------------------------------------------------------------
 * Dynamic blockwise 8-bit codec ("Compression techniques", item 1).
 *
 * The tensor is treated as a flat contiguous array of n fp16 values cut into blocks of `block`
 * consecutive elements (the last block may be short).  Per block b:
 *     absmax[b] = max |x_i|                                  (fp32, exact)
 *     v_i       = f32(x_i) * (1.0f / absmax[b])              (0 if absmax[b] == 0)
 *     codes[i]  = number of midpoints Mid[j] (j = 0..254) with v_i > Mid[j]
 * and decoding is  out[i] = f16( T[codes[i]] * absmax[b] )  (fp32 product, round to nearest even).
 * T is the 256-entry signed dynamic code: magnitudes 10^-e (0.1 + 0.9 (j + 1/2) / 2^(6-e)),
 * e = 0..6, j = 0..2^(6-e)-1, both signs, plus 0 and +1.0; Mid[j] = f32((T[j] + T[j+1]) / 2).
 * `block` must be a multiple of 64 with 64 <= block <= 4096, else MMD8_E_SHAPE.
 * x, out: 16-byte aligned; codes: 8-byte aligned (both directions); absmax: 4-byte aligned; else MMD8_E_ARG.
 * ------------------------------------------------------------------------------------------ */
int mmd8_quantize_blockwise(const mmd8_half* x /*DEVICE [n]*/, size_t n, int block,
                            uint8_t* codes /*DEVICE [n]*/, float* absmax /*DEVICE [ceil(n/block)]*/,
                            void* stream);
int mmd8_dequantize_blockwise(const uint8_t* codes /*DEVICE [n]*/, const float* absmax /*DEVICE*/,
                              size_t n, int block, mmd8_half* out /*DEVICE [n]*/, void* stream);
/* The other reading of how a block's scale is stored ("Compression techniques", item 1 names the technique, not
 * the width of the scale): every absmax is the magnitude of an fp16 element, so 2 bytes hold it exactly.  Same
 * codes, same decoded values, absmax as fp16 bit patterns: (1 + 2 / block) / 2 of the fp16 tensor's bytes instead of
 * (1 + 4 / block) / 2.  absmax: DEVICE [ceil(n/block)] fp16, 2-byte aligned; everything else as above. */
int mmd8_quantize_blockwise_h(const mmd8_half* x /*DEVICE [n]*/, size_t n, int block,
                              uint8_t* codes /*DEVICE [n]*/, mmd8_half* absmax /*DEVICE [ceil(n/block)]*/,
                              void* stream);
int mmd8_dequantize_blockwise_h(const uint8_t* codes /*DEVICE [n]*/, const mmd8_half* absmax /*DEVICE*/,
                                size_t n, int block, mmd8_half* out /*DEVICE [n]*/, void* stream);
/* HOST pointers to the 256 code values (ascending) and the 255 midpoints. */
const float* mmd8_code_table(void);
const float* mmd8_code_midpoints(void);

/* ------------------------------------------------------------------------------------------
 * Mixed int8 linear layer ("Compression techniques", item 2).   Y[M,N] = X[M,K] W[K,N]
 *
 * Weight pre-quantization (once per weight matrix):
 *     col_absmax[n] = max_k |W[k,n]|
 *     Wq[k,n]       = clamp(rint(f32(W[k,n]) * (127.0f / col_absmax[n])), -127, 127)   (0 if absmax 0)
 * W is read as W[k*ldw + n] (ldw >= N).  Wq is written in an opaque layout of
 * mmd8_packed_weight_bytes(K, N) bytes; mmd8_unpack_weight recovers the plain row-major
 * int8 [K,N] matrix (for checking).  mmd8_packed_weight_layout() identifies the layout this build of the
 * library writes and reads.  Whoever stores a blob stores that value with it and hands it back as
 * `Wq_layout` to every call that reads the blob: a call given another value returns MMD8_E_VERSION
 * and launches nothing (the weights must be packed again from W).
 * Requirements: K % 16 == 0, 16 <= K <= MMD8_MAX_K, N % 8 == 0, N >= 8 (else MMD8_E_SHAPE);
 * W 16-byte aligned and ldw % 8 == 0, Wq_packed 256-byte aligned (else MMD8_E_ARG).
 * ------------------------------------------------------------------------------------------ */
uint32_t mmd8_packed_weight_layout(void);
size_t   mmd8_packed_weight_bytes(int K, int N);
int mmd8_prequantize_weight(const mmd8_half* W /*DEVICE*/, int K, int N, int ldw,
                            int8_t* Wq_packed /*DEVICE*/, float* col_absmax /*DEVICE [N]*/, void* stream);
int mmd8_unpack_weight(const int8_t* Wq_packed /*DEVICE*/, uint32_t Wq_layout, int K, int N,
                       int8_t* Wq_rowmajor /*DEVICE [K,N]*/, void* stream);

/* Optional taps that expose the intermediates of one mmd8_mixed_int8_linear call (for parity
 * checks).  Any member may be NULL.  All are DEVICE pointers.  The output of a call does not depend on
 * which taps are asked for.  (For up to 8 rows the kernels that multiply also prepare their own operands;
 * asking for outlier_mask, row_absmax, xq, n_outliers or outlier_idx makes the separate preparation kernels
 * run as well, which produce the same quantities.) */
typedef struct {
  uint8_t* outlier_mask;  /* [K]    1 = critical feature dimension                         */
  float*   row_absmax;    /* [M]    r[m]                                                   */
  int8_t*  xq;            /* [M,K]  row-major activation codes                             */
  int32_t* acc;           /* [M,N]  row-major int32 accumulators of the integer product    */
  int32_t* n_outliers;    /* [1]                                                           */
  int32_t* outlier_idx;   /* [K]    ascending indices of the critical dimensions; entries
                                    past n_outliers are unspecified                         */
  /* Optional hipEvent_t handles (HOST, created by the caller) recorded on `stream`: when the
     call starts, after the first kernel of the activation preparation (the one pass over X, or
     the scan), just before the GEMM kernel and just after it.  For per-stage timing.           */
  void* event_begin;
  void* event_prep_mid;
  void* event_gemm_begin;
  void* event_gemm_end;
  /* Kernel choice of this one call, for tests and tuning: 0 = the library's own choice, else an OR of the
     MMD8_TUNE_* values below.  Every choice computes the same integers (mask, scales, codes, accumulators);
     Y may differ in the last fp16 bit between choices that add the 16-bit part in another order.  A value
     that does not fit the shape is ignored.  Per call, no global state: other threads are unaffected.       */
  uint32_t tuning;
} mmd8_debug_taps;
#define MMD8_TUNE_GEMM_TILES(v)    ((uint32_t)((v) + 1) & 0xfu) /* tiled GEMM (more than 128 rows): tile configuration v = 0..5 */
#define MMD8_TUNE_SEPARATE_PREP    0x10u  /* up to 8 rows: run the scan and pack kernels instead of letting the multiplying kernel prepare its own operands */
#define MMD8_TUNE_NO_ROWS_KERNEL   0x20u  /* one or two rows: use the split-K kernels instead of the single-kernel form */

/* The layer, per call (tau: threshold; X read as X[m*ldx + k]; Y written as Y[m*ldy + n]):
 *     flag[k]  = any_m |X[m,k]| >= tau
 *     r[m]     = max over k of |X[m,k]| restricted to |X[m,k]| < tau        (0 if none)
 *     Xq[m,k]  = flag[k] ? 0 : clamp(rint(f32(X[m,k]) * (127.0f / r[m])), -127, 127)
 *     acc[m,n] = sum_k Xq[m,k] * Wq[k,n]                                     (int32, exact)
 *     Y[m,n]   = f16( acc[m,n] r[m] c[n] / 127^2
 *                     + sum_{k: flag[k]} X[m,k] * f16(Wq[k,n] * (c[n] / 127.0f))   (fp32 accumulation)
 *                     + bias[n] )
 * tau may be 0 (every dimension critical: a pure fp16 product) or +INFINITY (pure int8).
 * Requirements: shapes as for mmd8_prequantize_weight; X, Y 16-byte aligned, ldx % 8 == 0,
 * ldx >= K, ldy % 8 == 0, ldy >= N; Y must not alias X; workspace 256-byte aligned and at
 * least mmd8_linear_workspace_bytes(M, K, N) bytes.
 *
 * Workspace protocol: a workspace is set up once with mmd8_linear_workspace_init (it zeroes a
 * small head of counters and column flags; everything else may hold anything).  Every call
 * leaves the head zeroed again, so the same workspace serves any number of calls of any shape
 * that fits, one after the other on one stream.  Two calls must not use one workspace at the
 * same time.  After a call that returned MMD8_E_HIP, set the workspace up again.
 * mmd8_linear_workspace_init also sets the kernels' attributes on the current device; the calls of the layer made
 * after it allocate nothing, synchronise nothing and change no device state, so they can be captured in a HIP
 * graph (set the workspace up before the capture starts). */
size_t mmd8_linear_workspace_bytes(int M, int K, int N);
int mmd8_linear_workspace_init(void* workspace /*DEVICE*/, size_t workspace_bytes, void* stream);
int mmd8_mixed_int8_linear(const mmd8_half* X /*DEVICE*/, int M, int K, int ldx,
                           const int8_t* Wq_packed /*DEVICE*/, uint32_t Wq_layout, const float* col_absmax /*DEVICE [N]*/, int N,
                           const mmd8_half* bias /*DEVICE [N] or NULL*/, float tau,
                           mmd8_half* Y /*DEVICE*/, int ldy,
                           void* workspace /*DEVICE*/, size_t workspace_bytes,
                           const mmd8_debug_taps* taps /*HOST struct or NULL*/, void* stream);

/* mmd8_mixed_int8_linear for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, results (bit for bit) and errors, without the
 * workspace: the library's own device array of MMD8_STATIC_WORKSPACE_BYTES serves as one (every GPU the library
 * runs on holds it until the process ends; that is enough for up to 64 rows of every Llama-7B- and
 * 70B-shaped linear).  The array takes the layout of a workspace of mmd8_linear_workspace_bytes(M, K, N) bytes,
 * or, where that does not fit, the same less the slabs in which calls of more than 128 rows gather the critical
 * columns beyond the first 256 (those are then gathered tile by tile, and an output may differ from the other
 * entry point's in its last bit for inputs that have so many); a problem that does not fit either way returns
 * MMD8_E_WORKSPACE and launches nothing.  The call allocates and frees nothing and synchronises nothing; the
 * first call on a device looks up the array's address and sets kernel attributes (make it before a capture
 * starts).  All calls on one GPU share the one array: calls that overlap in time (two streams, two threads)
 * race; order them. */
#define MMD8_STATIC_WORKSPACE_BYTES (32u << 20)
int mmd8_mixed_int8_linear_static(const mmd8_half* X /*DEVICE*/, int M, int K, int ldx,
                                  const int8_t* Wq_packed /*DEVICE*/, uint32_t Wq_layout, const float* col_absmax /*DEVICE [N]*/, int N,
                                  const mmd8_half* bias /*DEVICE [N] or NULL*/, float tau,
                                  mmd8_half* Y /*DEVICE*/, int ldy,
                                  const mmd8_debug_taps* taps /*HOST struct or NULL*/, void* stream);

/* The layer under the other readings of "Compression techniques", item 2 ("a small fraction of critical weights at
 * 16-bit precision"; the paper gives no formula for the scale of the 8-bit part nor for where the 16-bit weights
 * come from).  Two switches, independent of each other:
 *   row_scale   MMD8_ROW_SCALE_SUB_THRESHOLD: r[m] = max{|X[m,k]| : |X[m,k]| < tau}, as in mmd8_mixed_int8_linear;
 *               MMD8_ROW_SCALE_NON_CRITICAL:  r[m] = max{|X[m,k]| : flag[k] == 0}, the largest magnitude among the
 *               columns that stay in the 8-bit part (needs the flags of every row first: one more pass over X).
 *   W_master    NULL: the 16-bit weights of the critical dimensions are re-created from the codes,
 *               f16(Wq[k,n] * (c[n] / 127.0f)), as in mmd8_mixed_int8_linear (1 byte per weight resident);
 *               else DEVICE [K][ldw] fp16, the original weight matrix W (the one mmd8_prequantize_weight read):
 *               its rows W[k,:] multiply the critical columns as they are (3 bytes per weight resident; tau = 0
 *               then gives the fp16 product X W itself).  16-byte aligned, ldw >= N, ldw % 8 == 0.
 * Everything else (flags, codes given the scale, the integer product, the dequantization, one rounding) is as in
 * mmd8_mixed_int8_linear, and so are the other arguments, the workspace and the errors (MMD8_E_ARG for a NULL
 * `readings`, an unknown row_scale or a bad W_master / ldw).  These readings always run the separate scan and pack
 * kernels, and with W_master the tiled GEMM for any number of rows. */
enum { MMD8_ROW_SCALE_SUB_THRESHOLD = 0, MMD8_ROW_SCALE_NON_CRITICAL = 1 };
typedef struct {
  int row_scale;              /* MMD8_ROW_SCALE_*                                   */
  const mmd8_half* W_master;  /* DEVICE [K][ldw] fp16 or NULL                       */
  int ldw;
} mmd8_readings;
int mmd8_mixed_int8_linear_readings(const mmd8_half* X /*DEVICE*/, int M, int K, int ldx,
                                    const int8_t* Wq_packed /*DEVICE*/, uint32_t Wq_layout, const float* col_absmax /*DEVICE [N]*/, int N,
                                    const mmd8_half* bias /*DEVICE [N] or NULL*/, float tau,
                                    const mmd8_readings* readings /*HOST struct*/,
                                    mmd8_half* Y /*DEVICE*/, int ldy,
                                    void* workspace /*DEVICE*/, size_t workspace_bytes,
                                    const mmd8_debug_taps* taps /*HOST struct or NULL*/, void* stream);

/* The same layer applied to activations that arrive in blockwise-coded form (the hidden state a
 * shard receives from its predecessor: "Compression techniques", item 1 feeding item 2):
 *     X = dequantize_blockwise(codes, absmax, block)        as [M, K], contiguous (ldx = K)
 *     Y = mixed_int8_linear(X, ...)
 * with every value identical to the two calls made one after the other.  X_decoded (DEVICE [M*K],
 * 16-byte aligned) receives X, which the caller usually needs as well (residual connection).  For more
 * than 128 rows and K <= 16384 the decoding happens inside the preparation kernel of the layer: the
 * hidden state is read once, as codes.  Requirements: those of both calls (block a multiple of 64 in
 * [64, 4096]; codes 16-byte aligned; K % 16 == 0; ...). */
int mmd8_mixed_int8_linear_from_codes(const uint8_t* codes /*DEVICE [M*K]*/, const float* absmax /*DEVICE [ceil(M*K/block)]*/,
                                      int block, int M, int K, mmd8_half* X_decoded /*DEVICE [M*K], written*/,
                                      const int8_t* Wq_packed /*DEVICE*/, uint32_t Wq_layout, const float* col_absmax /*DEVICE [N]*/, int N,
                                      const mmd8_half* bias /*DEVICE [N] or NULL*/, float tau,
                                      mmd8_half* Y /*DEVICE*/, int ldy,
                                      void* workspace /*DEVICE*/, size_t workspace_bytes,
                                      const mmd8_debug_taps* taps /*HOST struct or NULL*/, void* stream);

/* The same layer followed by the GELU activation (the first linear of a transformer MLP block, e.g. of a
 * ViT: bias, then GELU), applied in the kernel that writes the output:
 *     Y[m,n] = f16( gelu( f16(the three terms of mmd8_mixed_int8_linear) ) ),   gelu(x) = x Phi(x) = x erfc(-x/sqrt 2)/2
 * i.e. the exact (erf-based) form evaluated in fp32 on the fp16 layer output, as the two steps made one after
 * the other give.  Arguments, requirements, workspace and errors as for mmd8_mixed_int8_linear. */
int mmd8_mixed_int8_linear_gelu(const mmd8_half* X /*DEVICE*/, int M, int K, int ldx,
                                const int8_t* Wq_packed /*DEVICE*/, uint32_t Wq_layout, const float* col_absmax /*DEVICE [N]*/, int N,
                                const mmd8_half* bias /*DEVICE [N] or NULL*/, float tau,
                                mmd8_half* Y /*DEVICE*/, int ldy,
                                void* workspace /*DEVICE*/, size_t workspace_bytes,
                                const mmd8_debug_taps* taps /*HOST struct or NULL*/, void* stream);

/* The same layer added onto a residual stream (the attention output projection and the second MLP linear of
 * a transformer block), in the kernel that writes the output:
 *     Y[m,n] = f16( f16(the three terms of mmd8_mixed_int8_linear) + residual[m,n] )        an fp16 addition
 * as the layer followed by an fp16 addition gives.  residual: DEVICE [M][ldr] fp16, 16-byte aligned, ldr >= N,
 * ldr % 8 == 0; it may be the very buffer Y (with ldr == ldy): the stream is then updated in place.  Other
 * arguments, requirements, workspace and errors as for mmd8_mixed_int8_linear. */
int mmd8_mixed_int8_linear_residual(const mmd8_half* X /*DEVICE*/, int M, int K, int ldx,
                                    const int8_t* Wq_packed /*DEVICE*/, uint32_t Wq_layout, const float* col_absmax /*DEVICE [N]*/, int N,
                                    const mmd8_half* bias /*DEVICE [N] or NULL*/, float tau,
                                    const mmd8_half* residual /*DEVICE [M][ldr]*/, int ldr,
                                    mmd8_half* Y /*DEVICE*/, int ldy,
                                    void* workspace /*DEVICE*/, size_t workspace_bytes,
                                    const mmd8_debug_taps* taps /*HOST struct or NULL*/, void* stream);

/* The same layer with its result leaving in blockwise-coded form (the hidden state a shard hands to its
 * successor: "Compression techniques", item 2 feeding item 1):
 *     Y = mixed_int8_linear(X, ...)                           fp16, as above
 *     H[m,n] = f16( Y[m,n] + residual[m,n] )                  fp16 addition; H = Y when residual is NULL
 *     (codes, absmax) = quantize_blockwise(H as M*N contiguous elements, row after row, block)
 * with every value identical to those steps made one after the other.  residual: NULL, or DEVICE [M][ldr]
 * fp16 (the residual stream the layer's output is added to), 16-byte aligned, ldr >= N, ldr % 8 == 0.
 * codes: DEVICE [M*N], 16-byte aligned; absmax: DEVICE [ceil(M*N/block)].  H: NULL, or DEVICE [M*N] fp16
 * (contiguous, 16-byte aligned) that receives the encoded tensor itself.  The layer's last kernel does the
 * encoding where no block is shared between its workgroups: up to 64 rows, up to 128 rows when
 * 64*N % block == 0, more rows when block is 64, 128 or 256 and divides N; otherwise (and for one or two rows,
 * where the layer is a single kernel) the encoder runs after the layer.  Requirements: those of mmd8_mixed_int8_linear and of mmd8_quantize_blockwise; workspace of at
 * least mmd8_linear_to_codes_workspace_bytes(M, K, N, block) bytes, set up and reused like any other
 * workspace of the layer.  Errors as for the two calls; nothing is launched when one is returned. */
size_t mmd8_linear_to_codes_workspace_bytes(int M, int K, int N, int block);
int mmd8_mixed_int8_linear_to_codes(const mmd8_half* X /*DEVICE*/, int M, int K, int ldx,
                                    const int8_t* Wq_packed /*DEVICE*/, uint32_t Wq_layout, const float* col_absmax /*DEVICE [N]*/, int N,
                                    const mmd8_half* bias /*DEVICE [N] or NULL*/, float tau,
                                    const mmd8_half* residual /*DEVICE [M][ldr] or NULL*/, int ldr, int block,
                                    uint8_t* codes /*DEVICE [M*N], written*/, float* absmax /*DEVICE, written*/,
                                    mmd8_half* H /*DEVICE [M*N] or NULL, written*/,
                                    void* workspace /*DEVICE*/, size_t workspace_bytes,
                                    const mmd8_debug_taps* taps /*HOST struct or NULL*/, void* stream);

/* The layer with a low-rank adapter ("BSNS with parameter-efficient fine-tuning via adapters":
 * W' = W + B A with A in R^{r x n}, B in R^{n x r}, r << n), the base weight staying in its 8-bit form:
 *     T[m,j] = f16( sum_k X[m,k] * A[j,k] )                      (fp32 accumulation, one rounding)
 *     Y[m,n] = f16( the three terms of mmd8_mixed_int8_linear + sum_j T[m,j] * B[n,j] )
 * lora_A: [r][K] fp16, row-major, contiguous; lora_B: [N][r] fp16, row-major, contiguous (a scale
 * such as alpha / r is the caller's to fold into B); lora_T: NULL, or [M][r] fp16 that receives T.
 * Requirements: those of mmd8_mixed_int8_linear; r a multiple of 8 with 8 <= r <= MMD8_MAX_LORA_RANK
 * (else MMD8_E_SHAPE; pad a smaller adapter with zero rows of A and zero columns of B); lora_A, lora_B,
 * lora_T 16-byte aligned; workspace of at least mmd8_linear_lora_workspace_bytes(M, K, N, r) bytes,
 * set up and reused like any other workspace of the layer. */
#define MMD8_MAX_LORA_RANK 64
size_t mmd8_linear_lora_workspace_bytes(int M, int K, int N, int r);
int mmd8_mixed_int8_linear_lora(const mmd8_half* X /*DEVICE*/, int M, int K, int ldx,
                                const int8_t* Wq_packed /*DEVICE*/, uint32_t Wq_layout, const float* col_absmax /*DEVICE [N]*/, int N,
                                const mmd8_half* bias /*DEVICE [N] or NULL*/, float tau,
                                const mmd8_half* lora_A /*DEVICE [r*K]*/, const mmd8_half* lora_B /*DEVICE [N*r]*/, int r,
                                mmd8_half* lora_T /*DEVICE [M*r] or NULL, written*/,
                                mmd8_half* Y /*DEVICE*/, int ldy,
                                void* workspace /*DEVICE*/, size_t workspace_bytes,
                                const mmd8_debug_taps* taps /*HOST struct or NULL*/, void* stream);

/* HOST helper: the bit pattern of the smallest non-negative fp16 value that is >= tau (0 for
 * tau <= 0, 0x7c00 = +inf when no finite fp16 value reaches tau).  The outlier scan compares fp16
 * magnitudes against this pattern, which is equivalent to |x| >= tau for every fp16 x. */
uint32_t mmd8_threshold_fp16_pattern(float tau);

#ifdef __cplusplus
}
#endif
#endif /* MMD8_H */
