// Decode-shaped (at most 64 tokens) mixed int8 GEMM ("Compression techniques", item 2): bound by
// streaming the int8 weights once from HBM, not by the matrix pipes.
//
//   acc[m,n] = sum_k Xq[m,k] Wt[n,k]                                   v_mfma_i32_32x32x32_i8
//   Y[m,n]   = f16( acc r[m] c[n] / 127^2 + sum_{k critical} X[m,k] f16(Wt[n,k] c[n]/127) + bias[n] )
//
// No weight byte is used by more than one wave, so the weights go straight from HBM into the
// registers of the lane that feeds them to the MFMA (no LDS): a wave owns 32 rows of Wt (32 output
// columns) and reads their 64-byte slabs; the blocked layout is fragment-major, so each of the two
// loads per slab is 1 KB of consecutive addresses.  The activation side of a slab is shared by the
// waves of a workgroup through LDS.  When there are too few weight panels to give every CU a
// workgroup, the K range is split between workgroups, which write fp32 partial outputs that a
// second small kernel adds in a fixed order (the result does not depend on timing).
//
// Heavy-tailed decode activations flag a large share of the feature dimensions, so the 16-bit part
// is a second product over the same weights rather than a small correction.  For a slab that holds
// a critical column the lane turns the weight bytes it already has into fp16 and multiplies them
// with Xf, a copy of X in which the non-critical columns are zero (written by the pack kernel).
// To keep that conversion off the critical path the fp16 operand is the integer code itself (exact
// in fp16, one byte permute and one packed fp16 subtraction per two codes) and the column step
// c[n]/127 is applied in fp32 to the accumulated sum: the sum over the critical columns of
// X[m,k] q[n,k] c[n]/127 with one rounding at the end, instead of rounding each dequantized weight
// to fp16 first.  The two differ by at most the fp16 rounding of the weights (2^-11 relative per
// term), far inside the tolerance of the fp16 output.  A slab without a critical column skips the
// 16-bit part (the same decision for the whole workgroup).
#include <type_traits>
#include <utility>

#include <atomic>

#include "codec_device.h"
#include "common.h"
#include "operand_layout.h"
#include "skinny.h"

namespace mmd8 {

// ------------------------------------------------------------------------------------------------
// If every wave fetched its own copy of the activation fragments from L2, that would be up to 6
// times the bytes of the weights it streams (64 rows).  So the kWaves waves of a workgroup own
// neighbouring 32-column groups of one weight panel and walk the same slabs together: the
// activation side of a slab (int8 codes and the fp16 critical columns, kMT 32-row groups each) is
// fetched once per workgroup, parked in LDS (a ring of four buffers) and read from there by every
// wave; the weights go from HBM straight into the registers of the lane that feeds them to the
// MFMA, three slabs ahead.  All waits are the compiler's.  Measured per workgroup: about 19 GB/s
// of weights at 64 rows (the MFMAs and the code-to-fp16 conversions of a slab take about as long
// as its 16 KB take to arrive), so every CU must have a workgroup.
// ------------------------------------------------------------------------------------------------
template <int MT, int WAVES>
struct PanelCfg {
  static constexpr int kMT = MT, kWaves = WAVES;
  static constexpr int kThreads = WAVES * kWave;
  static constexpr int kCols = WAVES * 32;
  static constexpr int XQ_BYTES = MT * 2048, XF_BYTES = MT * 4096, STAGE_BYTES = XQ_BYTES + XF_BYTES;
  static constexpr int kPieces = STAGE_BYTES / 1024;               // 1 KB pieces of a slab's activation side
  static constexpr int kFetch = (kPieces + WAVES - 1) / WAVES;     // per wave and slab; surplus ones repeat the last
  static constexpr int kMaxSlabs = MMD8_MAX_K / kSlabBytes;        // flags "slab holds a critical column"
};

// kPrep (at most kPanelPrepMaxM rows): the activation side is not fetched from packed operands but made here.
// Every workgroup streams the rows of X once for the row scales (the maximum of the magnitudes below the
// threshold, as the scan kernel finds it), keeps the columns of its own K range in LDS with one "critical" flag
// per column, and writes the codes and the fp16 critical columns of a slab into the ring two slabs ahead of the
// MFMAs: wave w owns the 16-column piece w % 4 of the slab, a lane one column of one of four rows.  The
// arithmetic is the pack kernel's (IEEE 127 / r, rint, clamp; critical columns zero in the codes and kept in the
// fp16 copy).  Rows of the ring beyond M are zeroed once and never written.
template <class Cfg, bool kSplit, bool kTap, bool kPrep>
__global__ __launch_bounds__(Cfg::kThreads, 2) void k_gemm_panel(const SkinnyArgs a) {
  constexpr int MT = Cfg::kMT, WAVES = Cfg::kWaves;
  static_assert(!kPrep || MT == 1, "own preparation is for a few rows");
  __shared__ __attribute__((aligned(16))) int8_t s_x[4][Cfg::STAGE_BYTES];
  __shared__ uint8_t s_any[Cfg::kMaxSlabs];
  __shared__ __attribute__((aligned(16))) uint16_t s_row[kPrep ? kPanelPrepMaxRowSlabs * kSlabBytes : 8];   // [M][cnt x 64]
  __shared__ __attribute__((aligned(16))) uint8_t s_crit[kPrep ? kPanelPrepMaxSlabs * kSlabBytes : 16];                                    // [cnt x 64]
  __shared__ uint32_t s_part[kPanelPrepMaxM][WAVES];
  __shared__ float s_r[kPanelPrepMaxM], s_scale[kPanelPrepMaxM];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int lr = lane & 31, lg = lane >> 5;
  reset_column_flags(a.flag_reset, a.Kpad);
  const int tile = blockIdx.x % a.tiles_n, split = blockIdx.x / a.tiles_n;
  const int n0 = tile * Cfg::kCols + wave * 32;                    // < Npad: the padding rows of Wt are zero
  const int n = n0 + lr;
  const int s_begin = split * a.slabs_per_split;
  const int cnt = min(a.n_slabs, s_begin + a.slabs_per_split) - s_begin;   // >= 1 by construction of the plan

  const int8_t* wgrp = a.Wt + (size_t)(n0 >> 8) * a.n_slabs * kBlockBytes + (size_t)((n0 & 255) >> 5) * 2048 + lane * 16 +
                       (size_t)s_begin * kBlockBytes;
  if constexpr (!kPrep) {
    for (int t = threadIdx.x; t < cnt; t += Cfg::kThreads) {
      const v4u* mk = reinterpret_cast<const v4u*>(a.mask + (size_t)(s_begin + t) * kSlabBytes);
      const v4u m = mk[0] | mk[1] | mk[2] | mk[3];
      s_any[t] = (m[0] | m[1] | m[2] | m[3]) != 0;
    }
  }

  // piece i of a slab's activation side: first the int8 codes (MT 32-row groups x 2 k-steps), then
  // the fp16 pieces (MT groups x 4); the first MT groups of a slab are contiguous in both arrays
  const int8_t* x_src[Cfg::kFetch];
  int x_dst[Cfg::kFetch], x_step[Cfg::kFetch];
#pragma unroll
  for (int d = 0; d < Cfg::kFetch; ++d) {
    const int i = min(wave + d * WAVES, Cfg::kPieces - 1);
    const bool codes = i < MT * 2;
    x_src[d] = (codes ? a.Xq + (size_t)s_begin * kBlockBytes + i * 1024
                      : reinterpret_cast<const int8_t*>(a.Xf) + (size_t)s_begin * 8192 + (i - MT * 2) * 1024) + lane * 16;
    x_step[d] = codes ? kBlockBytes : 8192;
    x_dst[d] = i * 1024 + lane * 16;
  }
  auto fetch_x = [&](int j, v4i (&xr)[Cfg::kFetch]) {
    if constexpr (kPrep) return;
#pragma unroll
    for (int d = 0; d < Cfg::kFetch; ++d) xr[d] = *reinterpret_cast<const v4i*>(x_src[d] + (size_t)j * x_step[d]);
  };
  // kPrep: slab j of the workgroup's range -> ring buffer `stage` (see the kernel's header comment)
  const int row_stride = cnt * kSlabBytes;                         // elements of s_row per row
  auto make_slab = [&](int j, int stage) {
    const int ch = wave & 3, ks = ch >> 1, g = ch & 1, col = lane & 15;
    const int kl = j * kSlabBytes + ch * 16 + col;
    const bool crit = s_crit[kl] != 0;
    for (int m = (wave >> 2) * 4 + (lane >> 4); m < a.M; m += WAVES) {
      const uint32_t x = s_row[m * row_stride + kl];
      const uint32_t code = crit ? 0u : to_code_byte(half_lo_to_float(x), s_scale[m]);
      s_x[stage][ks * 1024 + (32 * g + m) * 16 + col] = (int8_t)code;
      *reinterpret_cast<uint16_t*>(&s_x[stage][Cfg::XQ_BYTES + (2 * ks + (col >> 3)) * 1024 + (32 * g + m) * 16 +
                                               (col & 7) * 2]) = crit ? (uint16_t)x : (uint16_t)0;
    }
  };
  auto park_x = [&](int stage, const v4i (&xr)[Cfg::kFetch], int j) {   // j: the slab these pieces belong to
    if constexpr (kPrep) {
      make_slab(j, stage);
    } else {
#pragma unroll
      for (int d = 0; d < Cfg::kFetch; ++d) *reinterpret_cast<v4i*>(&s_x[stage][x_dst[d]]) = xr[d];
    }
  };
  struct W2 {
    v4i w[2];
  };
  auto fetch_w = [&](int j, W2& f) {
    const int8_t* p = wgrp + (size_t)j * kBlockBytes;
    f.w[0] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(p));
    f.w[1] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(p + 1024));
  };

  v16i acc[MT];
  v16f accf[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[mt][e] = 0, accf[mt][e] = 0.0f;

  struct Frags {
    v4i x[MT][2];      // int8 codes, k-steps 0 and 1
    v8h xf[MT][4];     // fp16 critical columns, pieces 2 ks + t (valid when the slab has any)
  };
  auto read_frags = [&](int stage, bool any, Frags& g) {
    const int8_t* base = &s_x[stage][lane * 16];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) g.x[mt][ks] = *reinterpret_cast<const v4i*>(base + mt * 2048 + ks * 1024);
    if (any) {                                                     // the same for the whole workgroup
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int p = 0; p < 4; ++p)
          g.xf[mt][p] = *reinterpret_cast<const v8h*>(base + Cfg::XQ_BYTES + mt * 4096 + p * 1024);
    }
  };
  auto multiply = [&](bool any, const Frags& g, const W2& f) {
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[mt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(g.x[mt][ks], f.w[ks], acc[mt], 0, 0, 0);
    if (any) {
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const v4u wu = __builtin_bit_cast(v4u, f.w[ks]) ^ 0x80808080u;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const v8h wh = codes_to_half8(wu, t);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) accf[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(g.xf[mt][2 * ks + t], wh, accf[mt], 0, 0, 0);
        }
      }
    }
  };

  // Software pipeline (past the end the requests repeat the last slab: L2 hits, uniform loop body).
  // In iteration j: request the activation pieces of slab j + 5 and the weights of slab j + 3; read the fragments
  // of slab j + 1 from LDS (they overlap the MFMAs of slab j, whose fragments were read an iteration
  // ago); park the pieces of slab j + 2 (requested three iterations ago) in the buffer that slab j - 1
  // used (a ring of four, so that every index is static in a loop unrolled four times); barrier.
  const int last = cnt - 1;
  W2 f[4];
  // Activation pieces on their way from L2 to LDS: slab s >= 1 travels in xr[s % 4] (slab 0 in x0), requested three
  // iterations before it is parked (the pieces were written by another kernel, possibly through another XCD's
  // L2; four registers per set).
  v4i x0[Cfg::kFetch], xr[4][Cfg::kFetch];
  Frags fr[2];
  // (requests in the order the loop issues them, so that what the compiler counts as in flight on entry to the
  // loop is what it counts when coming round)
  fetch_x(0, x0);
  fetch_x(min(1, last), xr[1]);
  fetch_x(min(2, last), xr[2]);
  fetch_w(0, f[0]);
  fetch_x(min(3, last), xr[3]);
  fetch_w(min(1, last), f[1]);
  fetch_x(min(4, last), xr[0]);
  fetch_w(min(2, last), f[2]);
  if constexpr (kPrep) {
    // (the weight requests above are in flight meanwhile)
    for (int i = threadIdx.x; i < 4 * Cfg::STAGE_BYTES / 16; i += Cfg::kThreads)
      reinterpret_cast<v4u*>(&s_x[0][0])[i] = v4u{0, 0, 0, 0};
    const us2 th2 = __builtin_bit_cast(us2, a.th | (a.th << 16));
    // rows innermost, so that the loads of all rows are in flight together
    us2 best[kPanelPrepMaxM];
#pragma unroll
    for (int m = 0; m < kPanelPrepMaxM; ++m) best[m] = __builtin_bit_cast(us2, 0u);
    for (int c = threadIdx.x; c < a.K / 8; c += Cfg::kThreads) {
      v4u raw[kPanelPrepMaxM];
#pragma unroll
      for (int m = 0; m < kPanelPrepMaxM; ++m) {
        raw[m] = v4u{0, 0, 0, 0};
        if (m < a.M) raw[m] = *reinterpret_cast<const v4u*>(a.X + (size_t)m * a.ldx + c * 8);
      }
#pragma unroll
      for (int m = 0; m < kPanelPrepMaxM; ++m)
#pragma unroll
        for (int w = 0; w < 4; ++w)   // per half, wraps mod 2^16: entries below the threshold get the top bit
          best[m] = __builtin_elementwise_max(best[m], (us2)(__builtin_bit_cast(us2, raw[m][w] & 0x7fff7fffu) - th2));
    }
    // this workgroup's columns (the K padding reads as zero)
    for (int c = threadIdx.x; c < cnt * (kSlabBytes / 8); c += Cfg::kThreads) {
      const int k = s_begin * kSlabBytes + c * 8;
      v4u raw[kPanelPrepMaxM];
#pragma unroll
      for (int m = 0; m < kPanelPrepMaxM; ++m) {
        raw[m] = v4u{0, 0, 0, 0};
        if (m < a.M && k < a.K) raw[m] = *reinterpret_cast<const v4u*>(a.X + (size_t)m * a.ldx + k);
      }
#pragma unroll
      for (int m = 0; m < kPanelPrepMaxM; ++m)
        if (m < a.M) *reinterpret_cast<v4u*>(&s_row[m * row_stride + c * 8]) = raw[m];
    }
#pragma unroll
    for (int m = 0; m < kPanelPrepMaxM; ++m) {
      if (m < a.M) {                                                  // the same for every lane
        const uint32_t both = __builtin_bit_cast(uint32_t, best[m]);
        const uint32_t wmax = wave_max_u32(max(both & 0xffffu, both >> 16));
        if (lane == 0) s_part[m][wave] = wmax;
      }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < row_stride; c += Cfg::kThreads) {
      bool crit = false;
      for (int m = 0; m < a.M; ++m) crit = crit || (s_row[m * row_stride + c] & 0x7fffu) >= a.th;
      s_crit[c] = crit ? 1 : 0;
    }
    if ((int)threadIdx.x < a.M) {
      uint32_t mm = 0;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) mm = max(mm, s_part[threadIdx.x][w]);
      // top bit set: an entry below the threshold exists and its pattern is mm + th (mod 2^16)
      const float r = (mm & 0x8000u) ? half_lo_to_float((mm + a.th) & 0xffffu) : 0.0f;
      s_r[threadIdx.x] = r;
      s_scale[threadIdx.x] = (r == 0.0f) ? 0.0f : 127.0f / r;       // IEEE division
    }
    __syncthreads();
    for (int t = threadIdx.x; t < cnt; t += Cfg::kThreads) {         // "slab t holds a critical column"
      const v4u* fl = reinterpret_cast<const v4u*>(&s_crit[t * kSlabBytes]);
      const v4u m = fl[0] | fl[1] | fl[2] | fl[3];
      s_any[t] = (m[0] | m[1] | m[2] | m[3]) != 0;
    }
  }
  park_x(0, x0, 0);
  park_x(1, xr[1], min(1, last));
  __syncthreads();
  // The flags of the next 64 slabs as one scalar mask (bit i: slab base + i, the last slab repeated past the end),
  // refilled every 64 iterations: no LDS read and no vector compare between a slab's fragments and its MFMAs.
  uint64_t any_mask = __builtin_amdgcn_ballot_w64(s_any[min(lane, last)] != 0);
  bool any_next = any_mask & 1u;
  read_frags(0, any_next, fr[0]);
  auto iteration = [&](int j, auto u_tag) {
    constexpr int u = decltype(u_tag)::value;                        // j % 4
    const bool any_cur = any_next;
    if constexpr (u == 3) {                                          // 64 is a multiple of four: only here can j + 1 start a window
      if (((j + 1) & 63) == 0) any_mask = __builtin_amdgcn_ballot_w64(s_any[min(j + 1 + lane, last)] != 0);
    }
    any_next = (any_mask >> ((j + 1) & 63)) & 1u;
    fetch_x(min(j + 5, last), xr[(u + 1) & 3]);
    fetch_w(min(j + 3, last), f[(u + 3) & 3]);
    read_frags((u + 1) & 3, any_next, fr[(u + 1) & 1]);
    multiply(any_cur, fr[u & 1], f[u & 3]);
    park_x((u + 2) & 3, xr[(u + 2) & 3], min(j + 2, last));
    __syncthreads();
  };
  // Whole groups of four iterations run without a way out in between: with an exit after every iteration the
  // compiler's count of the requests still in flight is merged over all those paths, and it then waits for
  // weights requested one iteration earlier instead of three (every iteration took a whole memory latency).
  int j0 = 0;
  for (; j0 + 4 <= cnt; j0 += 4) {
    iteration(j0, std::integral_constant<int, 0>{});
    iteration(j0 + 1, std::integral_constant<int, 1>{});
    iteration(j0 + 2, std::integral_constant<int, 2>{});
    iteration(j0 + 3, std::integral_constant<int, 3>{});
  }
  if (j0 < cnt) iteration(j0, std::integral_constant<int, 0>{});
  if (j0 + 1 < cnt) iteration(j0 + 1, std::integral_constant<int, 1>{});
  if (j0 + 2 < cnt) iteration(j0 + 2, std::integral_constant<int, 2>{});

  // ---- outputs.  C layout of the 32x32 MFMA: lane = column n (lane % 32), register e = row
  // 8 (e / 4) + 4 (lane / 32) + (e % 4).
  const float cs = (n < a.N) ? a.c[n] / 16129.0f : 0.0f;
  const float step = (n < a.N) ? a.c[n] / 127.0f : 0.0f;
  const float b = (!kSplit && a.bias && n < a.N) ? half_lo_to_float(a.bias[n]) : 0.0f;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int m = mt * 32 + 8 * (e >> 2) + 4 * lg + (e & 3);
      if (m < a.M && n < a.N) {
        const float rm = kPrep ? s_r[m] : a.r[m];
        const float y = (float)acc[mt][e] * (rm * cs) + accf[mt][e] * step;
        if constexpr (kSplit)
          a.partial[((size_t)split * a.M + m) * a.N + n] = y;
        else
          a.Y[(size_t)m * a.ldy + n] = (uint16_t)float_to_half_bits(y + b);
        if constexpr (kTap) {
          if constexpr (kSplit)
            atomicAdd(a.tap_acc + (size_t)m * a.N + n, acc[mt][e]);   // tap buffer zeroed by the launcher
          else
            a.tap_acc[(size_t)m * a.N + n] = acc[mt][e];
        }
      }
    }
}

// Y[m,n] = f16( sum_s partial[s][m][n] + bias[n] + sum_j T[m][j] B[n][j] ), splits added in index
// order, then the bias, then the low-rank term (T: [M][ldt] fp16, B: [N][r] fp16, r a multiple of 8;
// r == 0: no such term).
__global__ __launch_bounds__(256) void k_skinny_finalize(const float* __restrict__ partial, int splits, int M, int N,
                                                         const uint16_t* __restrict__ bias,
                                                         const uint16_t* __restrict__ T, int ldt,
                                                         const uint16_t* __restrict__ B, int r,
                                                         const uint16_t* residual /* may alias Y */, int ldr, int gelu,
                                                         uint16_t* Y, int ldy, uint8_t* flag_reset, int Kpad) {
  reset_column_flags(flag_reset, Kpad);
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)M * N) return;
  const int m = (int)(i / N), n = (int)(i % N);
  float y = 0.0f;
  for (int s = 0; s < splits; ++s) y += partial[(size_t)s * M * N + i];
  if (bias) y += half_lo_to_float(bias[n]);
  if (r > 0) {
    float low = 0.0f;
    for (int j = 0; j < r; j += 8) {
      const v4u t = *reinterpret_cast<const v4u*>(T + (size_t)m * ldt + j);
      const v4u b = *reinterpret_cast<const v4u*>(B + (size_t)n * r + j);
#pragma unroll
      for (int e = 0; e < 4; ++e)
        low += half_lo_to_float(t[e]) * half_lo_to_float(b[e]) + half_hi_to_float(t[e]) * half_hi_to_float(b[e]);
    }
    y += low;
  }
  uint32_t h = float_to_half_bits(y);
  if (gelu) h = gelu_to_half_bits(half_lo_to_float(h));
  if (residual) h = float_to_half_bits(half_lo_to_float(h) + half_lo_to_float(residual[(size_t)m * ldr + n]));
  Y[(size_t)m * ldy + n] = (uint16_t)h;
}

// The same sum as the source of the blockwise encoder (output leaving in coded form, no low-rank term): eight
// neighbouring columns of a row per call; H = f16(Y + residual) is stored where wanted and handed to the encoder.
__device__ const DynamicCode kExitCode = make_dynamic_code();
struct FinalizedHalves {
  const float* partial;
  int splits, N;
  size_t MN;
  const uint16_t* bias;
  const uint16_t* residual;
  int ldr;
  uint16_t* H;            // [M N] or null
  __device__ v4u chunk(size_t e0, int /*valid: N is a multiple of 8, chunks are whole*/) const {
    const int m = (int)(e0 / N), n = (int)(e0 % N);
    float y[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) y[i] = 0.0f;
    // four splits' loads in flight at a time; the additions stay in split order
    int s = 0;
    for (; s + 4 <= splits; s += 4) {
      v4f p0[4], p1[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        p0[u] = *reinterpret_cast<const v4f*>(partial + (size_t)(s + u) * MN + e0);
        p1[u] = *reinterpret_cast<const v4f*>(partial + (size_t)(s + u) * MN + e0 + 4);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < 4; ++i) y[i] += p0[u][i], y[4 + i] += p1[u][i];
    }
    for (; s < splits; ++s) {
      const v4f p0 = *reinterpret_cast<const v4f*>(partial + (size_t)s * MN + e0);
      const v4f p1 = *reinterpret_cast<const v4f*>(partial + (size_t)s * MN + e0 + 4);
#pragma unroll
      for (int i = 0; i < 4; ++i) y[i] += p0[i], y[4 + i] += p1[i];
    }
    if (bias) {
#pragma unroll
      for (int i = 0; i < 8; ++i) y[i] += half_lo_to_float(bias[n + i]);
    }
    v4u h;
#pragma unroll
    for (int w = 0; w < 4; ++w) h[w] = float_to_half_bits(y[2 * w]) | (float_to_half_bits(y[2 * w + 1]) << 16);
    if (residual) {
      const v4u res = *reinterpret_cast<const v4u*>(residual + (size_t)m * ldr + n);
#pragma unroll
      for (int w = 0; w < 4; ++w)
        h[w] = float_to_half_bits(half_lo_to_float(h[w]) + half_lo_to_float(res[w])) |
               (float_to_half_bits(half_hi_to_float(h[w]) + half_hi_to_float(res[w])) << 16);
    }
    if (H) *reinterpret_cast<v4u*>(H + e0) = h;
    return h;
  }
};
__global__ __launch_bounds__(kCodecThreads) void k_skinny_finalize_coded(const FinalizedHalves src, int block,
                                                                         uint8_t* __restrict__ codes,
                                                                         float* __restrict__ absmax,
                                                                         int blocks_per_span, size_t n_spans,
                                                                         uint8_t* flag_reset, int Kpad) {
  reset_column_flags(flag_reset, Kpad);
  encode_spans(src, src.MN, block, codes, absmax, blocks_per_span, n_spans, kExitCode);
}

__global__ void k_fill_i32(int32_t* __restrict__ p, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

// Decode plan: `waves` neighbouring 32-column groups per workgroup.
static SkinnyPlan plan_panel(int M, int K, int N, int waves) {
  SkinnyPlan p;
  p.waves = waves;
  p.n_slabs = packed_k(K) / kSlabBytes;
  p.tiles_n = packed_n(N) / (32 * waves);
  // as many workgroups as the chip holds at once (two of four waves or one of eight per CU), every
  // workgroup with at least 8 slabs, no second round
  const int slots = device_cu_count() * (waves == 4 ? 2 : 1);
  const int want = max(1, min(p.n_slabs / 8, slots / p.tiles_n));
  p.slabs_per_split = ceil_div(p.n_slabs, want);
  p.splits = ceil_div(p.n_slabs, p.slabs_per_split);
  p.partial_bytes = p.splits > 1 ? (size_t)p.splits * M * N * sizeof(float) : 0;
  return p;
}
SkinnyPlan plan_skinny(int M, int K, int N) {
  const SkinnyPlan p4 = plan_panel(M, K, N, 4), p8 = plan_panel(M, K, N, 8);
  // measured on the Llama-7B linears: eight waves per panel beat four (half the LDS fills per weight byte)
  SkinnyPlan p = p8;
  p.partial_bytes = max(p4.partial_bytes, p8.partial_bytes);     // the workspace serves either
  return p;
}

template <class Cfg, bool kSplit, bool kTap, bool kPrep>
static hipError_t launch_panel_one(const SkinnyArgs& a, int splits, hipStream_t stream) {
  hipLaunchKernelGGL((k_gemm_panel<Cfg, kSplit, kTap, kPrep>), dim3(a.tiles_n * splits), dim3(Cfg::kThreads), 0, stream, a);
  return hipGetLastError();
}
template <class Cfg, bool kPrep>
static hipError_t launch_panel_cfg(const SkinnyArgs& a, int splits, hipStream_t stream) {
  const bool split = splits > 1 || a.lora_r > 0 || a.residual || a.codes || a.gelu, tap = a.tap_acc != nullptr;
  if (split)
    return tap ? launch_panel_one<Cfg, true, true, kPrep>(a, splits, stream)
               : launch_panel_one<Cfg, true, false, kPrep>(a, splits, stream);
  return tap ? launch_panel_one<Cfg, false, true, kPrep>(a, splits, stream)
             : launch_panel_one<Cfg, false, false, kPrep>(a, splits, stream);
}
static hipError_t launch_panel(const SkinnyArgs& a, const SkinnyPlan& plan, hipStream_t stream) {
  const bool two = a.M > 32;
  if (a.X) {                                                         // the kernel prepares its own operands
    if (two || !panel_prep_fits(a.M, plan)) return hipErrorInvalidValue;
    return plan.waves == 8 ? launch_panel_cfg<PanelCfg<1, 8>, true>(a, plan.splits, stream)
                           : launch_panel_cfg<PanelCfg<1, 4>, true>(a, plan.splits, stream);
  }
  if (plan.waves == 8)
    return two ? launch_panel_cfg<PanelCfg<2, 8>, false>(a, plan.splits, stream)
               : launch_panel_cfg<PanelCfg<1, 8>, false>(a, plan.splits, stream);
  return two ? launch_panel_cfg<PanelCfg<2, 4>, false>(a, plan.splits, stream)
             : launch_panel_cfg<PanelCfg<1, 4>, false>(a, plan.splits, stream);
}

hipError_t launch_gemm_skinny(SkinnyArgs a, const SkinnyPlan& plan, hipStream_t stream) {
  a.n_slabs = plan.n_slabs;
  a.tiles_n = plan.tiles_n;
  a.slabs_per_split = plan.slabs_per_split;
  // with a low-rank term, an activation, a residual or a coded output the result always goes through the partial
  // buffer: the kernel that sums it adds the term, applies the activation and encodes
  const bool split = plan.splits > 1 || a.lora_r > 0 || a.residual || a.codes || a.gelu, tap = a.tap_acc != nullptr;
  const size_t n = (size_t)a.M * a.N;
  if (split && tap) hipLaunchKernelGGL(k_fill_i32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, a.tap_acc, n);
  if (a.flag_reset_late && !split) return hipErrorInvalidValue;    // no kernel after the panel kernel to clear them
  hipError_t e = launch_panel(a, plan, stream);
  if (e != hipSuccess) return e;
  if (split && a.codes) {
    // spans of about 2048 elements (every thread of the workgroup has a chunk), whole blocks each
    const int blocks_per_span = a.code_block >= 2048 ? 1 : 2048 / a.code_block;
    const size_t span = (size_t)blocks_per_span * a.code_block, n_spans = (n + span - 1) / span;
    const FinalizedHalves src = {a.partial, plan.splits, a.N, n, a.bias, a.residual, a.ldr, a.Y};
    hipLaunchKernelGGL(k_skinny_finalize_coded, dim3((unsigned)n_spans), dim3(kCodecThreads), 0, stream, src, a.code_block,
                       a.codes, a.code_absmax, blocks_per_span, n_spans, a.flag_reset_late, a.Kpad);
    e = hipGetLastError();
  } else if (split) {
    hipLaunchKernelGGL(k_skinny_finalize, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, a.partial, plan.splits,
                       a.M, a.N, a.bias, a.lora_T, a.lora_ldt, a.lora_B, a.lora_r, a.residual, a.ldr, a.gelu, a.Y, a.ldy,
                       a.flag_reset_late, a.Kpad);
    e = hipGetLastError();
  }
  return e;
}

// ------------------------------------------------------------------------------------------------
// One or two rows: the whole layer in one kernel.  A workgroup owns 32 output columns (one 32-row group of
// Wt); wave w of its eight takes slabs w, w + 8, ... of the K range, straight from HBM into registers four
// slabs ahead, with no barrier in the loop: the activation side is read-only by then.  It is made once per
// workgroup, for the whole of K, as in the kPrep panel kernel (row scales from a pass over the rows, then
// codes with the critical columns zero and an fp16 copy that keeps only them), stored as plain rows in LDS;
// a lane builds its MFMA fragment from the row it stands for and lanes beyond M feed zeros.  The eight partial
// results meet in LDS: the int32 sums are exact, the fp32 sums of the 16-bit part are added in wave order, so
// the output does not depend on timing.  No split between workgroups, hence no partial outputs in HBM and no
// second kernel.
// ------------------------------------------------------------------------------------------------
// kCols: output columns per workgroup.  32 (one group of Wt, v_mfma_i32_32x32x32_i8) by default; 16 (half a group,
// v_mfma_i32_16x16x64_i8 / v_mfma_f32_16x16x32_f16, whose lanes take the same 16-byte pieces of the blocked layout in
// another order) when 32 would leave compute units without a workgroup (N up to 8192 on 256 of them).  (Two groups
// per workgroup, for shapes with more groups than the chip holds workgroups at once, was slower: the registers then
// allow a prefetch of only two slabs, and the 4096 -> 22016 linear took 29.9 us instead of 21.6.)
constexpr int kRowsAhead = 4;   // weight slabs a wave has requested ahead of the one it multiplies (2 KB each); 8: slower (registers: 4 instead of 7 waves per SIMD; a 7B layer at one token 64 us instead of 56)
template <bool kTap, int kCols>
__global__ __launch_bounds__(512, 4) void k_gemm_rows(const SkinnyArgs a) {
  static_assert(kCols == 32 || kCols == 16, "one group of 32 weight rows, or half of one");
  constexpr int WAVES = 8, kThreads = WAVES * kWave, kAhead = kRowsAhead;
  constexpr int kPieces = kCols == 32 ? 2 : 1;                       // 16-byte weight pieces per lane and slab
  extern __shared__ __attribute__((aligned(16))) int8_t s_ops[];     // [M][Kpad] codes, then [M][Kpad] fp16
  __shared__ uint8_t s_any[MMD8_MAX_K / kSlabBytes];
  __shared__ uint32_t s_part[kRowsMaxM][WAVES];
  __shared__ float s_r[kRowsMaxM], s_scale[kRowsMaxM];
  __shared__ uint8_t s_over[kRowsMaxOperandBytes / 3 / 8];   // per 8-column chunk, rows one after the other: bits "at or above the threshold"
  __shared__ int32_t s_acc[WAVES][kRowsMaxM][kCols];
  __shared__ float s_accf[WAVES][kRowsMaxM][kCols];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  // the operand row / output column a lane stands for, and which 16-byte piece of the k range it holds
  const int lr = lane & (kCols - 1), lg = lane / kCols;
  const int n_slabs = a.n_slabs, Kpad = n_slabs * kSlabBytes;
  reset_column_flags(a.flag_reset, Kpad);
  const int n0 = blockIdx.x * kCols;                                 // < Npad: the grid covers whole groups only
  int8_t* s_code = s_ops;
  uint16_t* s_xf = reinterpret_cast<uint16_t*>(s_ops + (size_t)a.M * Kpad);

  const int mine = wave < n_slabs ? (n_slabs - wave + WAVES - 1) / WAVES : 0;   // slabs of this wave
  // a group of 32 weight rows is 2 KB per slab: [k-step 0..1][lane group 0..1][row 0..31] 16-byte pieces
  const int8_t* wgrp = a.Wt + (size_t)(n0 >> 8) * n_slabs * kBlockBytes + (size_t)((n0 & 255) >> 5) * 2048 +
                       (kCols == 32 ? lane * 16 : (lg >> 1) * 1024 + (32 * (lg & 1) + (n0 & 16) + lr) * 16);
  struct W2 {
    v4i w[kPieces];
  };
  auto fetch_w = [&](int i, W2& f) {                                  // this wave's i-th slab (clamped past the end)
    const int slab = wave + WAVES * min(i, max(mine - 1, 0));
    const int8_t* p = wgrp + (size_t)min(slab, n_slabs - 1) * kBlockBytes;
#pragma unroll
    for (int ks = 0; ks < kPieces; ++ks) f.w[ks] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(p + ks * 1024));
  };
  W2 f[kAhead];
#pragma unroll
  for (int i = 0; i < kAhead; ++i) fetch_w(i, f[i]);

  // ---- the activation side, once per workgroup (the weight requests above are in flight meanwhile).  The rows
  // are read once: a thread keeps its 8-column chunks (at most kChunks, rows and columns flattened) in registers
  // from the pass that finds the row scales to the pass that writes codes and fp16 critical columns.
  constexpr int kChunks = (kRowsMaxOperandBytes / 3 / 8 + kThreads - 1) / kThreads;    // 6
  for (int t = threadIdx.x; t < n_slabs; t += kThreads) s_any[t] = 0;
  const us2 th2 = __builtin_bit_cast(us2, a.th | (a.th << 16));
  const int row_chunks = Kpad / 8, all_chunks = a.M * row_chunks;
  v4u raw[kChunks];
  us2 best[kRowsMaxM];
#pragma unroll
  for (int m = 0; m < kRowsMaxM; ++m) best[m] = __builtin_bit_cast(us2, 0u);
#pragma unroll
  for (int i = 0; i < kChunks; ++i) {
    const int q = i * kThreads + threadIdx.x;
    const int m = q / row_chunks, k = (q - m * row_chunks) * 8;
    raw[i] = v4u{0, 0, 0, 0};
    if (q < all_chunks && k < a.K) raw[i] = *reinterpret_cast<const v4u*>(a.X + (size_t)m * a.ldx + k);
  }
#pragma unroll
  for (int i = 0; i < kChunks; ++i) {
    const int q = i * kThreads + threadIdx.x;
    us2 t = __builtin_bit_cast(us2, 0u);
    uint32_t over = 0;                                                // bit j: |element j| >= threshold
#pragma unroll
    for (int w = 0; w < 4; ++w) {   // per half, wraps mod 2^16: entries below the threshold get the top bit
      const us2 d = (us2)(__builtin_bit_cast(us2, raw[i][w] & 0x7fff7fffu) - th2);
      t = __builtin_elementwise_max(t, d);
      const uint32_t dd = __builtin_bit_cast(uint32_t, d);
      over |= ((~dd >> 15) & 1u) << (2 * w) | ((~dd >> 31) & 1u) << (2 * w + 1);
    }
    if (q < all_chunks) {                                               // (a chunk of the K padding is all zeros)
      const int m = q / row_chunks, c = q - m * row_chunks;
#pragma unroll
      for (int mm = 0; mm < kRowsMaxM; ++mm)
        if (mm == m) best[mm] = __builtin_elementwise_max(best[mm], t);
      s_over[q] = (c * 8 < a.K) ? (uint8_t)over : (uint8_t)0;           // K padding: never critical
    }
  }
#pragma unroll
  for (int m = 0; m < kRowsMaxM; ++m) {
    if (m < a.M) {
      const uint32_t both = __builtin_bit_cast(uint32_t, best[m]);
      const uint32_t wmax = wave_max_u32(max(both & 0xffffu, both >> 16));
      if (lane == 0) s_part[m][wave] = wmax;
    }
  }
  __syncthreads();
  if ((int)threadIdx.x < a.M) {
    uint32_t mm = 0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) mm = max(mm, s_part[threadIdx.x][w]);
    const float r = (mm & 0x8000u) ? half_lo_to_float((mm + a.th) & 0xffffu) : 0.0f;
    s_r[threadIdx.x] = r;
    s_scale[threadIdx.x] = (r == 0.0f) ? 0.0f : 127.0f / r;          // IEEE division
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kChunks; ++i) {
    const int q = i * kThreads + threadIdx.x;
    // one chunk at a time (the 48 conversions of a thread in flight together would take 190 registers): the
    // chunk passes through an opaque statement, and such statements keep their order
    asm volatile("" : "+v"(raw[i][0]), "+v"(raw[i][1]), "+v"(raw[i][2]), "+v"(raw[i][3]) : : "memory");
    if (q < all_chunks) {
      const int m = q / row_chunks, c = q - m * row_chunks, k = c * 8;
      uint32_t crit = 0;                                              // bit j: column k + j is critical
      for (int mm = 0; mm < a.M; ++mm) crit |= s_over[mm * row_chunks + c];
      const float sc = s_scale[m];
      uint32_t code[2] = {0, 0}, xf[4];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint32_t h = (raw[i][j >> 1] >> (16 * (j & 1))) & 0xffffu;
        const bool cr = (crit >> j) & 1u;
        code[j >> 2] |= (cr ? 0u : to_code_byte(half_lo_to_float(h), sc)) << (8 * (j & 3));
      }
#pragma unroll
      for (int w = 0; w < 4; ++w)
        xf[w] = (((crit >> (2 * w)) & 1u) ? (raw[i][w] & 0xffffu) : 0u) | (((crit >> (2 * w + 1)) & 1u) ? (raw[i][w] & 0xffff0000u) : 0u);
      *reinterpret_cast<v2u*>(s_code + (size_t)m * Kpad + k) = v2u{code[0], code[1]};
      *reinterpret_cast<v4u*>(s_xf + (size_t)m * Kpad + k) = v4u{xf[0], xf[1], xf[2], xf[3]};
      if (crit) s_any[k >> 6] = 1;
    }
  }
  __syncthreads();

  // ---- this wave's slabs
  typedef typename std::conditional<kCols == 32, v16i, v4i>::type AccI;
  typedef typename std::conditional<kCols == 32, v16f, v4f>::type AccF;
  AccI acc;
  AccF accf;
#pragma unroll
  for (int e = 0; e < (kCols == 32 ? 16 : 4); ++e) acc[e] = 0, accf[e] = 0.0f;
  const bool row_live = lr < a.M;
  const int row = row_live ? lr : 0;                                  // lanes beyond M read row 0 and feed zeros
  const int8_t* my_code = s_code + (size_t)row * Kpad + lg * 16;
  const uint16_t* my_xf = s_xf + (size_t)row * Kpad + lg * 16;
  // "slab holds a critical column" for this wave's next 64 slabs as one scalar mask (a flag read from LDS when it
  // is needed would stand between the slab's arrival and its MFMAs)
  uint64_t any_mask = 0;
  // this wave's i-th slab: multiply what was requested kAhead slabs ago, then request slab i + kAhead into the
  // registers just used
  auto step = [&](int i, auto u_tag) __attribute__((always_inline)) {
    constexpr int u = decltype(u_tag)::value;                        // i % kAhead
    const W2& w = f[u];
    const int slab = wave + WAVES * i;
    if constexpr (u == 0) {                                          // 64 is a multiple of kAhead: only here can i start a window
      if ((i & 63) == 0) any_mask = __builtin_amdgcn_ballot_w64(s_any[wave + WAVES * min(i + lane, max(mine - 1, 0))] != 0);
    }
    const bool any = (any_mask >> (i & 63)) & 1u;                    // the same for the whole wave
    if constexpr (kCols == 32) {
      // lane group lg of k-step ks holds columns 32 ks + 16 lg .. + 16 of the slab
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        v4i xa = *reinterpret_cast<const v4i*>(my_code + slab * kSlabBytes + ks * 32);
        if (!row_live) xa = v4i{0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(xa, w.w[ks], acc, 0, 0, 0);
      }
      if (any) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          const v4u wu = __builtin_bit_cast(v4u, w.w[ks]) ^ 0x80808080u;
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            v4u xr = *reinterpret_cast<const v4u*>(my_xf + slab * kSlabBytes + ks * 32 + t * 8);
            if (!row_live) xr = v4u{0, 0, 0, 0};
            accf = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, xr), codes_to_half8(wu, t), accf, 0, 0, 0);
          }
        }
      }
    } else {
      // lane group lg (0..3) holds columns 16 lg .. + 16 of the slab; the two fp16 instructions take the two
      // halves of every lane group's piece (any split of the 64 columns does, as long as both operands agree)
      v4i xa = *reinterpret_cast<const v4i*>(my_code + slab * kSlabBytes);
      if (!row_live) xa = v4i{0, 0, 0, 0};
      acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa, w.w[0], acc, 0, 0, 0);
      if (any) {
        const v4u wu = __builtin_bit_cast(v4u, w.w[0]) ^ 0x80808080u;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          v4u xr = *reinterpret_cast<const v4u*>(my_xf + slab * kSlabBytes + t * 8);
          if (!row_live) xr = v4u{0, 0, 0, 0};
          accf = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, xr), codes_to_half8(wu, t), accf, 0, 0, 0);
        }
      }
    }
    fetch_w(i + kAhead, f[u]);
  };
  // Whole groups of kAhead slabs run without a way out in between (with an exit after every slab the compiler
  // waited for every request in flight at the end of each group, emptying the queue of weights four slabs deep).
  static_assert(64 % kAhead == 0, "a window of slab flags starts at the head of a group");
  auto group = [&]<int... kU>(int i0, std::integer_sequence<int, kU...>) __attribute__((always_inline)) {
    (step(i0 + kU, std::integral_constant<int, kU>{}), ...);
  };
  auto tail = [&]<int... kU>(int i0, std::integer_sequence<int, kU...>) __attribute__((always_inline)) {
    (void)((i0 + kU < mine ? (step(i0 + kU, std::integral_constant<int, kU>{}), true) : false) && ...);
  };
  int i0 = 0;
  for (; i0 + kAhead <= mine; i0 += kAhead) group(i0, std::make_integer_sequence<int, kAhead>{});
  tail(i0, std::make_integer_sequence<int, kAhead - 1>{});

  // ---- the eight partial results.  C layout of both MFMA shapes: lane = column (lane % kCols); row m < 4 is
  // register m of the first kCols lanes
  if (lg == 0) {
#pragma unroll
    for (int m = 0; m < kRowsMaxM; ++m) {
      s_acc[wave][m][lr] = acc[m];
      s_accf[wave][m][lr] = accf[m];
    }
  }
  __syncthreads();
  if ((int)threadIdx.x < kCols * a.M) {
    const int m = threadIdx.x / kCols, col = threadIdx.x % kCols, nn = n0 + col;
    if (nn < a.N) {
      int32_t sum = 0;
      float sumf = 0.0f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) sum += s_acc[w][m][col], sumf += s_accf[w][m][col];
      const float cn = a.c[nn];
      float y = (float)sum * (s_r[m] * (cn / 16129.0f)) + sumf * (cn / 127.0f);
      if (a.bias) y += half_lo_to_float(a.bias[nn]);
      if (a.lora_r > 0) {                                             // the low-rank term, as k_skinny_finalize adds it
        float low = 0.0f;
        for (int j = 0; j < a.lora_r; j += 8) {
          const v4u t = *reinterpret_cast<const v4u*>(a.lora_T + (size_t)m * a.lora_ldt + j);
          const v4u b = *reinterpret_cast<const v4u*>(a.lora_B + (size_t)nn * a.lora_r + j);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            low += half_lo_to_float(t[e]) * half_lo_to_float(b[e]) + half_hi_to_float(t[e]) * half_hi_to_float(b[e]);
        }
        y += low;
      }
      uint32_t h = float_to_half_bits(y);
      if (a.gelu) h = gelu_to_half_bits(half_lo_to_float(h));
      if (a.residual) h = float_to_half_bits(half_lo_to_float(h) + half_lo_to_float(a.residual[(size_t)m * a.ldr + nn]));
      a.Y[(size_t)m * a.ldy + nn] = (uint16_t)h;
      if constexpr (kTap) a.tap_acc[(size_t)m * a.N + nn] = sum;
    }
  }
}

// more than the default 64 KB of LDS: an attribute per kernel and device
hipError_t prepare_rows_kernels() {
  static std::atomic<bool> attr_set[64] = {};                      // setting an attribute twice is harmless
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (attr_set[dev]) return hipSuccess;
  const void* fns[4] = {reinterpret_cast<const void*>(&k_gemm_rows<true, 32>), reinterpret_cast<const void*>(&k_gemm_rows<false, 32>),
                        reinterpret_cast<const void*>(&k_gemm_rows<true, 16>), reinterpret_cast<const void*>(&k_gemm_rows<false, 16>)};
  for (const void* fn : fns) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kRowsMaxOperandBytes);
    if (e != hipSuccess) return e;
  }
  attr_set[dev] = true;
  return hipSuccess;
}

hipError_t launch_gemm_rows(SkinnyArgs a, hipStream_t stream) {
  a.n_slabs = packed_k(a.K) / kSlabBytes;
  const int Kpad = a.n_slabs * kSlabBytes;
  if (!a.X || !rows_kernel_fits(a.M, Kpad) || a.codes) return hipErrorInvalidValue;
  // 16 columns per workgroup when 32 would leave compute units without one
  const bool narrow = packed_n(a.N) / 32 <= device_cu_count();
  const unsigned grid = packed_n(a.N) / (narrow ? 16 : 32);
  const size_t lds = (size_t)3 * a.M * Kpad;
  if (hipError_t e = prepare_rows_kernels(); e != hipSuccess) return e;
  if (narrow) {
    if (a.tap_acc)
      hipLaunchKernelGGL((k_gemm_rows<true, 16>), dim3(grid), dim3(512), lds, stream, a);
    else
      hipLaunchKernelGGL((k_gemm_rows<false, 16>), dim3(grid), dim3(512), lds, stream, a);
  } else {
    if (a.tap_acc)
      hipLaunchKernelGGL((k_gemm_rows<true, 32>), dim3(grid), dim3(512), lds, stream, a);
    else
      hipLaunchKernelGGL((k_gemm_rows<false, 32>), dim3(grid), dim3(512), lds, stream, a);
  }
  return hipGetLastError();
}

}  // namespace mmd8
