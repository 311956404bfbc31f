// Decode-shaped (at most 64 tokens) mixed int8 GEMM ("Compression techniques", item 2): bound by
// streaming the int8 weights once from HBM, not by the matrix pipes.
//
//   acc[m,n] = sum_k Xq[m,k] Wt[n,k]                                   v_mfma_i32_32x32x32_i8
//   Y[m,n]   = f16( acc r[m] c[n] / 127^2 + sum_{k critical} X[m,k] f16(Wt[n,k] c[n]/127) + bias[n] )
//
// No weight byte is used by more than one wave, so the weights go straight from HBM into the
// registers of the lane that feeds them to the MFMA (no LDS): a wave owns 32 rows of Wt (32 output
// columns) and reads their 64-byte slabs; the blocked layout is fragment-major, so each of the two
// loads per slab is 1 KB of consecutive addresses.  The
// eight waves of a workgroup share the 32 rows and take every eighth slab; their partial results
// are added in a fixed order through LDS.  When there are too few 32-row tiles to fill the chip,
// the K range is also split between workgroups, which write fp32 partial outputs that a second
// small kernel adds (again in a fixed order, so the result does not depend on timing).
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
// term), far inside the tolerance of the fp16 output.
// A wave whose slabs mostly hold critical columns runs the 16-bit part for every slab (adding
// exact zeros where nothing is flagged), which keeps all loads unconditional and pipelined; a wave
// with few flagged slabs branches around it.
#include "common.h"
#include "operand_layout.h"
#include "skinny.h"

namespace mmd8 {

constexpr int kSkinnyWaves = 8;
constexpr int kSkinnyThreads = kSkinnyWaves * kWave;

// eight weight codes (bytes [8 t, 8 t + 8) of the lane's 16, already XORed with 0x80: u = q + 128)
// -> the integers q as fp16.  The fp16 number 1024 + u has the bit pattern 0x6400 | u.
__device__ inline v8h codes_to_half8(const v4u& wu, int t) {
  typedef _Float16 h2 __attribute__((ext_vector_type(2)));
  v4u out;
#pragma unroll
  for (int d = 0; d < 2; ++d) {
    const uint32_t word = wu[2 * t + d];
    // bytes of {0x64646464 : word}: selectors 0-3 = word bytes, 4-7 = 0x64
    const uint32_t lo = __builtin_amdgcn_perm(0x64646464u, word, 0x04010400u);   // [b0, 0x64, b1, 0x64] little end first
    const uint32_t hi = __builtin_amdgcn_perm(0x64646464u, word, 0x04030402u);   // [b2, 0x64, b3, 0x64]
    const h2 bias = {(_Float16)1152.0f, (_Float16)1152.0f};
    out[2 * d] = __builtin_bit_cast(uint32_t, (h2)(__builtin_bit_cast(h2, lo) - bias));
    out[2 * d + 1] = __builtin_bit_cast(uint32_t, (h2)(__builtin_bit_cast(h2, hi) - bias));
  }
  return __builtin_bit_cast(v8h, out);
}

template <int MT>
struct SkinnyFrags {
  v4i w[2];          // weight codes of the two k-steps
  v4i x[MT][2];      // activation codes
};
template <int MT>
struct SkinnyFragsF {
  v8h xf[MT][4];     // critical columns of X (fp16), pieces (ks, t)
};

template <int MT, bool kSplit, bool kTap>
__global__ __launch_bounds__(kSkinnyThreads) void k_gemm_skinny(const SkinnyArgs a) {
  extern __shared__ __attribute__((aligned(16))) float s_red[];    // [wave][MT * 16][64]
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int lr = lane & 31, lg = lane >> 5;
  reset_column_flags(a.flag_reset, a.Kpad);
  const int tile = blockIdx.x % a.tiles_n, split = blockIdx.x / a.tiles_n;
  const int n = tile * 32 + lr;                                    // < Npad
  const int s_begin = split * a.slabs_per_split;
  const int s_end = min(a.n_slabs, s_begin + a.slabs_per_split);

  // a wave's operand fragment of one k-step is 1 KB contiguous: group of 32 rows, [k-step][lane]
  const int8_t* wgrp = a.Wt + (size_t)(n >> 8) * a.n_slabs * kBlockBytes + (size_t)((n & 255) >> 5) * 2048 + lane * 16;
  const int8_t* xgrp = a.Xq + lane * 16;                           // + mt * 2048: rows 32 mt .. of panel 0

  // Which of this wave's slabs (s_begin + wave + 8 j) hold a critical column: lane j (and j + 64)
  // ORs the 64 mask bytes of its slab, two ballots give up to 128 bits.
  uint64_t any_bits[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int sj = s_begin + wave + kSkinnyWaves * (lane + 64 * h);
    v4u m = v4u{0, 0, 0, 0};
    if (sj < s_end) {
      const v4u* mk = reinterpret_cast<const v4u*>(a.mask + (size_t)sj * kSlabBytes);
      m = mk[0] | mk[1] | mk[2] | mk[3];
    }
    any_bits[h] = __builtin_amdgcn_ballot_w64((m[0] | m[1] | m[2] | m[3]) != 0);
  }

  v16i acc[MT];
  v16f accf[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[mt][e] = 0, accf[mt][e] = 0.0f;

  auto load = [&](int s, SkinnyFrags<MT>& f) {
    const int8_t* wp = wgrp + (size_t)s * kBlockBytes;
    const int8_t* xp = xgrp + (size_t)s * kBlockBytes;
    f.w[0] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wp));
    f.w[1] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wp + 1024));
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      f.x[mt][0] = *reinterpret_cast<const v4i*>(xp + mt * 2048);
      f.x[mt][1] = *reinterpret_cast<const v4i*>(xp + mt * 2048 + 1024);
    }
  };
  // the lane's bytes [8 t, 8 t + 8) of piece 2 ks + lg are k = 64 s + 16 (2 ks + lg) + 8 t ...
  const uint16_t* xf_lane = a.Xf + (size_t)lr * a.Kpad + 16 * lg;
  auto load_f = [&](int s, SkinnyFragsF<MT>& f) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int t = 0; t < 2; ++t)
          f.xf[mt][2 * ks + t] = *reinterpret_cast<const v8h*>(xf_lane + (size_t)mt * 32 * a.Kpad + s * kSlabBytes + 32 * ks + 8 * t);
  };
  auto mfma_i8 = [&](const SkinnyFrags<MT>& f) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      acc[mt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.x[mt][0], f.w[0], acc[mt], 0, 0, 0);
      acc[mt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.x[mt][1], f.w[1], acc[mt], 0, 0, 0);
    }
  };
  auto mfma_f16 = [&](const SkinnyFrags<MT>& f, const SkinnyFragsF<MT>& ff) {
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const v4u wu = __builtin_bit_cast(v4u, f.w[ks]) ^ 0x80808080u;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const v8h wh = codes_to_half8(wu, t);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          accf[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ff.xf[mt][2 * ks + t], wh, accf[mt], 0, 0, 0);
      }
    }
  };

  // this wave's slabs: s0 + 8 j, j < cnt.  Loads run kDepth - 1 slabs ahead and are unconditional
  // (past the end they re-read the last slab), so the compiler can count them.
  constexpr int W8 = kSkinnyWaves;
  constexpr int kDepth = (MT == 1) ? 3 : 2;
  const int s0 = s_begin + wave;
  const int cnt = (s0 < s_end) ? (s_end - s0 + W8 - 1) / W8 : 0;
  const int flagged = __builtin_popcountll(any_bits[0]) + __builtin_popcountll(any_bits[1]);
  if (cnt > 0) {
    const int s_last = s0 + W8 * (cnt - 1);
    SkinnyFrags<MT> f[kDepth];
    if (2 * flagged > cnt) {
      // ---- most slabs hold a critical column: the 16-bit part runs for every slab
      SkinnyFragsF<MT> ff[kDepth];
#pragma unroll
      for (int d = 0; d < kDepth - 1; ++d) {
        load(min(s0 + W8 * d, s_last), f[d]);
        load_f(min(s0 + W8 * d, s_last), ff[d]);
      }
      for (int j = 0; j < cnt; j += kDepth) {
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
          const int sn = min(s0 + W8 * (j + u + kDepth - 1), s_last);
          load(sn, f[(u + kDepth - 1) % kDepth]);
          load_f(sn, ff[(u + kDepth - 1) % kDepth]);
          if (j + u < cnt) {
            mfma_i8(f[u]);
            mfma_f16(f[u], ff[u]);
          }
        }
      }
    } else {
      // ---- few flagged slabs: branch around the 16-bit part (its loads stall the wave when taken)
#pragma unroll
      for (int d = 0; d < kDepth - 1; ++d) load(min(s0 + W8 * d, s_last), f[d]);
      for (int j = 0; j < cnt; j += kDepth) {
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
          load(min(s0 + W8 * (j + u + kDepth - 1), s_last), f[(u + kDepth - 1) % kDepth]);
          if (j + u < cnt) {
            mfma_i8(f[u]);
            if ((any_bits[(j + u) >> 6] >> ((j + u) & 63)) & 1) {
              SkinnyFragsF<MT> ff;
              load_f(s0 + W8 * (j + u), ff);
              mfma_f16(f[u], ff);
            }
          }
        }
      }
    }
  }

  // ---- add the eight waves' results.  C layout of the 32x32 MFMA: lane = column n (lane % 32),
  // register e = row m = 8 (e / 4) + 4 (lane / 32) + (e % 4).
  const float cs = (n < a.N) ? a.c[n] / 16129.0f : 0.0f;
  const float step = (n < a.N) ? a.c[n] / 127.0f : 0.0f;
  constexpr int kPairs = MT * 16;                                   // (m-tile, register) pairs
  float* mine = s_red + (size_t)wave * kPairs * kWave;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int m = mt * 32 + 8 * (e >> 2) + 4 * lg + (e & 3);
      const float y = (float)acc[mt][e] * (a.r[m] * cs) + accf[mt][e] * step;
      mine[(mt * 16 + e) * kWave + lane] = y;
    }
  __syncthreads();
  constexpr int kPairsPerWave = kPairs / kSkinnyWaves;              // 2 or 4
#pragma unroll
  for (int i = 0; i < kPairsPerWave; ++i) {
    const int pr = wave * kPairsPerWave + i, mt = pr >> 4, e = pr & 15;
    float y = 0.0f;
#pragma unroll
    for (int w = 0; w < kSkinnyWaves; ++w) y += s_red[((size_t)w * kPairs + pr) * kWave + lane];
    const int m = mt * 32 + 8 * (e >> 2) + 4 * lg + (e & 3);
    if (m < a.M && n < a.N) {
      if constexpr (kSplit) {
        a.partial[((size_t)split * a.M + m) * a.N + n] = y;
      } else {
        const float b = a.bias ? half_lo_to_float(a.bias[n]) : 0.0f;
        a.Y[(size_t)m * a.ldy + n] = (uint16_t)float_to_half_bits(y + b);
      }
    }
  }
  if constexpr (kTap) {
    // the raw integer accumulators, added the same way (exact in any order)
    __syncthreads();
    int* mine_i = reinterpret_cast<int*>(mine);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int e = 0; e < 16; ++e) mine_i[(mt * 16 + e) * kWave + lane] = acc[mt][e];
    __syncthreads();
    const int* red_i = reinterpret_cast<const int*>(s_red);
#pragma unroll
    for (int i = 0; i < kPairsPerWave; ++i) {
      const int pr = wave * kPairsPerWave + i, mt = pr >> 4, e = pr & 15;
      int v = 0;
#pragma unroll
      for (int w = 0; w < kSkinnyWaves; ++w) v += red_i[((size_t)w * kPairs + pr) * kWave + lane];
      const int m = mt * 32 + 8 * (e >> 2) + 4 * lg + (e & 3);
      if (m < a.M && n < a.N) {
        if constexpr (kSplit)
          atomicAdd(a.tap_acc + (size_t)m * a.N + n, v);           // tap buffer zeroed by the caller
        else
          a.tap_acc[(size_t)m * a.N + n] = v;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// At most 16 rows: v_mfma_i32_16x16x64_i8 takes a whole 64-byte slab of 16 rows per instruction, so
// the activation side needs half the registers and loads of the 32-row form, which leaves room
// for 16 waves per CU with three slabs of weights in flight each.  The 16-bit part runs for every
// slab (exact zeros where nothing is flagged): all loads are unconditional.
//   operands: lane = 16 (16-byte piece of the slab) + row;  result: lane = 16 (row / 4) + column,
//   register = row % 4.
// For the fp16 product (v_mfma_f32_16x16x32_f16, 8 halves per lane) lane group G uses bytes
// [8 h, 8 h + 8) of its own piece G in half-slab pass h: any k order is fine as long as both
// operands agree.
// ------------------------------------------------------------------------------------------------
__device__ inline v8h codes_to_half8_of(const v4i& w, int t) { return codes_to_half8(__builtin_bit_cast(v4u, w) ^ 0x80808080u, t); }

template <bool kSplit, bool kTap>
__global__ __launch_bounds__(kSkinnyThreads, 4) void k_gemm_skinny16(const SkinnyArgs a) {
  __shared__ float s_red[kSkinnyWaves][8][kWave];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int l16 = lane & 15, grp = lane >> 4;
  reset_column_flags(a.flag_reset, a.Kpad);
  const int tile = blockIdx.x % a.tiles_n, split = blockIdx.x / a.tiles_n;
  const int n_base = tile * 32;
  const int s_begin = split * a.slabs_per_split;
  const int s_end = min(a.n_slabs, s_begin + a.slabs_per_split);

  // piece `grp` of row rho of a 32-row group sits at (grp / 2) * 1024 + ((grp % 2) * 32 + rho) * 16
  const int piece = (grp >> 1) * 1024 + ((grp & 1) * 32 + l16) * 16;
  const int8_t* wgrp = a.Wt + (size_t)(n_base >> 8) * a.n_slabs * kBlockBytes + (size_t)((n_base & 255) >> 5) * 2048 + piece;
  const int8_t* xgrp = a.Xq + piece;
  const uint16_t* xf_lane = a.Xf + (size_t)l16 * a.Kpad + 16 * grp;

  struct Frags {
    v4i w[2];      // n rows n_base + 16 h + l16
    v4i x;         // m row l16
    v8h xf[2];     // half-slab passes
  };
  auto load = [&](int s, Frags& f) {
    const int8_t* wp = wgrp + (size_t)s * kBlockBytes;
    f.w[0] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wp));
    f.w[1] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wp + 256));
    f.x = *reinterpret_cast<const v4i*>(xgrp + (size_t)s * kBlockBytes);
    f.xf[0] = *reinterpret_cast<const v8h*>(xf_lane + s * kSlabBytes);
    f.xf[1] = *reinterpret_cast<const v8h*>(xf_lane + s * kSlabBytes + 8);
  };
  v4i acc[2] = {v4i{0, 0, 0, 0}, v4i{0, 0, 0, 0}};
  v4f accf[2] = {v4f{0, 0, 0, 0}, v4f{0, 0, 0, 0}};
  auto compute = [&](const Frags& f) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      acc[h] = __builtin_amdgcn_mfma_i32_16x16x64_i8(f.x, f.w[h], acc[h], 0, 0, 0);
#pragma unroll
      for (int t = 0; t < 2; ++t)
        accf[h] = __builtin_amdgcn_mfma_f32_16x16x32_f16(f.xf[t], codes_to_half8_of(f.w[h], t), accf[h], 0, 0, 0);
    }
  };

  constexpr int W8 = kSkinnyWaves, kDepth = 4;
  const int s0 = s_begin + wave;
  const int cnt = (s0 < s_end) ? (s_end - s0 + W8 - 1) / W8 : 0;
  if (cnt > 0) {
    const int s_last = s0 + W8 * (cnt - 1);
    Frags f[kDepth];
#pragma unroll
    for (int d = 0; d < kDepth - 1; ++d) load(min(s0 + W8 * d, s_last), f[d]);
    for (int j = 0; j < cnt; j += kDepth) {
#pragma unroll
      for (int u = 0; u < kDepth; ++u) {
        load(min(s0 + W8 * (j + u + kDepth - 1), s_last), f[(u + kDepth - 1) % kDepth]);
        if (j + u < cnt) compute(f[u]);
      }
    }
  }

  // ---- add the eight waves' results (fixed order); lane: n = n_base + 16 h + l16, m = 4 grp + e
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int n = n_base + 16 * h + l16;
    const float cs = (n < a.N) ? a.c[n] / 16129.0f : 0.0f;
    const float step = (n < a.N) ? a.c[n] / 127.0f : 0.0f;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      s_red[wave][h * 4 + e][lane] = (float)acc[h][e] * (a.r[4 * grp + e] * cs) + accf[h][e] * step;
  }
  __syncthreads();
  {
    const int pr = wave, h = pr >> 2, e = pr & 3;                 // 8 (h, e) pairs, one per wave
    float y = 0.0f;
#pragma unroll
    for (int w = 0; w < kSkinnyWaves; ++w) y += s_red[w][pr][lane];
    const int m = 4 * grp + e, n = n_base + 16 * h + l16;
    if (m < a.M && n < a.N) {
      if constexpr (kSplit) {
        a.partial[((size_t)split * a.M + m) * a.N + n] = y;
      } else {
        const float b = a.bias ? half_lo_to_float(a.bias[n]) : 0.0f;
        a.Y[(size_t)m * a.ldy + n] = (uint16_t)float_to_half_bits(y + b);
      }
    }
  }
  if constexpr (kTap) {
    __syncthreads();
    int (*red_i)[8][kWave] = reinterpret_cast<int (*)[8][kWave]>(s_red);
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int e = 0; e < 4; ++e) red_i[wave][h * 4 + e][lane] = acc[h][e];
    __syncthreads();
    const int pr = wave, h = pr >> 2, e = pr & 3;
    int v = 0;
#pragma unroll
    for (int w = 0; w < kSkinnyWaves; ++w) v += red_i[w][pr][lane];
    const int m = 4 * grp + e, n = n_base + 16 * h + l16;
    if (m < a.M && n < a.N) {
      if constexpr (kSplit)
        atomicAdd(a.tap_acc + (size_t)m * a.N + n, v);
      else
        a.tap_acc[(size_t)m * a.N + n] = v;
    }
  }
}

// Y[m,n] = f16( sum_s partial[s][m][n] + bias[n] ), splits added in index order
__global__ __launch_bounds__(256) void k_skinny_finalize(const float* __restrict__ partial, int splits, int M, int N,
                                                         const uint16_t* __restrict__ bias,
                                                         uint16_t* __restrict__ Y, int ldy) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)M * N) return;
  const int m = (int)(i / N), n = (int)(i % N);
  float y = 0.0f;
  for (int s = 0; s < splits; ++s) y += partial[(size_t)s * M * N + i];
  if (bias) y += half_lo_to_float(bias[n]);
  Y[(size_t)m * ldy + n] = (uint16_t)float_to_half_bits(y);
}

__global__ void k_fill_i32(int32_t* __restrict__ p, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

SkinnyPlan plan_skinny(int M, int K, int N) {
  SkinnyPlan p;
  p.n_slabs = packed_k(K) / kSlabBytes;
  p.tiles_n = packed_n(N) / 32;
  // Two workgroups fit on a CU.  Pick the K split that minimises (rounds of workgroups) x (slabs per
  // workgroup + a fixed start-up and drain cost worth about 6 slabs), with at least 2 slabs per wave.
  const int slots = 2 * device_cu_count();
  const int max_splits = max(1, p.n_slabs / (2 * kSkinnyWaves));
  int splits = 1;
  long best = -1;
  for (int cand = 1; cand <= min(max_splits, 16); ++cand) {
    const int per = ceil_div(p.n_slabs, cand), real = ceil_div(p.n_slabs, per);
    const long cost = (long)ceil_div(p.tiles_n * real, slots) * (per + 6);
    if (best < 0 || cost < best) best = cost, splits = real;
  }
  p.slabs_per_split = ceil_div(p.n_slabs, splits);
  p.splits = ceil_div(p.n_slabs, p.slabs_per_split);
  p.partial_bytes = p.splits > 1 ? (size_t)p.splits * M * N * sizeof(float) : 0;
  return p;
}

template <int MT, bool kSplit, bool kTap>
static hipError_t launch_one(const SkinnyArgs& a, int splits, hipStream_t stream) {
  const size_t lds = (size_t)kSkinnyWaves * MT * 16 * kWave * sizeof(float);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_skinny<MT, kSplit, kTap>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((k_gemm_skinny<MT, kSplit, kTap>), dim3(a.tiles_n * splits), dim3(kSkinnyThreads), lds, stream, a);
  return hipGetLastError();
}

hipError_t launch_gemm_skinny(SkinnyArgs a, const SkinnyPlan& plan, hipStream_t stream) {
  a.n_slabs = plan.n_slabs;
  a.tiles_n = plan.tiles_n;
  a.slabs_per_split = plan.slabs_per_split;
  const bool split = plan.splits > 1, tap = a.tap_acc != nullptr;
  const int mt = a.M <= 32 ? 1 : 2;
  if (split && tap) {
    const size_t n = (size_t)a.M * a.N;
    hipLaunchKernelGGL(k_fill_i32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, a.tap_acc, n);
  }
  hipError_t e;
#define MMD8_SK(MT_, S_, T_) e = launch_one<MT_, S_, T_>(a, plan.splits, stream)
  if (a.M <= 16) {
    const dim3 grid(a.tiles_n * plan.splits), block(kSkinnyThreads);
    if (split) {
      if (tap) hipLaunchKernelGGL((k_gemm_skinny16<true, true>), grid, block, 0, stream, a);
      else hipLaunchKernelGGL((k_gemm_skinny16<true, false>), grid, block, 0, stream, a);
    } else {
      if (tap) hipLaunchKernelGGL((k_gemm_skinny16<false, true>), grid, block, 0, stream, a);
      else hipLaunchKernelGGL((k_gemm_skinny16<false, false>), grid, block, 0, stream, a);
    }
    e = hipGetLastError();
  } else if (mt == 1) {
    if (split) { if (tap) MMD8_SK(1, true, true); else MMD8_SK(1, true, false); }
    else       { if (tap) MMD8_SK(1, false, true); else MMD8_SK(1, false, false); }
  } else {
    if (split) { if (tap) MMD8_SK(2, true, true); else MMD8_SK(2, true, false); }
    else       { if (tap) MMD8_SK(2, false, true); else MMD8_SK(2, false, false); }
  }
#undef MMD8_SK
  if (e != hipSuccess) return e;
  if (split) {
    const size_t n = (size_t)a.M * a.N;
    hipLaunchKernelGGL(k_skinny_finalize, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, a.partial, plan.splits,
                       a.M, a.N, a.bias, a.Y, a.ldy);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace mmd8
