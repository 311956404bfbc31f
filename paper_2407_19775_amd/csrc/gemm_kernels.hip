// int8 MFMA GEMM with the fused mixed-decomposition epilogue ("Compression techniques", item 2).
//
//   acc[m,n] = sum_k Xq[m,k] Wt[n,k]                      v_mfma_i32_32x32x32_i8, exact
//   Y[m,n]   = f16( acc r[m] c[n] / 127^2                  outer-product dequantization
//                   + sum_j X[m,O_j] f16(Wt[n,O_j] c[n]/127)   v_mfma_f32_32x32x16_f16 on the critical columns
//                   + bias[n] )
//
// Both operands are K-contiguous int8 codes in the blocked layout of operand_layout.h, padded to
// whole tiles, so the main loop has no bounds checks.  A workgroup owns one BM x BN tile of Y.
// K is walked in slabs of 64 bytes.  A slab of both operands goes from global memory straight
// into LDS (global_load_lds_dwordx4: no register staging, every wave instruction copies 1 KB that
// is contiguous in HBM) through a ring of LDS buffers, two or three slabs ahead of the MFMAs.  The
// blocks are fragment-major already in HBM: the 64 lanes of an MFMA operand read 64 consecutive
// 16-byte pieces.  A lane's 16 bytes feed one operand row of the 32x32x32 MFMA; the k order
// inside the instruction is irrelevant as long as both operands use the same piece for the same
// lane group, which they do.
//
// One kernel, k_gemm_mixed, instantiated for several tile configurations (256 x 256 with eight waves for
// large problems, smaller tiles for small ones); fragments are double-buffered in registers.
#include <atomic>
#include <type_traits>

#include "codec_device.h"
#include "common.h"
#include "gemm.h"
#include "operand_layout.h"

namespace mmd8 {

// the code table of the blockwise encoder, for outputs that leave in coded form
__device__ const DynamicCode kExitCode = make_dynamic_code();

constexpr int BK = 64;                  // bytes of K per slab
constexpr int CPR = BK / 16;            // 16-byte chunks per LDS row
constexpr int ROWS_PER_DMA = kWave / CPR;

static_assert(BK == kSlabBytes, "one LDS slab is one slab of the packed operands");

// Address of the first byte that DMA instruction j of `wave` copies for slab 0 of an operand tile
// whose first row is row0 (a multiple of 16 inside one panel): 16 rows x 64 bytes, contiguous.
__device__ __forceinline__ const int8_t* dma_source(const int8_t* base, int row0, int n_slabs, int j, int waves, int wave,
                                           int lane) {
  return base + (size_t)(row0 >> 8) * n_slabs * kBlockBytes +
         (size_t)((row0 & 255) + (j * waves + wave) * ROWS_PER_DMA) * kSlabBytes + lane * 16;
}

template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, int STAGES_, int WAVES_PER_SIMD_>
struct GemmCfg {
  static constexpr int kWavesPerSimd = WAVES_PER_SIMD_;           // register budget: 512 / this
  static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int kWaves = WAVES_M * WAVES_N;
  static constexpr int kThreads = kWaves * kWave;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  static constexpr int TI = WM / 32, TJ = WN / 32;                 // MFMA tiles per wave
  static constexpr int NKS = BK / 32;                              // MFMA k-steps per slab
  static constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int kStages = STAGES_;
  static constexpr int RING_BYTES = STAGE_BYTES * kStages;
  static constexpr int R_BYTES = 1024;                             // 256 row scales, one DMA instruction
  static constexpr int LDS_BYTES = RING_BYTES + R_BYTES;
  static constexpr int A_DMA = BM / ROWS_PER_DMA / kWaves;         // DMA instructions per wave per slab
  static constexpr int B_DMA = BN / ROWS_PER_DMA / kWaves;
  static constexpr int DMA_PER_SLAB = A_DMA + B_DMA;
  static constexpr int kAhead = kStages - 1;                       // slabs requested ahead of the MFMAs
  static_assert(BM % (ROWS_PER_DMA * kWaves) == 0 && BN % (ROWS_PER_DMA * kWaves) == 0, "tile/wave mismatch");
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be whole MFMA tiles");
  static_assert(NKS == 2, "fragment buffering below is written for two k-steps per slab");
  static_assert(kStages >= 3 && kStages <= 4, "ring of three or four slabs");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS");
  static_assert(BM <= 256, "row scales are staged with one 1 KB request");
  // gather staging of critical columns beyond the slab: [rows][16 k] fp16 for both operands
  static_assert((BM + BN) * 32 <= RING_BYTES, "epilogue staging must fit in the slab buffers");
};

// own requests older than the newest kVm have landed, own LDS reads have returned; after the
// barrier that holds for every wave of the workgroup
template <int kVm>
__device__ inline void wait_slab_and_sync() {
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" : : "n"(kVm) : "memory");
}
__device__ inline void wait_lds_and_sync() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" : : : "memory"); }
__device__ inline void sync_only() { asm volatile("s_barrier" : : : "memory"); }

// Tile assignment.  Consecutive workgroup ids land on different XCDs (8 of them, each with its own L2), so XCD x
// gets the ids x, x + 8, ...: a contiguous run of the tile order below, 32 tiles (one per CU) at a time.  The order
// walks blocks of 8 tile rows x 4 tile columns (bands of 4 columns; inside a band blocks of 8 rows; inside a
// block rows fastest), so the 32 tiles an XCD works on at once share 8 activation panels and 4 weight panels:
// 12 panel streams through its L2 instead of the 18 of a plain rows-fastest order with 16 tile rows (measured on
// the 70B-shaped linears at 4096 tokens: 1.4-2.1 % faster; identical for up to 8 tile rows).
__device__ inline bool tile_of_block(const GemmArgs& a, int bid, int& tm, int& tn) {
  constexpr int kBlockRows = 8, kBandCols = 4;
  const int n_tiles = a.tiles_m * a.tiles_n;
  const int per_xcd = ceil_div(n_tiles, 8);
  const int logical = (bid % 8) * per_xcd + bid / 8;
  if (logical >= n_tiles) return false;
  const int band_tiles = a.tiles_m * kBandCols;                    // (every band but the last is full)
  const int band = logical / band_tiles;
  const int w = min(kBandCols, a.tiles_n - band * kBandCols);      // width of this band
  const int q = logical - band * band_tiles;                       // index inside the band
  const int full_blocks = a.tiles_m / kBlockRows, rest_rows = a.tiles_m - full_blocks * kBlockRows;
  if (q < full_blocks * kBlockRows * w) {
    const int r = q % (kBlockRows * w);
    tm = (q / (kBlockRows * w)) * kBlockRows + r % kBlockRows;
    tn = band * kBandCols + r / kBlockRows;
  } else {                                                         // the last, shorter block of rows
    const int r = q - full_blocks * kBlockRows * w;
    tm = full_blocks * kBlockRows + r % rest_rows;
    tn = band * kBandCols + r / rest_rows;
  }
  return true;
}

// ------------------------------------------------------------------------------------------------
// Epilogue pieces.  C layout of the 32x32 MFMA: a lane holds column (lane % 32); register e holds
// row 8 (e / 4) + 4 (lane / 32) + (e % 4).  The accumulators stay where the MFMAs left them: they
// are dequantized in place (the registers then hold fp32 bits), the fp16 MFMAs of the critical
// columns accumulate onto them in place, and each 32x32 tile is converted and stored on its own.
// ------------------------------------------------------------------------------------------------
template <class Cfg>
struct WavePos {
  int m0, n0, wm, wn, lane, lr, lg, mw, nw;
  __device__ WavePos(int m0_, int n0_, int wave, int lane_)
      : m0(m0_), n0(n0_), wm(wave / Cfg::WAVES_N), wn(wave % Cfg::WAVES_N), lane(lane_), lr(lane_ & 31),
        lg(lane_ >> 5), mw(m0_ + (wave / Cfg::WAVES_N) * Cfg::WM), nw(n0_ + (wave % Cfg::WAVES_N) * Cfg::WN) {}
};

template <class Cfg>
__device__ __forceinline__ void tap_accumulators(const GemmArgs& a, const WavePos<Cfg>& p, v16i (&acc)[Cfg::TI][Cfg::TJ]) {
#pragma unroll
  for (int i = 0; i < Cfg::TI; ++i)
#pragma unroll
    for (int j = 0; j < Cfg::TJ; ++j) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = p.mw + i * 32 + 8 * (e / 4) + 4 * p.lg + (e % 4), n = p.nw + j * 32 + p.lr;
        if (m < a.M && n < a.N) a.tap_acc[(size_t)m * a.tap_ld + n] = acc[i][j][e];
      }
      __builtin_amdgcn_sched_barrier(0);
    }
}

// acc := bits( acc * r[m] * (c[n] / 127^2) ).  r_tile points at the 256 (or fewer) row scales of
// this workgroup tile, in LDS or in global memory.
template <class Cfg, class RPtr>
__device__ __forceinline__ void dequantize_in_place(const WavePos<Cfg>& p, v16i (&acc)[Cfg::TI][Cfg::TJ], RPtr r_tile,
                                           const float (&cs)[Cfg::TJ]) {
#pragma unroll
  for (int i = 0; i < Cfg::TI; ++i) {
    float rm[16];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const v4f v = *reinterpret_cast<const v4f*>(r_tile + p.wm * Cfg::WM + i * 32 + 8 * q + 4 * p.lg);
      rm[4 * q] = v[0], rm[4 * q + 1] = v[1], rm[4 * q + 2] = v[2], rm[4 * q + 3] = v[3];
    }
#pragma unroll
    for (int j = 0; j < Cfg::TJ; ++j) {
      v16f y;
#pragma unroll
      for (int e = 0; e < 16; ++e) y[e] = (float)acc[i][j][e] * (rm[e] * cs[j]);
      acc[i][j] = __builtin_bit_cast(v16i, y);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// Critical columns j_begin .. n_out-1, 16 at a time: every thread helps to stage X[m, O_j] (fp16)
// and f16(Wt[n, O_j] c[n] / 127) for the whole tile in LDS as [row][16] fp16, then one 32x32x16
// fp16 MFMA per output tile.  General (any number of columns); the slab buffers must be free.
// A thread owns one of the 16 columns and every (kThreads / 16)-th row; all its gathers of a step are
// issued together (clamped addresses, results masked), so a step costs a few memory latencies, not one
// per element.
template <class Cfg>
__device__ __forceinline__ void gather_outlier_columns(const GemmArgs& a, const WavePos<Cfg>& p, v16i (&acc)[Cfg::TI][Cfg::TJ],
                                              int8_t* smem, int j_begin, int n_out) {
  constexpr int TI = Cfg::TI, TJ = Cfg::TJ, TILE_M = Cfg::BM, TILE_N = Cfg::BN;
  constexpr int RSTEP = Cfg::kThreads / 16;                        // rows between a thread's items
  constexpr int NX = TILE_M / RSTEP, NW = TILE_N / RSTEP;          // its rows of X, then of Wt
  static_assert(TILE_M % RSTEP == 0 && TILE_N % RSTEP == 0, "whole rows per thread");
  uint16_t* sXo = reinterpret_cast<uint16_t*>(smem);             // [TILE_M][16], then [TILE_N][16]
  uint16_t* sWo = sXo + TILE_M * 16;
  const int kk = threadIdx.x & 15, r0 = threadIdx.x >> 4;
  const int n_slabs = a.Kpad / BK;
  __syncthreads();                                               // every wave is done with the slab ring
  // (the column index of a step is asked for one step ahead, and a step's loads of X and of the weights go out
  // together: one memory latency per step instead of three)
  int k_next = j_begin + kk < n_out ? a.idx[j_begin + kk] : 0;
  for (int j0 = j_begin; j0 < n_out; j0 += 16) {
    const bool col_ok = j0 + kk < n_out;
    const int k = k_next;
    k_next = j0 + 16 + kk < n_out ? a.idx[j0 + 16 + kk] : 0;
    // eight rows at a time: enough loads in flight, few registers next to the accumulators
    constexpr int BX = NX < 8 ? NX : 8, BW = NW < 8 ? NW : 8;
    static_assert(NX % BX == 0 && NW % BW == 0, "whole batches");
    constexpr int kBatches = NX / BX > NW / BW ? NX / BX : NW / BW;
    const uint16_t* xcol = a.X + k;
    const int xld = a.ldx;
#pragma unroll 1
    for (int b = 0; b < kBatches; ++b) {
      const bool has_x = b < NX / BX, has_w = b < NW / BW;
      uint16_t xv[BX], wv[BW];
      int8_t wq[BW];
      float wc[BW];
      if (has_x) {
#pragma unroll
        for (int i = 0; i < BX; ++i) xv[i] = xcol[(size_t)min(p.m0 + r0 + (b * BX + i) * RSTEP, a.M - 1) * xld];
      }
      if (has_w) {
        if (a.W_master) {                                     // the original 16-bit rows, as they are
#pragma unroll
          for (int i = 0; i < BW; ++i)
            wv[i] = a.W_master[(size_t)k * a.ldw_master + min(p.n0 + r0 + (b * BW + i) * RSTEP, a.N - 1)];
        } else {
#pragma unroll
          for (int i = 0; i < BW; ++i) {
            const int n = min(p.n0 + r0 + (b * BW + i) * RSTEP, a.N - 1);
            wq[i] = a.Wt[packed_offset(n, k, n_slabs)];
            wc[i] = a.c[n];
          }
        }
      }
      if (has_x) {
#pragma unroll
        for (int i = 0; i < BX; ++i) {
          const int row = r0 + (b * BX + i) * RSTEP;
          sXo[row * 16 + kk] = (col_ok && p.m0 + row < a.M) ? xv[i] : (uint16_t)0;
        }
      }
      if (has_w) {
#pragma unroll
        for (int i = 0; i < BW; ++i) {
          const int row = r0 + (b * BW + i) * RSTEP;
          const uint16_t v = a.W_master ? wv[i] : (uint16_t)rounded_float_to_half_bits((float)wq[i] * (wc[i] / 127.0f));
          sWo[row * 16 + kk] = (col_ok && p.n0 + row < a.N) ? v : (uint16_t)0;
        }
      }
    }
    __syncthreads();
    v8h fxa[TI], fxb[TJ];
#pragma unroll
    for (int i = 0; i < TI; ++i)
      fxa[i] = *reinterpret_cast<const v8h*>(sXo + (p.wm * Cfg::WM + i * 32 + p.lr) * 16 + p.lg * 8);
#pragma unroll
    for (int j = 0; j < TJ; ++j)
      fxb[j] = *reinterpret_cast<const v8h*>(sWo + (p.wn * Cfg::WN + j * 32 + p.lr) * 16 + p.lg * 8);
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j)
        acc[i][j] = __builtin_bit_cast(
            v16i, __builtin_amdgcn_mfma_f32_32x32x16_f16(fxa[i], fxb[j], __builtin_bit_cast(v16f, acc[i][j]), 0, 0, 0));
    __syncthreads();
  }
}

// The 16-bit product over the critical feature dimensions ("Compression techniques", item 2) for an input where
// hundreds or thousands of them are critical (dense_critical_path: none of them travelled as an fp16 slab then):
// slab after slab of 64 columns.
//   A side: the tile's rows of X itself (fp16, 128 contiguous bytes per row and slab), columns that are not
//           critical set to zero, parked in LDS as rows of 144 bytes;
//   B side: the slab of weight codes, fetched like in the main loop, the codes turned into fp16 integers in
//           registers (codes_to_half8) as the decode kernels do.
// The accumulators hold Y so far in fp32; sum_k X[m,k] q[n,k] lacks the column's step c[n] / 127, so they are
// divided by it on entry and multiplied by it on exit (columns with c[n] = 0 have only zero codes: factor 1).
// Against the slabs prepared by the pack kernel the weights are not rounded to fp16 after scaling: at most 2^-11
// relative per term, as in the decode kernels.  Requests run several slabs ahead of the MFMAs (see kDepth).
template <class Cfg>
__device__ __forceinline__ void dense_critical_columns(const GemmArgs& a, const WavePos<Cfg>& p, v16i (&acc)[Cfg::TI][Cfg::TJ],
                                                       int8_t* smem, const float (&cs)[Cfg::TJ]) {
  constexpr int TI = Cfg::TI, TJ = Cfg::TJ;
  constexpr int TPR = Cfg::kThreads / Cfg::BM;                      // threads per row of the activation tile
  static_assert(Cfg::kThreads % Cfg::BM == 0 && TPR >= 1 && TPR <= 8, "whole threads per row");
  constexpr int CPT = BK / TPR, NL = CPT / 8;                        // columns per thread, 16-byte loads per thread
  constexpr int kRowBytes = 2 * BK + 16;                             // 144: rows 8 apart share banks, not rows next to each other
  constexpr int A_LDS = (Cfg::BM * kRowBytes + 1023) / 1024 * 1024;
  // Slabs in flight.  A slab's requests (this thread's pieces of the rows of X and the slab's mask byte into
  // registers, the weight codes into an LDS buffer) go out kDepth slabs ahead: a slab's MFMAs take a quarter of the
  // time its data takes to arrive.  One weight buffer more than that, so that a request never targets the buffer
  // being read.  Every slab position issues the same kPerSlab requests in the same order (positions past the end
  // ask for the last slab again), so the number still in flight behind a slab's weight codes is known; the loads
  // into registers are the compiler's to wait for, and it counts only those, so its waits come out stricter than
  // needed (about two slabs ahead instead of kDepth - 1), never looser.
  constexpr int kBuffers = (Cfg::RING_BYTES - A_LDS) / Cfg::B_BYTES < 5 ? (Cfg::RING_BYTES - A_LDS) / Cfg::B_BYTES : 5;
  constexpr int kDepth = kBuffers - 1;
  constexpr int kPerSlab = NL + 1 + Cfg::B_DMA;                      // requests per slab and lane
  static_assert(kDepth >= 1 && (kDepth - 1) * kPerSlab <= 63, "at least two weight buffers; the count fits the wait instruction");
  int8_t* sA = smem;
  int8_t* sB = smem + A_LDS;
  const int lane = p.lane, wm = p.wm, wn = p.wn;
  const int wave = wm * Cfg::WAVES_N + wn;
  const int n_slabs = a.Kpad / BK;
  const int row = threadIdx.x / TPR, part = threadIdx.x % TPR;
  const uint16_t* xrow = a.X + (size_t)min(p.m0 + row, a.M - 1) * a.ldx + part * CPT;

  float back[TJ];
#pragma unroll
  for (int j = 0; j < TJ; ++j) {
    const float step = cs[j] * 127.0f;                               // c[n] / 127
    back[j] = step != 0.0f ? step : 1.0f;
    const float inv = step != 0.0f ? 1.0f / step : 1.0f;
#pragma unroll
    for (int i = 0; i < TI; ++i) {
      v16f y = __builtin_bit_cast(v16f, acc[i][j]);
#pragma unroll
      for (int e = 0; e < 16; ++e) y[e] *= inv;
      acc[i][j] = __builtin_bit_cast(v16i, y);
    }
  }

  v4u ra[kDepth][NL];
  uint8_t fl[kDepth];
  const uint32_t ldsB = (uint32_t)(uintptr_t)sB + wave * (kWave * 16);
  // position `pos` of the sequence (slab pos, or the last slab again past the end) into register set u and weight
  // buffer pos % kBuffers (a repeated request lands in a buffer that is not read any more)
  auto request = [&](int pos, auto u_tag) __attribute__((always_inline)) {
    constexpr int u = decltype(u_tag)::value;
    const int s = min(pos, n_slabs - 1);
#pragma unroll
    for (int q = 0; q < NL; ++q) {
      // pieces beyond the row's end (the padding of K) re-read the row's first piece; none of their columns is critical
      const int col = s * BK + part * CPT + 8 * q;
      ra[u][q] = *reinterpret_cast<const v4u*>(xrow + (col < a.ldx ? col - part * CPT : -part * CPT));
    }
    fl[u] = a.mask[s * BK + lane];
    const uint32_t dst = ldsB + (pos % kBuffers) * Cfg::B_BYTES;
#pragma unroll
    for (int j = 0; j < Cfg::B_DMA; ++j)
      dma16(dma_source(a.Wt, p.n0, n_slabs, j, Cfg::kWaves, wave, lane) + (size_t)s * kBlockBytes,
            dst + j * Cfg::kWaves * (kWave * 16));
  };
  auto iteration = [&](int s, auto u_tag) __attribute__((always_inline)) {
    constexpr int u = decltype(u_tag)::value;                        // s % kDepth
    // the weight codes of slab s have landed once only the requests of the kDepth - 1 positions after it are out
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"((kDepth - 1) * kPerSlab) : "memory");
    // bit c: column 64 s + c is critical (positions past the end: nothing to multiply)
    const uint64_t bits = s < n_slabs ? __builtin_amdgcn_ballot_w64(fl[u] != 0) : 0;
    // park the rows of slab s, critical columns only
#pragma unroll
    for (int q = 0; q < NL; ++q) {
      const uint32_t b8 = (uint32_t)(bits >> (part * CPT + 8 * q)) & 0xffu;
      v4u v = ra[u][q];
#pragma unroll
      for (int w = 0; w < 4; ++w)
        v[w] &= (((b8 >> (2 * w)) & 1u) ? 0x0000ffffu : 0u) | (((b8 >> (2 * w + 1)) & 1u) ? 0xffff0000u : 0u);
      *reinterpret_cast<v4u*>(sA + row * kRowBytes + (part * CPT + 8 * q) * 2) = v;
    }
    wait_lds_and_sync();
    // (past the end the last slab is asked for again: the count of requests in flight stays what the waits assume)
    request(s + kDepth, u_tag);
    if (bits != 0) {
      const int8_t* fbase = sB + (s % kBuffers) * Cfg::B_BYTES + (wn * Cfg::WN / 32) * 2048 + lane * 16;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        v4u wu[TJ];
#pragma unroll
        for (int j = 0; j < TJ; ++j)
          wu[j] = *reinterpret_cast<const v4u*>(fbase + j * 32 * BK + ks * 1024) ^ 0x80808080u;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          v8h xa[TI];
#pragma unroll
          for (int i = 0; i < TI; ++i)
            xa[i] = *reinterpret_cast<const v8h*>(sA + (wm * Cfg::WM + i * 32 + (lane & 31)) * kRowBytes +
                                                  (32 * ks + 16 * (lane >> 5) + 8 * t) * 2);
#pragma unroll
          for (int j = 0; j < TJ; ++j) {
            const v8h wh = codes_to_half8(wu[j], t);
#pragma unroll
            for (int i = 0; i < TI; ++i)
              acc[i][j] = __builtin_bit_cast(
                  v16i, __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[i], wh, __builtin_bit_cast(v16f, acc[i][j]), 0, 0, 0));
          }
        }
      }
    }
    wait_lds_and_sync();                                             // the parked rows and this weight buffer are read before they are written again
  };

  wait_lds_and_sync();                                               // every wave is done with the slab ring
  [&]<int... U>(std::integer_sequence<int, U...>) __attribute__((always_inline)) {
    (request(U, std::integral_constant<int, U>{}), ...);
    // whole groups of kDepth positions, one code path and no way out inside a group
    for (int s = 0; s < n_slabs; s += kDepth) (iteration(s + U, std::integral_constant<int, U>{}), ...);
  }(std::make_integer_sequence<int, kDepth>{});
  // the requests repeated past the end are still on their way into registers and LDS
  asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
  wait_lds_and_sync();
#pragma unroll
  for (int j = 0; j < TJ; ++j)
#pragma unroll
    for (int i = 0; i < TI; ++i) {
      v16f y = __builtin_bit_cast(v16f, acc[i][j]);
#pragma unroll
      for (int e = 0; e < 16; ++e) y[e] *= back[j];
      acc[i][j] = __builtin_bit_cast(v16i, y);
    }
}

// bias, rounding to fp16, and stores, through LDS (the slab buffers are free by now).  Neighbouring lanes hold
// neighbouring columns of the same rows; an even/odd lane pair swaps halves so that each lane has two adjacent
// columns (4 bytes): the even lane of row e, the odd lane of row e + 1.  A wave parks 64 (or 32) rows of its
// sub-tile at a time as fp16 rows in a region of its own and writes them out 16 bytes per lane, eight lanes
// per 128-byte row segment: a store instruction covers whole lines.  (Storing the 4-byte pairs directly
// takes four times as many store instructions and writes half lines that do not always meet in L2 before
// write-back: 2-5 % slower on the 256 x 256 tiles, 1.3 times the output in HBM write traffic.)
template <class Cfg, bool kFull>
__device__ __forceinline__ void store_tile(const GemmArgs& a, const WavePos<Cfg>& p, v16i (&acc)[Cfg::TI][Cfg::TJ],
                                      const float (&bn)[Cfg::TJ], int8_t* smem, int wave) {
  constexpr int TI = Cfg::TI, TJ = Cfg::TJ;
  constexpr int STRIDE = Cfg::WN * 2 + 16;                          // bytes per parked row (16 more: bank spread, 16-byte aligned)
  constexpr int IP = (TI >= 2 && Cfg::kWaves * 64 * STRIDE <= Cfg::RING_BYTES) ? 2 : 1;   // 32-row tiles per pass
  constexpr int RP = 32 * IP;                                       // rows per pass
  constexpr int CH = Cfg::WN / 8;                                   // 16-byte chunks per row
  static_assert(Cfg::kWaves * RP * STRIDE <= Cfg::RING_BYTES, "output staging must fit in the slab buffers");
  static_assert((RP * CH) % kWave == 0, "whole store instructions");
  int8_t* base = smem + wave * (RP * STRIDE);
  const int odd = p.lane & 1;
  __syncthreads();                                                  // every wave is done with the slab buffers
#pragma unroll
  for (int i0 = 0; i0 < TI; i0 += IP) {
#pragma unroll
    for (int ii = 0; ii < IP; ++ii) {
#pragma unroll
      for (int j = 0; j < TJ; ++j) {
        const v16f y = __builtin_bit_cast(v16f, acc[i0 + ii][j]);
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
          const uint32_t h = float_to_half_bits(y[e] + bn[j]) | (float_to_half_bits(y[e + 1] + bn[j]) << 16);
          const uint32_t q = (uint32_t)__builtin_amdgcn_mov_dpp((int)h, 0xb1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]
          const uint32_t out = odd ? ((q >> 16) | (h & 0xffff0000u)) : ((h & 0xffffu) | (q << 16));
          const int row = ii * 32 + 8 * (e / 4) + (e % 4) + 4 * p.lg + odd;
          *reinterpret_cast<uint32_t*>(base + row * STRIDE + (j * 32 + (p.lr & ~1)) * 2) = out;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int it = 0; it < RP * CH / kWave; ++it) {
      const int idx = it * kWave + p.lane, row = idx / CH, ch = idx % CH;
      const v4u v = *reinterpret_cast<const v4u*>(base + row * STRIDE + ch * 16);
      const int gm = p.mw + i0 * 32 + row, gn = p.nw + ch * 8;
      bool ok = true;
      if constexpr (!kFull) ok = gm < a.M && gn < a.N;
      if (ok) *reinterpret_cast<v4u*>(a.Y + (size_t)gm * a.ldy + gn) = v;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
}

// The same with more behind the layer: an activation (GELU, applied to the rounded output before it is parked), a
// residual, and / or an output that leaves in coded form ("Compression techniques", item 1 applied to the result
// of item 2): H = f16(Y + residual) (or Y), written where wanted, and its blockwise 8-bit codes.  Rows are parked
// as in store_tile.  Phase A (each wave on its own rows): add the residual in place, store H.  After a barrier,
// phase B: a lane takes 16 neighbouring columns of one row of the workgroup tile, whichever wave parked them,
// so that the lanes of a block are neighbours (4, 8 or 16 of them: the block maximum is a few DPP steps) and a
// wave instruction writes whole 256-byte (128-byte) rows of codes.
template <class Cfg, bool kFull>
__device__ __forceinline__ void store_tile_coded(const GemmArgs& a, const WavePos<Cfg>& p, v16i (&acc)[Cfg::TI][Cfg::TJ],
                                        const float (&bn)[Cfg::TJ], int8_t* smem, int wave) {
  constexpr int TI = Cfg::TI, TJ = Cfg::TJ;
  constexpr int STRIDE = Cfg::WN * 2 + 16;
  constexpr int CELL_BYTES = DynamicCode::kCells * 8;
  constexpr int IP = (TI >= 2 && Cfg::kWaves * 64 * STRIDE + CELL_BYTES <= Cfg::RING_BYTES) ? 2 : 1;
  constexpr int RP = 32 * IP;
  constexpr int CH = Cfg::WN / 8;
  constexpr int PARK_BYTES = Cfg::kWaves * RP * STRIDE;
  static_assert(PARK_BYTES + CELL_BYTES <= Cfg::RING_BYTES, "output staging and the code table must fit in the slab buffers");
  static_assert((RP * CH) % kWave == 0, "whole store instructions");
  constexpr int LPR = Cfg::BN / 16;                                  // lanes per row of the workgroup tile in phase B
  constexpr int TASKS = Cfg::WAVES_M * RP * LPR;
  static_assert(TASKS % Cfg::kThreads == 0 && (LPR == 8 || LPR == 16), "phase B covers the parked rows in whole rounds");
  int8_t* base = smem + wave * (RP * STRIDE);
  v2u* s_cells = reinterpret_cast<v2u*>(smem + PARK_BYTES);
  const int odd = p.lane & 1;
  const int lb = a.code_log_block;
  __syncthreads();                                                  // every wave is done with the slab buffers
  if (a.codes) stage_code_cells(s_cells, kExitCode, threadIdx.x, Cfg::kThreads);
  const uint32_t cells_biased = biased_cell_base(s_cells);
#pragma unroll
  for (int i0 = 0; i0 < TI; i0 += IP) {
#pragma unroll
    for (int ii = 0; ii < IP; ++ii) {
#pragma unroll
      for (int j = 0; j < TJ; ++j) {
        const v16f y = __builtin_bit_cast(v16f, acc[i0 + ii][j]);
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
          uint32_t h = float_to_half_bits(y[e] + bn[j]) | (float_to_half_bits(y[e + 1] + bn[j]) << 16);
          if (a.gelu) h = gelu_half_pair(h);                         // the activation, on the rounded layer output
          const uint32_t q = (uint32_t)__builtin_amdgcn_mov_dpp((int)h, 0xb1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]
          const uint32_t out = odd ? ((q >> 16) | (h & 0xffff0000u)) : ((h & 0xffffu) | (q << 16));
          const int row = ii * 32 + 8 * (e / 4) + (e % 4) + 4 * p.lg + odd;
          *reinterpret_cast<uint32_t*>(base + row * STRIDE + (j * 32 + (p.lr & ~1)) * 2) = out;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    // ---- phase A
    if (a.residual || a.Y) {
#pragma unroll
      for (int it = 0; it < RP * CH / kWave; ++it) {
        const int idx = it * kWave + p.lane, row = idx / CH, ch = idx % CH;
        int8_t* cell = base + row * STRIDE + ch * 16;
        v4u v = *reinterpret_cast<const v4u*>(cell);
        const int gm = p.mw + i0 * 32 + row, gn = p.nw + ch * 8;
        bool ok = true;
        if constexpr (!kFull) ok = gm < a.M && gn < a.N;
        if (a.residual) {
          v4u res = v4u{0, 0, 0, 0};
          if (ok) res = *reinterpret_cast<const v4u*>(a.residual + (size_t)gm * a.ldr + gn);
#pragma unroll
          for (int w = 0; w < 4; ++w)
            v[w] = float_to_half_bits(half_lo_to_float(v[w]) + half_lo_to_float(res[w])) |
                   (float_to_half_bits(half_hi_to_float(v[w]) + half_hi_to_float(res[w])) << 16);
          *reinterpret_cast<v4u*>(cell) = v;
        }
        if (a.Y && ok) *reinterpret_cast<v4u*>(a.Y + (size_t)gm * a.ldy + gn) = v;
      }
    }
    __syncthreads();                                                // the parked rows of every wave are final
    // ---- phase B
    if (a.codes) {
#pragma unroll
      for (int q = 0; q < TASKS / Cfg::kThreads; ++q) {
        const int t = q * Cfg::kThreads + threadIdx.x;
        const int col = (t % LPR) * 16, rowp = t / LPR, wm2 = rowp / RP, row = rowp % RP;
        const int8_t* src = smem + (wm2 * Cfg::WAVES_N + col / Cfg::WN) * (RP * STRIDE) + row * STRIDE + (col % Cfg::WN) * 2;
        const v4u h0 = *reinterpret_cast<const v4u*>(src), h1 = *reinterpret_cast<const v4u*>(src + 16);
        uint32_t m = max(chunk_absmax_pattern(h0), chunk_absmax_pattern(h1));
        m = dpp_max<0xB1>(m);                                       // 2 lanes
        m = dpp_max<0x4E>(m);                                       // 4 lanes: 64 elements
        if (lb >= 7) m = dpp_max<0x141>(m);                         // 8 lanes
        if (lb >= 8) m = dpp_max<0x140>(m);                         // 16 lanes
        const int gm = p.m0 + wm2 * Cfg::WM + i0 * 32 + row, gn = p.n0 + col;
        bool ok = true;
        if constexpr (!kFull) ok = gm < a.M && gn < a.N;
        const float am = half_lo_to_float(m);
        const float inv = (am == 0.0f) ? 0.0f : 1.0f / am;          // IEEE division
        if (ok) {
          const size_t e = (size_t)gm * a.code_ld + gn;
          if ((gn & ((1 << lb) - 1)) == 0) a.code_absmax[e >> lb] = am;
          const v2u c0 = encode_chunk(h0, inv, cells_biased), c1 = encode_chunk(h1, inv, cells_biased);
          *reinterpret_cast<v4u*>(a.codes + e) = v4u{c0[0], c0[1], c1[0], c1[1]};
        }
      }
    }
    __syncthreads();                                                // the next pass parks over these rows
  }
}

template <class Cfg>
__device__ __forceinline__ void load_column_terms(const GemmArgs& a, const WavePos<Cfg>& p, float (&cs)[Cfg::TJ],
                                         float (&bn)[Cfg::TJ]) {
#pragma unroll
  for (int j = 0; j < Cfg::TJ; ++j) {
    const int n = min(p.nw + j * 32 + p.lr, a.N - 1);
    cs[j] = a.c[n] / 16129.0f;
    bn[j] = a.bias ? half_lo_to_float(a.bias[n]) : 0.0f;
  }
}

// ------------------------------------------------------------------------------------------------
// Generic kernel: 4 waves, one wave per SIMD or two workgroups per CU, small tiles.
// kFull: M and N are multiples of the tile, so no output store needs a bounds check.
// kTap: also write the raw int32 accumulators (parity checks).
// kCoded: the output goes through an activation, takes a residual and / or leaves in blockwise-coded form
// (store_tile_coded).
// ------------------------------------------------------------------------------------------------
// kDense: the critical columns are handled by dense_critical_columns after the loop instead of through fp16 slabs
// and the gather (the kernel decides; the two cases are compiled apart, see k_gemm_mixed).
template <class Cfg, bool kTap, bool kFull, bool kCoded, bool kDense>
__device__ __forceinline__ void gemm_tile(const GemmArgs& a) {
  extern __shared__ __attribute__((aligned(1024))) int8_t smem[];
  constexpr int TI = Cfg::TI, TJ = Cfg::TJ, NKS = Cfg::NKS, STAGES = Cfg::kStages;

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  reset_column_flags(a.flag_reset, a.Kpad);
  int tm, tn;
  if (!tile_of_block(a, blockIdx.x, tm, tn)) return;
  const WavePos<Cfg> p(tm * Cfg::BM, tn * Cfg::BN, wave, lane);
  const int n_slabs = a.Kpad / BK;
  const int n_out = __builtin_amdgcn_readfirstlane(*a.n_out);
  // Behind the slabs of codes, through the same ring: the fp16 slabs of the critical columns that are in use (32
  // columns each: at most crit_slabs of them in Xo / Wo, then at most g_slabs further ones in Xg / Wg; columns
  // beyond those are gathered after the loop) and those of a low-rank adapter (T on the activation side, B on the
  // weight side), which start at slab crit_slabs of Xo / Wo.
  const int crit_all = kDense ? 0 : ceil_div(n_out, kOutlierSlab);
  const int crit_used = min(a.crit_slabs, crit_all);
  const int more_used = a.Xg ? min(a.g_slabs, crit_all - crit_used) : 0;
  const int total_slabs = n_slabs + crit_used + more_used + (a.f_slabs - a.crit_slabs);
  // from this tile's slabs in Xo / Wo to its further slabs in Xg / Wg: the same place in a panel, other panel sizes
  // (two allocations: the distance as a difference of addresses, not of pointers)
  const ptrdiff_t to_more_x = (ptrdiff_t)(reinterpret_cast<uintptr_t>(a.Xg) - reinterpret_cast<uintptr_t>(a.Xo)) +
                              (ptrdiff_t)(p.m0 >> 8) * (a.g_slabs - a.f_slabs) * kBlockBytes;
  const ptrdiff_t to_more_w = (ptrdiff_t)(reinterpret_cast<uintptr_t>(a.Wg) - reinterpret_cast<uintptr_t>(a.Wo)) +
                              (ptrdiff_t)(p.n0 >> 8) * (a.g_slabs - a.f_slabs) * kBlockBytes;

  // ---- DMA plan of this lane: instruction j of this wave fills LDS rows
  // [(j kWaves + wave) ROWS_PER_DMA, +ROWS_PER_DMA) of the operand tile: 1 KB, contiguous in
  // HBM and in LDS.
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
  const int8_t* srcA[Cfg::A_DMA];
  const int8_t* srcB[Cfg::B_DMA];
  const int8_t* srcXo[Cfg::A_DMA];
  const int8_t* srcWo[Cfg::B_DMA];
#pragma unroll
  for (int j = 0; j < Cfg::A_DMA; ++j) {
    srcA[j] = dma_source(a.Xq, p.m0, n_slabs, j, Cfg::kWaves, wave, lane);
    srcXo[j] = dma_source(reinterpret_cast<const int8_t*>(a.Xo), p.m0, a.f_slabs, j, Cfg::kWaves, wave, lane);
  }
#pragma unroll
  for (int j = 0; j < Cfg::B_DMA; ++j) {
    srcB[j] = dma_source(a.Wt, p.n0, n_slabs, j, Cfg::kWaves, wave, lane);
    srcWo[j] = dma_source(reinterpret_cast<const int8_t*>(a.Wo), p.n0, a.f_slabs, j, Cfg::kWaves, wave, lane);
  }
  // request d (0 .. DMA_PER_SLAB-1) of the slab at position `pos` of the ring's sequence: the A rows first, then the
  // B rows.  kFp16 says which kind of slab that position holds (known where the request is written down, so that
  // the loop over the codes carries no choice between the two)
  auto issue_dma = [&](int pos, int stage, int d, auto fp16_tag) {
    constexpr bool kF = decltype(fp16_tag)::value;
    const uint32_t base = lds0 + stage * Cfg::STAGE_BYTES + wave * (kWave * 16);
    const int f = pos - n_slabs;                                    // among the fp16 slabs in use
    // its place: slab f of Xo / Wo, slab f - crit_used of Xg / Wg, or an adapter's slab behind the crit_slabs of Xo / Wo
    ptrdiff_t off = (ptrdiff_t)(!kF ? pos : f < crit_used ? f : f - crit_used - more_used + a.crit_slabs) * kBlockBytes;
    if (kF && f >= crit_used && f < crit_used + more_used)
      off = (d < Cfg::A_DMA ? to_more_x : to_more_w) + (ptrdiff_t)(f - crit_used) * kBlockBytes;
    if (d < Cfg::A_DMA)
      dma16((kF ? srcXo[d] : srcA[d]) + off, base + d * Cfg::kWaves * (kWave * 16));
    else
      dma16((kF ? srcWo[d - Cfg::A_DMA] : srcB[d - Cfg::A_DMA]) + off,
            base + Cfg::A_BYTES + (d - Cfg::A_DMA) * Cfg::kWaves * (kWave * 16));
  };
  auto issue_slab = [&](int pos, int stage) {
#pragma unroll
    for (int d = 0; d < Cfg::DMA_PER_SLAB; ++d) {
      if (pos < n_slabs)
        issue_dma(pos, stage, d, std::false_type{});
      else
        issue_dma(pos, stage, d, std::true_type{});
    }
  };

  // ---- per-lane LDS read offsets: row (lane % 32) of an MFMA tile, piece (2 ks + lane / 32)
  int a_off[NKS], b_off[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    // group of 32 rows: 2 KB = [k-step][lane] 16-byte pieces
    a_off[ks] = (p.wm * Cfg::WM / 32) * 2048 + ks * 1024 + p.lane * 16;
    b_off[ks] = Cfg::A_BYTES + (p.wn * Cfg::WN / 32) * 2048 + ks * 1024 + p.lane * 16;
  }
  v4i fa[2][TI], fb[2][TJ];
  auto read_frags = [&](int stage, int ks, int buf) {
    const int8_t* base = smem + stage * Cfg::STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < TI; ++i) fa[buf][i] = *reinterpret_cast<const v4i*>(base + a_off[ks] + i * 32 * BK);
#pragma unroll
    for (int j = 0; j < TJ; ++j) fb[buf][j] = *reinterpret_cast<const v4i*>(base + b_off[ks] + j * 32 * BK);
  };

  v16i acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

  // ---- software pipeline over the slab ring.  In iteration s slab s is being multiplied and
  // slab s + kAhead is requested into the buffer that held slab s - 1 (every wave finished
  // reading it before the barrier that ended iteration s - 1).  At the end of iteration s the
  // wave waits until only the requests younger than slab s + 1 are outstanding.
  // A wave issues in order, and a request that finds the memory queue full blocks the MFMAs
  // behind it, so the requests of a slab are spread evenly between the MFMAs of the iteration.
  // issue_tag: slab s + kAhead exists and is requested in this iteration (1: it is a slab of codes, 2: an fp16 slab;
  // 0: no request); kNext: slab s + 1 exists.
  constexpr int AHEAD = Cfg::kAhead;
  constexpr int MFMAS = TI * TJ;                                   // per k-step
  // request d of a slab goes out after MFMA number d SLOTS / DMA_PER_SLAB of the iteration
  constexpr int SLOTS = NKS * MFMAS, DPS_ = Cfg::DMA_PER_SLAB;
  static_assert(DPS_ >= 1 && DPS_ <= SLOTS, "request spreading");
  // requests of the iteration that are out before the wait in the last k-step (slot (NKS-1) MFMAS)
  constexpr int kBeforeWait = ((NKS - 1) * MFMAS * DPS_ + SLOTS - 1) / SLOTS;
  float cs[TJ], bn[TJ];
  load_column_terms<Cfg>(a, p, cs, bn);
  int stage = 0;
  // kFp16: slab s is one of the fp16 slabs (fp16 operands, fp32 accumulation onto the accumulators, which
  // were dequantized before the first of them)
  auto iteration = [&](int s, auto issue_tag, auto next_tag, auto fp16_tag) {
    constexpr int kIssueKind = decltype(issue_tag)::value;
    constexpr bool kIssue = kIssueKind != 0, kNext = decltype(next_tag)::value;
    constexpr bool kFp16 = decltype(fp16_tag)::value;
    const int stage1 = (stage + 1 == STAGES) ? 0 : stage + 1;
    const int stage_req = (stage == 0) ? STAGES - 1 : stage - 1;   // (s + kAhead) mod kStages
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      const int cur = ks & 1, nxt = cur ^ 1;
#pragma unroll
      for (int t = 0; t < MFMAS; ++t) {
        const int i = t / TJ, j = t % TJ;
        if constexpr (kFp16)
          acc[i][j] = __builtin_bit_cast(
              v16i, __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, fa[cur][i]),
                                                           __builtin_bit_cast(v8h, fb[cur][j]),
                                                           __builtin_bit_cast(v16f, acc[i][j]), 0, 0, 0));
        else
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
        if (t == 0) {
          // the first MFMA of the k-step goes out before any new LDS read, so the wait for its
          // fragments (read during the previous k-step) is already satisfied
          __builtin_amdgcn_sched_barrier(0);
          if (ks + 1 < NKS) {
            read_frags(stage, ks + 1, nxt);
          } else {
            // last k-step of the slab: make slab s+1 visible, then prefetch its first fragments.
            // Still allowed in flight: slabs s+2 .. s+kAhead-1 in full and the part of slab
            // s+kAhead requested during the earlier k-steps of this iteration
            wait_slab_and_sync<kIssue ? (AHEAD - 2) * Cfg::DMA_PER_SLAB + kBeforeWait : 0>();
            if (kNext) read_frags(stage1, 0, nxt);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        // request d with ceil(d SLOTS / DPS) == slot, if there is one (at most one: DPS <= SLOTS)
        {
          const int slot = ks * MFMAS + t;
          const int d = slot * DPS_ / SLOTS;                             // the only candidate: d SLOTS / DPS in (slot - 1, slot]
          const bool here = d < DPS_ && (d * SLOTS + DPS_ - 1) / DPS_ == slot;
          if (kIssue && here) {
            __builtin_amdgcn_sched_barrier(0);
            issue_dma(s + AHEAD, stage_req, d, std::bool_constant<kIssueKind == 2>{});
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    stage = stage1;
  };
  using yes = std::true_type;
  using no = std::false_type;

  int issued = 0;
  for (; issued < AHEAD && issued < total_slabs; ++issued) issue_slab(issued, issued);
  if (issued == 1)
    wait_slab_and_sync<0>();
  else if (issued == 2)
    wait_slab_and_sync<Cfg::DMA_PER_SLAB>();
  else
    wait_slab_and_sync<2 * Cfg::DMA_PER_SLAB>();
  read_frags(0, 0, 0);
  int s = 0;
  using none = std::integral_constant<int, 0>;
  using codes = std::integral_constant<int, 1>;
  using halves = std::integral_constant<int, 2>;
  for (; s + AHEAD < n_slabs; ++s) iteration(s, codes{}, yes{}, no{});                      // nearly all of the time
  for (; s < n_slabs && s + AHEAD < total_slabs; ++s) iteration(s, halves{}, yes{}, no{});  // the first fp16 slabs requested
  for (; s < n_slabs && s + 1 < total_slabs; ++s) iteration(s, none{}, yes{}, no{});
  if (s < n_slabs) iteration(s++, none{}, no{}, no{});              // the last slab when nothing follows it
  if constexpr (kTap) tap_accumulators<Cfg>(a, p, acc);
  dequantize_in_place<Cfg>(p, acc, a.r + p.m0, cs);
  for (; s + AHEAD < total_slabs; ++s) iteration(s, halves{}, yes{}, yes{});
  for (; s + 1 < total_slabs; ++s) iteration(s, none{}, yes{}, yes{});
  if (s < total_slabs) iteration(s, none{}, no{}, yes{});
  // every wave passed the last barrier after its last LDS read of the ring: the slab buffers are
  // free for the gather staging, which starts with a barrier of its own before writing them
  if constexpr (kDense)
    dense_critical_columns<Cfg>(a, p, acc, smem, cs);
  else if (n_out > kOutlierSlab * (crit_used + more_used))
    gather_outlier_columns<Cfg>(a, p, acc, smem, kOutlierSlab * (crit_used + more_used), n_out);
  if constexpr (kCoded)
    store_tile_coded<Cfg, kFull>(a, p, acc, bn, smem, wave);
  else
    store_tile<Cfg, kFull>(a, p, acc, bn, smem, wave);
}

// The tile routine for input with very many critical columns, as a function of its own: the kernels sit at the edge
// of their register budget, and with this rarely taken path compiled into the same body every one of them spilled
// registers (up to 320; the gather of single columns next to it ran twice as long).  Its only argument is the
// address of the kernel's own arguments where the launch put them (a function does not receive that address by
// itself, and arguments arrive in vector registers: made uniform again here, so that the arguments are read into
// scalar registers as in the kernel).
template <class Cfg, bool kTap, bool kFull, bool kCoded>
__device__ __noinline__ void gemm_tile_dense(uint32_t args_lo, uint32_t args_hi) {
  using constant_bytes = const __attribute__((address_space(4))) char*;
  const uint64_t address = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)args_lo) |
                           (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)args_hi) << 32;
  const GemmArgs a = *(const GemmArgs*)(constant_bytes)address;
  gemm_tile<Cfg, kTap, kFull, kCoded, true>(a);
}

template <class Cfg, bool kTap, bool kFull, bool kCoded>
__global__ __launch_bounds__(Cfg::kThreads, Cfg::kWavesPerSimd) void k_gemm_mixed(const GemmArgs a) {
  const int n_out = __builtin_amdgcn_readfirstlane(*a.n_out);
  if (dense_critical_path(n_out, a.crit_slabs, a.dense_from, a.W_master != nullptr)) {
    const uint64_t address = (uint64_t)(const char*)__builtin_amdgcn_kernarg_segment_ptr();   // `a` is the first argument
    gemm_tile_dense<Cfg, kTap, kFull, kCoded>((uint32_t)address, (uint32_t)(address >> 32));
    return;
  }
  gemm_tile<Cfg, kTap, kFull, kCoded, false>(a);
}

// ------------------------------------------------------------------------------------------------
// The kernels need more LDS than a kernel gets by default; the attribute is set once per instantiation and device,
// by prepare_gemm_kernels() (called when a workspace is set up) or else by the first launch.
template <class Cfg, bool kTap, bool kFull, bool kCoded>
static hipError_t ensure_lds_attribute() {
  // per device: the attribute belongs to the device's code object.  Two threads may both find it unset and set
  // it twice, which is harmless.
  static std::atomic<bool> attr_set[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (attr_set[dev]) return hipSuccess;
  const void* fn = reinterpret_cast<const void*>(&k_gemm_mixed<Cfg, kTap, kFull, kCoded>);
  const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
  if (e == hipSuccess) attr_set[dev] = true;
  return e;
}

template <class Cfg, bool kTap, bool kFull, bool kCoded>
static hipError_t launch_one(const GemmArgs& a, hipStream_t stream) {
  if (hipError_t e = ensure_lds_attribute<Cfg, kTap, kFull, kCoded>(); e != hipSuccess) return e;
  const int grid = ceil_div(a.tiles_m * a.tiles_n, 8) * 8;
  hipLaunchKernelGGL((k_gemm_mixed<Cfg, kTap, kFull, kCoded>), dim3(grid), dim3(Cfg::kThreads), Cfg::LDS_BYTES, stream, a);
  return hipGetLastError();
}

template <class Cfg>
static hipError_t launch_cfg(GemmArgs a, hipStream_t stream) {
  a.tiles_m = ceil_div(a.M, Cfg::BM);
  a.tiles_n = ceil_div(a.N, Cfg::BN);
  const bool full = (a.M % Cfg::BM == 0) && (a.N % Cfg::BN == 0);
  if (a.codes || a.residual || a.gelu) {
    if (a.codes && Cfg::BN % (1 << a.code_log_block) != 0) return hipErrorInvalidValue;   // a block would leave the tile
    if (a.tap_acc) return launch_one<Cfg, true, false, true>(a, stream);
    return full ? launch_one<Cfg, false, true, true>(a, stream)
                : launch_one<Cfg, false, false, true>(a, stream);
  }
  if (a.tap_acc) return launch_one<Cfg, true, false, false>(a, stream);
  return full ? launch_one<Cfg, false, true, false>(a, stream)
              : launch_one<Cfg, false, false, false>(a, stream);
}

// every instantiation launch_cfg can reach
// The tile configurations, by the number a caller can force one with (gemm.h):
using Cfg0 = GemmCfg<128, 128, 2, 2, 3, 3>;   // 49 KB of LDS: three workgroups per CU
using Cfg1 = GemmCfg<256, 128, 2, 2, 3, 2>;
using Cfg2 = GemmCfg<128, 256, 2, 2, 3, 2>;
using Cfg3 = GemmCfg<256, 256, 2, 4, 3, 2>;
using Cfg4 = GemmCfg<256, 256, 2, 4, 4, 2>;   // the large tile: whole rounds of one tile per CU
using Cfg5 = GemmCfg<128, 256, 2, 4, 4, 2>;   // remainders and less than one round of large tiles
template <class Cfg>
static hipError_t prepare_cfg() {
  hipError_t e = ensure_lds_attribute<Cfg, true, false, false>();
  if (e == hipSuccess) e = ensure_lds_attribute<Cfg, false, true, false>();
  if (e == hipSuccess) e = ensure_lds_attribute<Cfg, false, false, false>();
  if (e == hipSuccess) e = ensure_lds_attribute<Cfg, true, false, true>();
  if (e == hipSuccess) e = ensure_lds_attribute<Cfg, false, true, true>();
  if (e == hipSuccess) e = ensure_lds_attribute<Cfg, false, false, true>();
  return e;
}
hipError_t prepare_gemm_kernels() {
  hipError_t e = prepare_cfg<Cfg0>();
  if (e == hipSuccess) e = prepare_cfg<Cfg1>();
  if (e == hipSuccess) e = prepare_cfg<Cfg2>();
  if (e == hipSuccess) e = prepare_cfg<Cfg3>();
  if (e == hipSuccess) e = prepare_cfg<Cfg4>();
  if (e == hipSuccess) e = prepare_cfg<Cfg5>();
  return e;
}

static hipError_t launch_variant(const GemmArgs& a, int variant, hipStream_t stream) {
  // coded output with blocks wider than the 128-column tiles: the 256-column tile of the same height class
  if (a.codes && a.code_log_block > 7 && (variant == 0 || variant == 1)) variant = 2;
  switch (variant) {
    case 1: return launch_cfg<Cfg1>(a, stream);
    case 2: return launch_cfg<Cfg2>(a, stream);
    case 3: return launch_cfg<Cfg3>(a, stream);
    case 4: return launch_cfg<Cfg4>(a, stream);
    case 5: return launch_cfg<Cfg5>(a, stream);
    default: return launch_cfg<Cfg0>(a, stream);
  }
}

// the same problem restricted to output columns [n0, n0 + n): n0 a multiple of 256
static GemmArgs column_range(const GemmArgs& a, int n0, int n) {
  GemmArgs b = a;
  const size_t panels = (size_t)n0 / kPanelRows;
  b.Wt = a.Wt + panels * (size_t)(a.Kpad / BK) * kBlockBytes;
  b.Wo = a.Wo + panels * a.f_slabs * (kBlockBytes / 2);            // uint16_t elements
  b.Wg = a.Wg ? a.Wg + panels * a.g_slabs * (kBlockBytes / 2) : nullptr;
  b.c = a.c + n0;
  b.bias = a.bias ? a.bias + n0 : nullptr;
  b.Y = a.Y ? a.Y + n0 : nullptr;
  b.residual = a.residual ? a.residual + n0 : nullptr;
  b.codes = a.codes ? a.codes + n0 : nullptr;
  b.code_absmax = a.codes ? a.code_absmax + (n0 >> a.code_log_block) : nullptr;   // n0 is a multiple of 256
  b.tap_acc = a.tap_acc ? a.tap_acc + n0 : nullptr;
  b.W_master = a.W_master ? a.W_master + n0 : nullptr;
  b.N = n;
  return b;
}

hipError_t launch_gemm_mixed(const GemmArgs& a, int variant, hipStream_t stream) {
  if (variant >= 0 && variant <= 5) return launch_variant(a, variant, stream);
  // Automatic.  The 256 x 256 tile with the four-slab ring is the most efficient per CU, but it runs
  // in rounds of one tile per CU.  Whole rounds go to it; a remainder that would leave a good part of
  // the chip idle is launched separately with 128 x 256 tiles (same ring depth, twice as many
  // workgroups).  With weights coming cold from HBM (every layer has its own) the deep prefetch
  // matters more than the better balance of small tiles, so small tiles are for small problems only.
  const int tiles_m = ceil_div(a.M, 256), tiles_n = ceil_div(a.N, 256);
  const long tiles_256 = (long)tiles_m * tiles_n;
  const long tiles_128x256 = (long)ceil_div(a.M, 128) * tiles_n;
  const long cus = device_cu_count();
  if (a.M > 128 && tiles_256 >= cus) {
    const long rest = tiles_256 % cus;
    const int n_tiles_main = (int)((tiles_256 - rest) / tiles_m);      // whole columns of tiles in the whole rounds
    const int n_tiles_rest = tiles_n - n_tiles_main;
    if (rest > 0 && 2 * rest <= cus && n_tiles_main > 0 && n_tiles_rest > 0) {
      hipError_t e = launch_variant(column_range(a, 0, n_tiles_main * 256), 4, stream);
      if (e != hipSuccess) return e;
      return launch_variant(column_range(a, n_tiles_main * 256, a.N - n_tiles_main * 256), 5, stream);
    }
    return launch_variant(a, 4, stream);
  }
  // Less than one round of large tiles: 128 x 256 with eight waves and the four-slab ring, unless that leaves most
  // of the chip without a workgroup and K is short, where 128 x 128 tiles (up to three per CU) do better.  Measured
  // on the 7B linears at 160-1024 rows: 4096 -> 12288 at 256 rows 39 us against 47 with the four-wave 128 x 256
  // tile chosen before, 11008 -> 4096 (32 workgroups, 172 slabs) 73 against 79 with 128 x 128; 4096 -> 4096 stays
  // with 128 x 128 (33 against 35).
  // (where the 128 x 256 tiles would need a second round and the 256 x 256 ones fit in one, the large tiles win:
  // 4096 -> 12288 at 768 rows 61 against 71 us, 4096 -> 22016 at 512 rows 61 against 70)
  if (a.M > 128 && tiles_128x256 > cus) return launch_variant(a, 4, stream);
  if (a.M > 64 && (tiles_128x256 >= 64 || a.Kpad / BK >= 128)) return launch_variant(a, 5, stream);
  return launch_variant(a, 0, stream);
}

}  // namespace mmd8
