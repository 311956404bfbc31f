// int8 MFMA GEMM with the fused mixed-decomposition epilogue ("Compression techniques", item 2).
//
//   acc[m,n] = sum_k Xq[m,k] Wt[n,k]                      v_mfma_i32_32x32x32_i8, exact
//   Y[m,n]   = f16( acc r[m] c[n] / 127^2                  outer-product dequantization
//                   + sum_j X[m,O_j] f16(Wt[n,O_j] c[n]/127)   v_mfma_f32_32x32x16_f16 on the critical columns
//                   + bias[n] )
//
// Both operands are K-contiguous byte matrices padded to whole tiles (rows to kPackN, K to
// kPackK), so the main loop has no bounds checks.  A workgroup owns one BM x BN tile of Y.
// K is walked in slabs of BK bytes.  A slab of both operands goes from global memory straight
// into LDS (global_load_lds_dwordx4: no register staging) through a ring of LDS buffers, two
// slabs ahead of the MFMAs.  LDS rows are BK bytes; the 16-byte chunks of a row are XOR-swizzled
// with a function of the row so that the rows read by neighbouring lanes of a ds_read_b128 fall
// in distinct banks.  A lane's 16 bytes feed one operand row of the 32x32x32 MFMA; the k order
// inside the instruction is irrelevant as long as both operands use the same chunk for the same
// lane group, which they do.  Operand fragments are double-buffered in registers, so the LDS
// reads of one k-step run under the MFMAs of the previous one.
#include <type_traits>

#include "common.h"
#include "gemm.h"
#include "weight_layout.h"

namespace mmd8 {

template <int kBK>
__device__ inline int swizzle(int r) {
  if constexpr (kBK == 64) {
    // 4 chunks per row: distinct for rows {r, r+2, r+4, r+6} and for rows {r, r+4, r+8, r+12}
    return (((r >> 1) ^ (r >> 3)) & 1) | (((r >> 2) & 1) << 1);
  } else {
    // 8 chunks per row: a bijection of rows r..r+7 and, for fixed parity, of r, r+2, .., r+14
    return ((r >> 1) & 3) | ((((r) ^ (r >> 3)) & 1) << 2);
  }
}

template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int STAGES_, int WAVES_PER_SIMD_>
struct GemmCfg {
  static constexpr int kWavesPerSimd = WAVES_PER_SIMD_;           // register budget: 512 / this
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int kWaves = WAVES_M * WAVES_N;
  static constexpr int kThreads = kWaves * kWave;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  static constexpr int TI = WM / 32, TJ = WN / 32;                 // MFMA tiles per wave
  static constexpr int NKS = BK / 32;                              // MFMA k-steps per slab
  static constexpr int CPR = BK / 16;                              // 16-byte chunks per LDS row
  static constexpr int ROWS_PER_DMA = kWave / CPR;                 // rows covered by one wave-wide DMA
  static constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int kStages = STAGES_;
  static constexpr int LDS_BYTES = STAGE_BYTES * kStages;
  static constexpr int A_DMA = BM / ROWS_PER_DMA / kWaves;         // DMA instructions per wave per slab
  static constexpr int B_DMA = BN / ROWS_PER_DMA / kWaves;
  static constexpr int DMA_PER_SLAB = A_DMA + B_DMA;
  static_assert(BM % (ROWS_PER_DMA * kWaves) == 0 && BN % (ROWS_PER_DMA * kWaves) == 0, "tile/wave mismatch");
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be whole MFMA tiles");
  static_assert(NKS % 2 == 0, "fragment double buffering assumes an even number of k-steps");
  static_assert(kStages >= 3, "the slab ring needs one slab in use, one landed and one in flight");
  static constexpr int kAhead = kStages - 1;                       // slabs requested ahead of the MFMAs
  static_assert(LDS_BYTES <= 160 * 1024, "LDS");
  // epilogue staging of the critical columns: [rows][16 k] fp16 for both operands
  static constexpr int EPI_BYTES = (BM + BN) * 32;
  static_assert(EPI_BYTES <= LDS_BYTES, "epilogue staging must fit in the slab buffers");
};

// One 16-byte-per-lane global -> LDS copy (no registers in between).  Lane i's 16 bytes land at
// lds_addr + 16 i.  Issued through asm so that the compiler does not serialise later LDS reads
// behind it: completion is tracked by hand with vmcnt (see the main loop).
__device__ inline void dma16(const int8_t* src, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(src), "s"(lds_addr)
               : "memory");
}

template <int kVm>
__device__ inline void wait_slab_and_sync() {
  // own DMA older than the newest kVm instructions has landed, own LDS reads have returned;
  // after the barrier that holds for every wave of the workgroup
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" : : "n"(kVm) : "memory");
}

// Epilogue of one workgroup tile.  C layout of the 32x32 MFMA: a lane holds column (lane % 32);
// register e holds row 8 (e / 4) + 4 (lane / 32) + (e % 4).
// kFull: the tile lies wholly inside Y, so no store needs a bounds check.
// kTap: also write the raw int32 accumulators (parity checks).
// The accumulators stay where the MFMAs left them: they are dequantized in place (the registers
// then hold fp32 bits), the fp16 MFMAs of the critical columns accumulate onto them in place,
// and each 32x32 tile is converted and stored on its own, so the working set stays small.
template <class Cfg, bool kFull, bool kTap>
__device__ inline void epilogue(const GemmArgs& a, v16i (&acc)[Cfg::TI][Cfg::TJ], int8_t* smem, int m0, int n0,
                                int wm, int wn, int lane) {
  constexpr int TI = Cfg::TI, TJ = Cfg::TJ, TILE_M = Cfg::BM, TILE_N = Cfg::BN;
  const int lr = lane & 31, lg = lane >> 5;
  const int mw = m0 + wm * Cfg::WM, nw = n0 + wn * Cfg::WN;       // first row / column of the wave tile

  if constexpr (kTap) {
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int m = mw + i * 32 + 8 * (e / 4) + 4 * lg + (e % 4), n = nw + j * 32 + lr;
          if (m < a.M && n < a.N) a.tap_acc[(size_t)m * a.N + n] = acc[i][j][e];
        }
        __builtin_amdgcn_sched_barrier(0);
      }
  }

  // outer-product dequantization in place: acc * r[m] * (c[n] / 127^2)
  float cs[TJ];
#pragma unroll
  for (int j = 0; j < TJ; ++j) cs[j] = a.c[min(nw + j * 32 + lr, a.N - 1)] / 16129.0f;
#pragma unroll
  for (int i = 0; i < TI; ++i) {
    float rm[16];
#pragma unroll
    for (int q = 0; q < 4; ++q) {                                  // r is padded to whole tiles: always in bounds
      const v4f v = *reinterpret_cast<const v4f*>(a.r + mw + i * 32 + 8 * q + 4 * lg);
      rm[4 * q] = v[0], rm[4 * q + 1] = v[1], rm[4 * q + 2] = v[2], rm[4 * q + 3] = v[3];
    }
#pragma unroll
    for (int j = 0; j < TJ; ++j) {
      v16f y;
#pragma unroll
      for (int e = 0; e < 16; ++e) y[e] = (float)acc[i][j][e] * (rm[e] * cs[j]);
      acc[i][j] = __builtin_bit_cast(v16i, y);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  const int n_out = *a.n_out;
  if (n_out > 0) {
    // Critical columns, 16 at a time: stage X[m, O_j] (fp16) and f16(Wt[n, O_j] c[n] / 127) for the
    // whole tile in LDS as [row][16] fp16, then one 32x32x16 fp16 MFMA per output tile.
    uint16_t* sXo = reinterpret_cast<uint16_t*>(smem);             // [TILE_M][16], then [TILE_N][16]
    uint16_t* sWo = sXo + TILE_M * 16;
    __syncthreads();                                               // every wave is done with the slab ring
    for (int j0 = 0; j0 < n_out; j0 += 16) {
      for (int t = threadIdx.x; t < (TILE_M + TILE_N) * 16; t += Cfg::kThreads) {
        const int row = t >> 4, kk = t & 15;
        const int k = (j0 + kk < n_out) ? a.idx[j0 + kk] : -1;
        uint16_t v = 0;
        if (row < TILE_M) {
          const int m = m0 + row;
          if (k >= 0 && m < a.M) v = a.X[(size_t)m * a.ldx + k];
        } else {
          const int n = n0 + row - TILE_M;
          if (k >= 0 && n < a.N) {
            const float step = a.c[n] / 127.0f;
            v = (uint16_t)rounded_float_to_half_bits((float)a.Wt[(size_t)n * a.Kpad + k] * step);
          }
        }
        sXo[t] = v;
      }
      __syncthreads();
      v8h fxa[TI], fxb[TJ];
#pragma unroll
      for (int i = 0; i < TI; ++i)
        fxa[i] = *reinterpret_cast<const v8h*>(sXo + (wm * Cfg::WM + i * 32 + lr) * 16 + lg * 8);
#pragma unroll
      for (int j = 0; j < TJ; ++j)
        fxb[j] = *reinterpret_cast<const v8h*>(sWo + (wn * Cfg::WN + j * 32 + lr) * 16 + lg * 8);
#pragma unroll
      for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
          acc[i][j] = __builtin_bit_cast(
              v16i, __builtin_amdgcn_mfma_f32_32x32x16_f16(fxa[i], fxb[j], __builtin_bit_cast(v16f, acc[i][j]), 0, 0, 0));
      __syncthreads();
    }
  }

  // bias, rounding to fp16, and stores.  Neighbouring lanes hold neighbouring columns of the same
  // rows; an even/odd lane pair swaps halves so that each lane stores two adjacent columns (4
  // bytes): the even lane of row e, the odd lane of row e + 1.
  const int odd = lane & 1;
  // lane part of the store offset (elements); the row/column part is wave-uniform
  const int lane_off = (4 * lg + odd) * a.ldy + (lr & ~1);
#pragma unroll
  for (int j = 0; j < TJ; ++j) {
    const int n = nw + j * 32 + lr;
    const float bn = a.bias ? half_lo_to_float(a.bias[min(n, a.N - 1)]) : 0.0f;
#pragma unroll
    for (int i = 0; i < TI; ++i) {
      const v16f y = __builtin_bit_cast(v16f, acc[i][j]);
      uint16_t* tile = a.Y + (size_t)(mw + i * 32) * a.ldy + nw + j * 32;   // wave-uniform
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const uint32_t h = float_to_half_bits(y[e] + bn) | (float_to_half_bits(y[e + 1] + bn) << 16);
        const uint32_t p = (uint32_t)__builtin_amdgcn_mov_dpp((int)h, 0xb1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]
        const uint32_t out = odd ? ((p >> 16) | (h & 0xffff0000u)) : ((h & 0xffffu) | (p << 16));
        const int row = 8 * (e / 4) + (e % 4);                                 // + 4 lg + odd via lane_off
        bool ok = true;
        if constexpr (!kFull) ok = (mw + i * 32 + row + 4 * lg + odd < a.M) && ((n & ~1) < a.N);
        if (ok) *reinterpret_cast<uint32_t*>(tile + (size_t)row * a.ldy + lane_off) = out;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// kFull: M and N are multiples of the tile, so no output store needs a bounds check.
template <class Cfg, bool kTap, bool kFull>
__global__ __launch_bounds__(Cfg::kThreads, Cfg::kWavesPerSimd) void k_gemm_mixed(const GemmArgs a) {
  extern __shared__ __attribute__((aligned(1024))) int8_t smem[];
  constexpr int TI = Cfg::TI, TJ = Cfg::TJ, CPR = Cfg::CPR, BK = Cfg::BK, NKS = Cfg::NKS;
  constexpr int TILE_M = Cfg::BM, TILE_N = Cfg::BN, WAVES_N = Cfg::WAVES_N, STAGES = Cfg::kStages;

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  // ---- tile assignment: consecutive workgroup ids land on different XCDs (8 of them), so give
  // each XCD a contiguous run of tiles that walk M fastest: the run shares a few Wt row panels
  // through that XCD's L2.
  const int n_tiles = a.tiles_m * a.tiles_n;
  const int per_xcd = ceil_div(n_tiles, 8);
  const int logical = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (logical >= n_tiles) return;
  const int tm = logical % a.tiles_m, tn = logical / a.tiles_m;
  const int m0 = tm * TILE_M, n0 = tn * TILE_N;
  const int n_slabs = a.Kpad / BK;

  // ---- DMA plan of this lane: instruction j of this wave fills LDS rows
  // [(j kWaves + wave) ROWS_PER_DMA, +ROWS_PER_DMA) of the operand tile; the lane brings the
  // 16-byte chunk that belongs in slot (lane % CPR) of row (lane / CPR) of that group.
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
  const int8_t* srcA[Cfg::A_DMA];
  const int8_t* srcB[Cfg::B_DMA];
#pragma unroll
  for (int j = 0; j < Cfg::A_DMA; ++j) {
    const int r = (j * Cfg::kWaves + wave) * Cfg::ROWS_PER_DMA + lane / CPR;
    srcA[j] = a.Xq + (size_t)(m0 + r) * a.Kpad + ((lane % CPR) ^ swizzle<BK>(r)) * 16;
  }
#pragma unroll
  for (int j = 0; j < Cfg::B_DMA; ++j) {
    const int r = (j * Cfg::kWaves + wave) * Cfg::ROWS_PER_DMA + lane / CPR;
    srcB[j] = a.Wt + (size_t)(n0 + r) * a.Kpad + ((lane % CPR) ^ swizzle<BK>(r)) * 16;
  }
  // request d (0 .. DMA_PER_SLAB-1) of a slab: the A rows first, then the B rows
  auto issue_dma = [&](int slab, int stage, int d) {
    const uint32_t base = lds0 + stage * Cfg::STAGE_BYTES + wave * (kWave * 16);
    if (d < Cfg::A_DMA)
      dma16(srcA[d] + (size_t)slab * BK, base + d * Cfg::kWaves * (kWave * 16));
    else
      dma16(srcB[d - Cfg::A_DMA] + (size_t)slab * BK,
            base + Cfg::A_BYTES + (d - Cfg::A_DMA) * Cfg::kWaves * (kWave * 16));
  };
  auto issue_slab = [&](int slab, int stage) {
#pragma unroll
    for (int d = 0; d < Cfg::DMA_PER_SLAB; ++d) issue_dma(slab, stage, d);
  };

  // ---- per-lane LDS read offsets: row (lane % 32) of an MFMA tile, chunk (2 ks + lane / 32)
  const int lr = lane & 31, lg = lane >> 5;
  int a_off[NKS], b_off[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    const int ra = wm * Cfg::WM + lr, rb = wn * Cfg::WN + lr;
    a_off[ks] = (ra * CPR + ((2 * ks + lg) ^ swizzle<BK>(ra))) * 16;
    b_off[ks] = Cfg::A_BYTES + (rb * CPR + ((2 * ks + lg) ^ swizzle<BK>(rb))) * 16;
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
  // kIssue: slab s + kAhead exists and is requested in this iteration; kNext: slab s + 1 exists.
  constexpr int AHEAD = Cfg::kAhead;
  constexpr int MFMAS = TI * TJ;                                   // per k-step
  constexpr int DMA_PER_KS = Cfg::DMA_PER_SLAB / NKS;
  static_assert(Cfg::DMA_PER_SLAB % NKS == 0 && DMA_PER_KS >= 1 && DMA_PER_KS <= MFMAS, "request spreading");
  int stage = 0;
  auto iteration = [&](int s, auto issue_tag, auto next_tag) {
    constexpr bool kIssue = decltype(issue_tag)::value, kNext = decltype(next_tag)::value;
    const int stage1 = (stage + 1 == STAGES) ? 0 : stage + 1;
    const int stage_req = (stage == 0) ? STAGES - 1 : stage - 1;   // (s + kAhead) mod kStages
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      const int cur = ks & 1, nxt = cur ^ 1;
#pragma unroll
      for (int t = 0; t < MFMAS; ++t) {
        const int i = t / TJ, j = t % TJ;
        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
        if (t == 0) {
          // the first MFMA of the k-step goes out before any new LDS read, so the wait for its
          // fragments (read during the previous k-step) is already satisfied
          __builtin_amdgcn_sched_barrier(0);
          if (ks + 1 < NKS) {
            read_frags(stage, ks + 1, nxt);
          } else {
            // last k-step of the slab: make slab s+1 visible, then prefetch its first fragments
            // still allowed in flight: slabs s+2 .. s+kAhead-1 in full and the part of slab
            // s+kAhead requested during the earlier k-steps of this iteration
            wait_slab_and_sync<kIssue ? (AHEAD - 2) * Cfg::DMA_PER_SLAB + DMA_PER_KS * (NKS - 1) : 0>();
            if (kNext) read_frags(stage1, 0, nxt);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        // requests number (t DMA_PER_KS) / MFMAS .. ((t + 1) DMA_PER_KS) / MFMAS - 1 of this k-step
        if (kIssue && (t * DMA_PER_KS) / MFMAS != ((t + 1) * DMA_PER_KS) / MFMAS) {
          __builtin_amdgcn_sched_barrier(0);
          issue_dma(s + AHEAD, stage_req, ks * DMA_PER_KS + (t * DMA_PER_KS) / MFMAS);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    stage = stage1;
  };
  using yes = std::true_type;
  using no = std::false_type;

  static_assert(AHEAD >= 2 && AHEAD <= 3, "prologue written for two or three slabs ahead");
  int issued = 0;
  for (; issued < AHEAD && issued < n_slabs; ++issued) issue_slab(issued, issued);
  if (issued == 1)
    wait_slab_and_sync<0>();
  else if (issued == 2)
    wait_slab_and_sync<Cfg::DMA_PER_SLAB>();
  else
    wait_slab_and_sync<2 * Cfg::DMA_PER_SLAB>();
  read_frags(0, 0, 0);
  int s = 0;
  for (; s + AHEAD < n_slabs; ++s) iteration(s, yes{}, yes{});
  for (; s + 1 < n_slabs; ++s) iteration(s, no{}, yes{});
  iteration(s, no{}, no{});
  // every wave passed the last barrier after its last LDS read of the ring: the slab buffers are
  // free for the epilogue, which starts with a barrier of its own before writing them

  // ------------------------------------------------------------------ epilogue
  epilogue<Cfg, kFull, kTap>(a, acc, smem, m0, n0, wm, wn, lane);
}

template <class Cfg, bool kTap, bool kFull>
static hipError_t launch_one(const GemmArgs& a, hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_mixed<Cfg, kTap, kFull>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int grid = ceil_div(a.tiles_m * a.tiles_n, 8) * 8;
  hipLaunchKernelGGL((k_gemm_mixed<Cfg, kTap, kFull>), dim3(grid), dim3(Cfg::kThreads), Cfg::LDS_BYTES, stream, a);
  return hipGetLastError();
}

template <class Cfg>
static hipError_t launch_cfg(GemmArgs a, hipStream_t stream) {
  a.tiles_m = ceil_div(a.M, Cfg::BM);
  a.tiles_n = ceil_div(a.N, Cfg::BN);
  if (a.tap_acc) return launch_one<Cfg, true, false>(a, stream);
  const bool full = (a.M % Cfg::BM == 0) && (a.N % Cfg::BN == 0);
  return full ? launch_one<Cfg, false, true>(a, stream) : launch_one<Cfg, false, false>(a, stream);
}

hipError_t launch_gemm_mixed(const GemmArgs& a, int variant, hipStream_t stream) {
  if (variant < 0) {
    // automatic: the large tile whenever it fills the chip reasonably, else smaller tiles
    const long tiles_256 = (long)ceil_div(a.M, 256) * ceil_div(a.N, 256);
    const long tiles_128x256 = (long)ceil_div(a.M, 128) * ceil_div(a.N, 256);
    if (a.M > 128 && tiles_256 >= 192)
      variant = 3;
    else if (a.M > 64 && tiles_128x256 >= 64)
      variant = 2;
    else
      variant = 0;
  }
  switch (variant) {
    case 1: return launch_cfg<GemmCfg<256, 128, 64, 2, 2, 3, 2>>(a, stream);
    case 2: return launch_cfg<GemmCfg<128, 256, 64, 2, 2, 3, 2>>(a, stream);
    case 3: return launch_cfg<GemmCfg<256, 256, 64, 2, 4, 3, 2>>(a, stream);
    case 4: return launch_cfg<GemmCfg<128, 256, 64, 2, 2, 4, 2>>(a, stream);
    case 5: return launch_cfg<GemmCfg<256, 256, 64, 4, 2, 4, 2>>(a, stream);
    case 6: return launch_cfg<GemmCfg<256, 256, 64, 2, 4, 4, 2>>(a, stream);
    default: return launch_cfg<GemmCfg<128, 128, 64, 2, 2, 3, 2>>(a, stream);
  }
}

}  // namespace mmd8
