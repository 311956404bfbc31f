// int8 MFMA GEMM with the fused mixed-decomposition epilogue ("Compression techniques", item 2).
//
//   acc[m,n] = sum_k Xq[m,k] Wt[n,k]                      v_mfma_i32_32x32x32_i8, exact
//   Y[m,n]   = f16( acc r[m] c[n] / 127^2                  outer-product dequantization
//                   + sum_j X[m,O_j] f16(Wt[n,O_j] c[n]/127)   v_mfma_f32_32x32x16_f16 on the critical columns
//                   + bias[n] )
//
// Both operands are K-contiguous byte matrices padded to whole tiles (rows to kPackN, K to
// kPackK), so the main loop has no bounds checks.  A workgroup owns one BM x BN tile of Y.
// K is walked in slabs of BK bytes; each slab of both operands is brought from global memory
// straight into LDS (global_load_lds_dwordx4, no register staging) one slab ahead of the MFMAs.
// LDS rows are BK bytes; the 16-byte chunks of a row are XOR-swizzled with a function of the
// row so that the 16 rows read by 16 neighbouring lanes of a ds_read_b128 fall in distinct
// banks.  A lane's 16 bytes feed one operand row of the 32x32x32 MFMA; the k order inside the
// instruction is irrelevant as long as both operands use the same chunk for the same lane
// group, which they do.
#include "common.h"
#include "weight_layout.h"
#include "gemm.h"

namespace mmd8 {

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int kBK>
__device__ inline int swizzle(int r) {
  if constexpr (kBK == 64) {
    // 4 chunks per row
    return (((r >> 1) ^ (r >> 3)) & 1) | (((r >> 2) & 1) << 1);
  } else {
    // 8 chunks per row
    return ((r >> 1) & 3) | ((((r) ^ (r >> 3)) & 1) << 2);
  }
}

template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_>
struct GemmCfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int kWaves = WAVES_M * WAVES_N;
  static constexpr int kThreads = kWaves * kWave;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  static constexpr int TI = WM / 32, TJ = WN / 32;                 // MFMA tiles per wave
  static constexpr int CPR = BK / 16;                              // 16-byte chunks per LDS row
  static constexpr int ROWS_PER_DMA = kWave / CPR;                 // rows covered by one wave-wide DMA
  static constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int kStages = 2;
  static constexpr int LDS_BYTES = STAGE_BYTES * kStages;
  static constexpr int A_DMA = BM / ROWS_PER_DMA / kWaves;         // DMA instructions per wave per slab
  static constexpr int B_DMA = BN / ROWS_PER_DMA / kWaves;
  static_assert(BM % (ROWS_PER_DMA * kWaves) == 0 && BN % (ROWS_PER_DMA * kWaves) == 0, "tile/wave mismatch");
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be whole MFMA tiles");
  // epilogue staging of the critical columns: [rows][16 k] fp16 for both operands
  static constexpr int EPI_BYTES = (BM + BN) * 32;
  static_assert(EPI_BYTES <= LDS_BYTES, "epilogue staging must fit in the slab buffers");
};

template <class Cfg, int ROWS, int NDMA>
__device__ inline void dma_slab(const int8_t* __restrict__ g_tile /* row 0 of the tile, at this slab's k */,
                                int ld, int8_t* lds_tile, int wave, int lane) {
  constexpr int CPR = Cfg::CPR;
#pragma unroll
  for (int j = 0; j < NDMA; ++j) {
    const int inst = j * Cfg::kWaves + wave;
    const int r = inst * Cfg::ROWS_PER_DMA + lane / CPR;
    const int cs = lane % CPR;                                     // chunk slot inside the LDS row
    const int c = cs ^ swizzle<CPR * 16>(r);                       // chunk of the global row that belongs there
    const int8_t* src = g_tile + (size_t)r * ld + c * 16;
    int8_t* dst = lds_tile + inst * (kWave * 16);                  // wave-uniform; lane i lands at +16 i
    __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)dst, 16, 0, 0);
  }
}

// Epilogue of one workgroup tile.  C layout of the 32x32 MFMA: a lane holds column (lane % 32);
// register e holds row 8 (e / 4) + 4 (lane / 32) + (e % 4).
// kFull: the tile lies wholly inside Y, so no store needs a bounds check.
template <class Cfg, bool kFull>
__device__ inline void epilogue(const GemmArgs& a, v16i (&acc)[Cfg::TI][Cfg::TJ], int8_t* smem, int m0, int n0,
                                int wm, int wn, int lane) {
  constexpr int TI = Cfg::TI, TJ = Cfg::TJ, TILE_M = Cfg::BM, TILE_N = Cfg::BN;
  const int lr = lane & 31, lg = lane >> 5;
  const int mw = m0 + wm * Cfg::WM, nw = n0 + wn * Cfg::WN;       // first row / column of the wave tile

  if (a.tap_acc) {
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int m = mw + i * 32 + 8 * (e / 4) + 4 * lg + (e % 4), n = nw + j * 32 + lr;
          if (m < a.M && n < a.N) a.tap_acc[(size_t)m * a.N + n] = acc[i][j][e];
        }
  }

  // outer-product dequantization: y = acc * r[m] * (c[n] / 127^2)
  float cs[TJ];
#pragma unroll
  for (int j = 0; j < TJ; ++j) cs[j] = a.c[min(nw + j * 32 + lr, a.N - 1)] / 16129.0f;
  v16f y[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i) {
    float rm[16];
#pragma unroll
    for (int q = 0; q < 4; ++q) {                                  // r is padded to whole tiles: always in bounds
      const v4f v = *reinterpret_cast<const v4f*>(a.r + mw + i * 32 + 8 * q + 4 * lg);
      rm[4 * q] = v[0], rm[4 * q + 1] = v[1], rm[4 * q + 2] = v[2], rm[4 * q + 3] = v[3];
    }
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) y[i][j][e] = (float)acc[i][j][e] * (rm[e] * cs[j]);
  }

  const int n_out = *a.n_out;
  if (n_out > 0) {
    // Critical columns, 16 at a time: stage X[m, O_j] (fp16) and f16(Wt[n, O_j] c[n] / 127) for the
    // whole tile in LDS as [row][16] fp16, then one 32x32x16 fp16 MFMA per output tile, which adds
    // straight onto the dequantized integer part.
    uint16_t* sXo = reinterpret_cast<uint16_t*>(smem);             // [TILE_M][16], then [TILE_N][16]
    uint16_t* sWo = sXo + TILE_M * 16;
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
            v = (uint16_t)float_to_half_bits((float)a.Wt[(size_t)n * a.Kpad + k] * step);
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
          y[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fxa[i], fxb[j], y[i][j], 0, 0, 0);
      __syncthreads();
    }
  }

  // bias, rounding to fp16, and stores.  Neighbouring lanes hold neighbouring columns of the same
  // rows; an even/odd lane pair swaps halves so that each lane stores two adjacent columns (4
  // bytes): the even lane of row e, the odd lane of row e + 1.
  const int odd = lane & 1;
#pragma unroll
  for (int j = 0; j < TJ; ++j) {
    const int n = nw + j * 32 + lr;
    const float bn = a.bias ? half_lo_to_float(a.bias[min(n, a.N - 1)]) : 0.0f;
    const int n2 = n & ~1;
#pragma unroll
    for (int i = 0; i < TI; ++i) {
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const uint32_t h = float_to_half_bits(y[i][j][e] + bn) | (float_to_half_bits(y[i][j][e + 1] + bn) << 16);
        const uint32_t p = (uint32_t)__builtin_amdgcn_mov_dpp((int)h, 0xb1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]
        const uint32_t out = odd ? ((p >> 16) | (h & 0xffff0000u)) : ((h & 0xffffu) | (p << 16));
        const int m = mw + i * 32 + 8 * (e / 4) + 4 * lg + (e % 4) + odd;
        if (kFull || (m < a.M && n2 < a.N))                       // N is even: the pair is inside together
          *reinterpret_cast<uint32_t*>(a.Y + (size_t)m * a.ldy + n2) = out;
      }
    }
  }
}

template <class Cfg>
__global__ __launch_bounds__(Cfg::kThreads) void k_gemm_mixed(const GemmArgs a) {
  extern __shared__ __attribute__((aligned(1024))) int8_t smem[];
  constexpr int TI = Cfg::TI, TJ = Cfg::TJ, CPR = Cfg::CPR, BK = Cfg::BK;
  constexpr int TILE_M = Cfg::BM, TILE_N = Cfg::BN, WAVES_N = Cfg::WAVES_N;

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

  const int8_t* gA = a.Xq + (size_t)m0 * a.Kpad;
  const int8_t* gB = a.Wt + (size_t)n0 * a.Kpad;
  const int n_slabs = a.Kpad / BK;

  v16i acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

  // per-lane LDS read offsets: row (lane % 32) of an MFMA tile, chunk (2 ks + lane / 32)
  const int lr = lane & 31, lg = lane >> 5;
  int a_off[BK / 32], b_off[BK / 32];
#pragma unroll
  for (int ks = 0; ks < BK / 32; ++ks) {
    const int ra = wm * Cfg::WM + lr, rb = wn * Cfg::WN + lr;
    a_off[ks] = (ra * CPR + ((2 * ks + lg) ^ swizzle<BK>(ra))) * 16;
    b_off[ks] = Cfg::A_BYTES + (rb * CPR + ((2 * ks + lg) ^ swizzle<BK>(rb))) * 16;
  }

  dma_slab<Cfg, TILE_M, Cfg::A_DMA>(gA, a.Kpad, smem, wave, lane);
  dma_slab<Cfg, TILE_N, Cfg::B_DMA>(gB, a.Kpad, smem + Cfg::A_BYTES, wave, lane);

  for (int s = 0; s < n_slabs; ++s) {
    int8_t* cur = smem + (s & 1) * Cfg::STAGE_BYTES;
    int8_t* nxt = smem + ((s + 1) & 1) * Cfg::STAGE_BYTES;
    // every wave waits for its own part of this slab (the barrier's fence drains vmcnt), then
    // all waves meet: the whole slab is in LDS and nobody still reads the other buffer
    __syncthreads();
    v4i fa[BK / 32][TI], fb[BK / 32][TJ];
#pragma unroll
    for (int ks = 0; ks < BK / 32; ++ks) {
#pragma unroll
      for (int i = 0; i < TI; ++i) fa[ks][i] = *reinterpret_cast<const v4i*>(cur + a_off[ks] + i * 32 * BK);
#pragma unroll
      for (int j = 0; j < TJ; ++j) fb[ks][j] = *reinterpret_cast<const v4i*>(cur + b_off[ks] + j * 32 * BK);
    }
    if (s + 1 < n_slabs) {
      dma_slab<Cfg, TILE_M, Cfg::A_DMA>(gA + (size_t)(s + 1) * BK, a.Kpad, nxt, wave, lane);
      dma_slab<Cfg, TILE_N, Cfg::B_DMA>(gB + (size_t)(s + 1) * BK, a.Kpad, nxt + Cfg::A_BYTES, wave, lane);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 32; ++ks)
#pragma unroll
      for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[ks][i], fb[ks][j], acc[i][j], 0, 0, 0);
  }
  __syncthreads();                                                 // slab buffers are free from here on

  // ------------------------------------------------------------------ epilogue
  const bool full = (m0 + TILE_M <= a.M) && (n0 + TILE_N <= a.N);
  if (full)
    epilogue<Cfg, true>(a, acc, smem, m0, n0, wm, wn, lane);
  else
    epilogue<Cfg, false>(a, acc, smem, m0, n0, wm, wn, lane);
}

template <class Cfg>
static hipError_t launch_cfg(GemmArgs a, hipStream_t stream) {
  static bool attr_set = false;
  constexpr int TILE_M = Cfg::BM, TILE_N = Cfg::BN;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_mixed<Cfg>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  a.tiles_m = ceil_div(a.M, TILE_M);
  a.tiles_n = ceil_div(a.N, TILE_N);
  const int grid = ceil_div(a.tiles_m * a.tiles_n, 8) * 8;
  hipLaunchKernelGGL((k_gemm_mixed<Cfg>), dim3(grid), dim3(Cfg::kThreads), Cfg::LDS_BYTES, stream, a);
  return hipGetLastError();
}

hipError_t launch_gemm_mixed(const GemmArgs& a, int variant, hipStream_t stream) {
  switch (variant) {
    case 1: return launch_cfg<GemmCfg<256, 256, 64, 2, 4>>(a, stream);
    case 2: return launch_cfg<GemmCfg<128, 256, 64, 2, 2>>(a, stream);
    case 3: return launch_cfg<GemmCfg<256, 256, 128, 2, 4>>(a, stream);
    default: return launch_cfg<GemmCfg<128, 128, 64, 2, 2>>(a, stream);
  }
}

}  // namespace mmd8
