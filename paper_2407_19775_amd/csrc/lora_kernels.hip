// Low-rank adapter W' = W + B A on top of the int8 layer ("BSNS with parameter-efficient
// fine-tuning via adapters"): Y = (int8 layer)(X) + T B^T with T = f16(X A^T).
//
// k_lora_down computes T on the matrix cores (v_mfma_f32_16x16x32_f16, fp32 accumulation, one
// rounding to fp16) and lays T and B out as extra fp16 slabs behind the slabs of the critical columns,
// so that the GEMM kernel adds T B^T exactly as it adds the critical columns: more fp16 MFMAs onto
// the dequantized accumulators.  For decode shapes T is kept as a plain matrix and the product
// with B is added by the kernel that sums the split-K partial outputs.
#include "lora.h"
#include "operand_layout.h"

namespace mmd8 {

namespace {
constexpr int kLoraThreads = 512, kLoraWaves = kLoraThreads / kWave;
constexpr int kLoraRows = 16;          // rows of X per workgroup

// Workgroups [0, t_blocks * splits): 16 rows of T each, over one of `splits` ranges of K.  Wave w takes
// the 64-column steps w, w + 8, ... of the range;
// in a step lane l holds, for row (or rank index) l % 16, the 16 columns 16 (l / 16) .. + 16 as two
// MFMA operands of 8 (which 8 columns meet in one MFMA does not matter: both operands use the same
// assignment).  A^T is the first operand, X^T the second, so a lane ends up with four consecutive
// rank indices of one row.  The eight partial sums meet in LDS and are added in wave order; with one
// range the sum is rounded and stored, with several it goes to P[range][m][64] as fp32 and k_lora_reduce
// adds the ranges in index order (so the result does not depend on timing) and rounds.
// Workgroups from t_blocks * splits on copy B into the weight-side slabs.
// eight sums of row m (rank indices 8 ch .. + 8; exact zeros past the rank): rounded to fp16 and stored as
// part of T, of the caller's copy of T and of the activation-side slabs
__device__ inline void store_low_rank_activation(const LoraArgs& a, int m, int ch, const float (&sum)[8]) {
  uint32_t out[4] = {0, 0, 0, 0};
#pragma unroll
  for (int e = 0; e < 8; ++e) out[e >> 1] |= float_to_half_bits(sum[e]) << (16 * (e & 1));
  const v4u v = {out[0], out[1], out[2], out[3]};
  const int j0 = 8 * ch;
  *reinterpret_cast<v4u*>(a.T + (size_t)m * kLoraMaxRank + j0) = v;
  if (a.T_user && j0 < a.r) *reinterpret_cast<v4u*>(a.T_user + (size_t)m * a.r + j0) = v;
  if (a.Xo)
    *reinterpret_cast<v4u*>(reinterpret_cast<int8_t*>(a.Xo) + packed_chunk_offset(m, a.crit_slabs + ch / 4, ch % 4, a.f_slabs)) = v;
}

template <int kTiles>   // 16-wide tiles of the rank: ceil(r / 16)
__global__ __launch_bounds__(kLoraThreads) void k_lora_down(const LoraArgs a, int t_blocks, int splits, int steps_per_split,
                                                            float* __restrict__ P) {
  constexpr int kCols = kTiles * 16;
  __shared__ __attribute__((aligned(16))) float s_part[kLoraWaves][kLoraRows][kCols];
  const int n_chunks = 4 * lora_slabs(a.r);                         // 8-column chunks of the slabs
  if ((int)blockIdx.x >= t_blocks * splits) {
    const int item = ((int)blockIdx.x - t_blocks * splits) * kLoraThreads + (int)threadIdx.x;
    if (item >= a.N * n_chunks) return;
    const int ch = item / a.N, n = item % a.N;
    v4u v = {0, 0, 0, 0};
    if (8 * ch < a.r) v = *reinterpret_cast<const v4u*>(a.B + (size_t)n * a.r + 8 * ch);
    *reinterpret_cast<v4u*>(reinterpret_cast<int8_t*>(a.Wo) + packed_chunk_offset(n, a.crit_slabs + ch / 4, ch % 4, a.f_slabs)) = v;
    return;
  }
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int m0 = ((int)blockIdx.x % t_blocks) * kLoraRows, split = (int)blockIdx.x / t_blocks;
  const int li = lane & 15, kq = lane >> 4;
  const uint16_t* xrow = a.X + (size_t)min(m0 + li, a.M - 1) * a.ldx + 16 * kq;
  const uint16_t* arow[kTiles];
  bool jvalid[kTiles];
#pragma unroll
  for (int t = 0; t < kTiles; ++t) {
    const int j = 16 * t + li;
    jvalid[t] = j < a.r;
    arow[t] = a.A + (size_t)min(j, a.r - 1) * a.K + 16 * kq;
  }
  v4f acc[kTiles];
#pragma unroll
  for (int t = 0; t < kTiles; ++t) acc[t] = v4f{0, 0, 0, 0};

  const int steps = min(ceil_div(a.K, 64), (split + 1) * steps_per_split);   // end of this range
  constexpr int U = kTiles <= 2 ? 4 : 2;
  for (int s0 = split * steps_per_split + wave; s0 < steps; s0 += kLoraWaves * U) {
    v4u xf[U][2], af[U][kTiles][2];
    // every load is issued before the first use; a step past the end re-reads step 0 and is masked
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int s = s0 + u * kLoraWaves;
      const bool ok = s < steps && 64 * s + 16 * kq < a.K;
      const int k = ok ? 64 * s : 0;
      const uint32_t keep = ok ? 0xffffffffu : 0u;
#pragma unroll
      for (int h = 0; h < 2; ++h) xf[u][h] = *reinterpret_cast<const v4u*>(xrow + k + 8 * h) & keep;
#pragma unroll
      for (int t = 0; t < kTiles; ++t) {
        const uint32_t keep_a = (ok && jvalid[t]) ? 0xffffffffu : 0u;
#pragma unroll
        for (int h = 0; h < 2; ++h) af[u][t][h] = *reinterpret_cast<const v4u*>(arow[t] + k + 8 * h) & keep_a;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int t = 0; t < kTiles; ++t)
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, af[u][t][h]),
                                                          __builtin_bit_cast(v8h, xf[u][h]), acc[t], 0, 0, 0);
  }
  // lane: row li, rank indices 16 t + 4 kq .. + 4
#pragma unroll
  for (int t = 0; t < kTiles; ++t) *reinterpret_cast<v4f*>(&s_part[wave][li][16 * t + 4 * kq]) = acc[t];
  __syncthreads();

  const int item = threadIdx.x;
  if (item >= kLoraRows * n_chunks) return;
  const int m = m0 + item / n_chunks, ch = item % n_chunks, j0 = 8 * ch;
  if (m >= a.M) return;
  float sum[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (j0 < kCols) {
    for (int w = 0; w < kLoraWaves; ++w) {
      const v4f lo = *reinterpret_cast<const v4f*>(&s_part[w][item / n_chunks][j0]);
      const v4f hi = *reinterpret_cast<const v4f*>(&s_part[w][item / n_chunks][j0 + 4]);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        sum[e] += lo[e];
        sum[4 + e] += hi[e];
      }
    }
  }
  if (splits > 1) {
    float* p = P + ((size_t)split * a.M + m) * kLoraMaxRank + j0;
    *reinterpret_cast<v4f*>(p) = v4f{sum[0], sum[1], sum[2], sum[3]};
    *reinterpret_cast<v4f*>(p + 4) = v4f{sum[4], sum[5], sum[6], sum[7]};
    return;
  }
  store_low_rank_activation(a, m, ch, sum);
}

// one thread per (row, 8 rank indices): the ranges' sums in index order, then as in the one-range case
__global__ __launch_bounds__(256) void k_lora_reduce(const LoraArgs a, int splits, const float* __restrict__ P) {
  const int n_chunks = 4 * lora_slabs(a.r);
  const int item = blockIdx.x * 256 + threadIdx.x;
  if (item >= a.M * n_chunks) return;
  const int m = item / n_chunks, ch = item % n_chunks;
  float sum[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int s = 0; s < splits; ++s) {
    const float* p = P + ((size_t)s * a.M + m) * kLoraMaxRank + 8 * ch;
    const v4f lo = *reinterpret_cast<const v4f*>(p), hi = *reinterpret_cast<const v4f*>(p + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      sum[e] += lo[e];
      sum[4 + e] += hi[e];
    }
  }
  store_low_rank_activation(a, m, ch, sum);
}
}  // namespace

LoraPlan plan_lora(int M, int K) {
  // One range of K per 16-row tile unless K is long (8192 columns or more): every kernel here has a floor
  // of a few microseconds, so the second kernel that adds the ranges must save more than that.  Then K is
  // split until there are two workgroups per compute unit, every range at least sixteen 64-column steps.
  const int t_blocks = ceil_div(M, kLoraRows), steps = ceil_div(K, 64), cus = device_cu_count();
  LoraPlan p;
  const int want = steps < 128 ? 1 : max(1, min(min(2 * cus / t_blocks, steps / 16), 32));
  p.steps_per_split = ceil_div(steps, want);
  p.splits = ceil_div(steps, p.steps_per_split);
  p.partial_bytes = p.splits > 1 ? (size_t)p.splits * M * kLoraMaxRank * sizeof(float) : 0;
  return p;
}

hipError_t launch_lora_down(const LoraArgs& a, const LoraPlan& plan, float* partial, hipStream_t stream) {
  const int t_blocks = ceil_div(a.M, kLoraRows);
  const int b_blocks = a.Wo ? ceil_div(a.N * 4 * lora_slabs(a.r), kLoraThreads) : 0;
  const dim3 grid(t_blocks * plan.splits + b_blocks), block(kLoraThreads);
  switch (ceil_div(a.r, 16)) {
    case 1: hipLaunchKernelGGL(k_lora_down<1>, grid, block, 0, stream, a, t_blocks, plan.splits, plan.steps_per_split, partial); break;
    case 2: hipLaunchKernelGGL(k_lora_down<2>, grid, block, 0, stream, a, t_blocks, plan.splits, plan.steps_per_split, partial); break;
    case 3: hipLaunchKernelGGL(k_lora_down<3>, grid, block, 0, stream, a, t_blocks, plan.splits, plan.steps_per_split, partial); break;
    case 4: hipLaunchKernelGGL(k_lora_down<4>, grid, block, 0, stream, a, t_blocks, plan.splits, plan.steps_per_split, partial); break;
    default: return hipErrorInvalidValue;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || plan.splits == 1) return e;
  hipLaunchKernelGGL(k_lora_reduce, dim3(ceil_div(a.M * 4 * lora_slabs(a.r), 256)), dim3(256), 0, stream, a, plan.splits, partial);
  return hipGetLastError();
}

}  // namespace mmd8
