// Activation-side kernels of the mixed int8 linear layer ("Compression techniques", item 2):
// outlier scan + row absmax, compaction of the critical feature dimensions, int8 packing.
//
// fp16 magnitudes order like their 15-bit patterns, so the scan works on packed 16-bit integers:
// with th = the smallest fp16 pattern whose value is >= tau, |x| >= tau is  a >= th  on patterns,
// and  t = a - th  (mod 2^16) has its top bit set exactly for the sub-threshold entries while
// keeping their order; a single unsigned max of t therefore yields the row scale.
#include "common.h"
#include "gemm.h"
#include "weight_layout.h"

namespace mmd8 {

constexpr int kThreads = 256;

struct PackOutliers {   // operands of the critical-column slab, written alongside the int8 codes
  const int32_t* idx;
  const int32_t* n_out;
  const int8_t* Wt;
  const float* c;
  int N;
  uint16_t* Xo;
  uint16_t* Wo;
};

__global__ void k_fill_u32(uint32_t* __restrict__ p, uint32_t v, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// ------------------------------------------------------------------ scan
// One workgroup owns kRows consecutive rows over all K columns: row scales need no atomics.
// A column is flagged by a plain store of 1 (every writer stores the same value); the flag
// array must be zero on entry.
constexpr int kScanRows = 4;
typedef unsigned short us2 __attribute__((ext_vector_type(2)));
__device__ inline us2 as_us2(uint32_t v) { return __builtin_bit_cast(us2, v); }
__device__ inline uint32_t as_u32(us2 v) { return __builtin_bit_cast(uint32_t, v); }

__global__ __launch_bounds__(kThreads) void k_scan(const uint16_t* __restrict__ X, int M, int K, int ldx,
                                                   uint32_t th, uint8_t* __restrict__ flag,
                                                   float* __restrict__ r) {
  __shared__ uint32_t s_part[kScanRows][kThreads / kWave];
  const int m0 = blockIdx.x * kScanRows;
  const us2 th2 = as_us2(th | (th << 16));
  us2 rowt[kScanRows];
#pragma unroll
  for (int i = 0; i < kScanRows; ++i) rowt[i] = as_us2(0u);

  for (int k0 = threadIdx.x * 8; k0 < K; k0 += kThreads * 8) {
    v4u raw[kScanRows];
#pragma unroll
    for (int i = 0; i < kScanRows; ++i) {
      // rows past M read as zeros: sub-threshold for tau > 0, and for tau <= 0 every column is
      // flagged by the real rows anyway
      raw[i] = v4u{0, 0, 0, 0};
      if (m0 + i < M) raw[i] = *reinterpret_cast<const v4u*>(X + (size_t)(m0 + i) * ldx + k0);
    }
    uint32_t col_and[4] = {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu};
#pragma unroll
    for (int i = 0; i < kScanRows; ++i) {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const us2 t = as_us2(raw[i][w] & 0x7fff7fffu) - th2;      // per-half, wraps mod 2^16
        rowt[i] = __builtin_elementwise_max(rowt[i], t);
        col_and[w] &= as_u32(t);
      }
    }
    const uint32_t all_and = col_and[0] & col_and[1] & col_and[2] & col_and[3];
    if ((~all_and) & 0x80008000u) {                   // rare: some entry of this thread is >= th
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        if (!(col_and[w] & 0x8000u)) flag[k0 + 2 * w] = 1;
        if (!(col_and[w] & 0x80000000u)) flag[k0 + 2 * w + 1] = 1;
      }
    }
  }
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
#pragma unroll
  for (int i = 0; i < kScanRows; ++i) {
    const uint32_t both = as_u32(rowt[i]);
    const uint32_t m = wave_max_u32_to_lane63(max(both & 0xffffu, both >> 16));
    if (lane == kWave - 1) s_part[i][wave] = m;
  }
  __syncthreads();
  if (threadIdx.x < kScanRows && m0 + threadIdx.x < M) {
    uint32_t m = 0;
#pragma unroll
    for (int w = 0; w < kThreads / kWave; ++w) m = max(m, s_part[threadIdx.x][w]);
    // top bit set: a sub-threshold entry exists and its pattern is m + th (mod 2^16)
    r[m0 + threadIdx.x] = (m & 0x8000u) ? half_lo_to_float((m + th) & 0xffffu) : 0.0f;
  }
}

// ------------------------------------------------------------------ compaction
// Single workgroup: ascending list of flagged columns, their count, and a copy of the mask.
constexpr int kCompactThreads = 1024;
__global__ __launch_bounds__(kCompactThreads) void k_compact(const uint8_t* __restrict__ flag, int K,
                                                             int32_t* __restrict__ idx,
                                                             int32_t* __restrict__ n_out,
                                                             uint8_t* __restrict__ tap_mask,
                                                             int32_t* __restrict__ tap_idx,
                                                             int32_t* __restrict__ tap_n) {
  __shared__ int s_wave_total[kCompactThreads / kWave];
  const int per = ceil_div(K, kCompactThreads);
  const int k_begin = threadIdx.x * per;
  const int k_end = min(K, k_begin + per);
  int cnt = 0;
  for (int k = k_begin; k < k_end; ++k) {
    const uint8_t f = flag[k];
    cnt += f ? 1 : 0;
    if (tap_mask) tap_mask[k] = f ? 1 : 0;
  }
  // inclusive scan inside the wave
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  int incl = cnt;
  for (int d = 1; d < kWave; d <<= 1) {
    const int up = __shfl_up(incl, d, kWave);
    if (lane >= d) incl += up;
  }
  if (lane == kWave - 1) s_wave_total[wave] = incl;
  __syncthreads();
  int before = 0;
  for (int w = 0; w < wave; ++w) before += s_wave_total[w];
  int pos = before + incl - cnt;
  for (int k = k_begin; k < k_end; ++k) {
    if (flag[k]) {
      idx[pos] = k;
      if (tap_idx) tap_idx[pos] = k;
      ++pos;
    }
  }
  if (threadIdx.x == kCompactThreads - 1) {
    *n_out = before + incl;
    if (tap_n) *tap_n = before + incl;
  }
}

// ------------------------------------------------------------------ pack
// Xq[m, k] for k < Kpad (row stride Kpad): codes of the non-critical columns, zeros in the
// critical columns and in the padding.  One thread converts 16 columns (two 16-byte loads, one
// 16-byte store) of kPackRows rows; the thread's 16 column flags are turned into byte masks once.
constexpr int kPackRows = 8;
__device__ inline uint32_t to_code_byte(float x, float scale) {
  float q = __builtin_rintf(x * scale);
  q = fminf(fmaxf(q, -127.0f), 127.0f);
  return (uint32_t)((int)q) & 0xffu;
}
// Rows of the critical-column slab, 8 columns (16 bytes) per thread: Xo[m][j] = X[m, O_j] for
// the first kOutlierSlab critical columns and Wo[n][j] = f16(Wt[n, O_j] c[n] / 127); zero for
// j >= n_out.  The weights are dequantized with two roundings (fp32 product, then fp16).
__device__ inline void gather_outlier_slab(const uint16_t* __restrict__ X, int M, int ldx, int Kpad,
                                           const PackOutliers& o, int item) {
  const int row = item / (kOutlierSlab / 8), j0 = (item % (kOutlierSlab / 8)) * 8;
  if (row >= M + o.N) return;
  const int n_out = min(*o.n_out, kOutlierSlab);
  uint32_t out[4] = {0, 0, 0, 0};
  if (row < M) {
    for (int t = 0; t < 8 && j0 + t < n_out; ++t)
      out[t >> 1] |= (uint32_t)X[(size_t)row * ldx + o.idx[j0 + t]] << (16 * (t & 1));
    *reinterpret_cast<v4u*>(o.Xo + (size_t)row * kOutlierSlab + j0) = v4u{out[0], out[1], out[2], out[3]};
  } else {
    const int n = row - M;
    const float step = o.c[n] / 127.0f;
    for (int t = 0; t < 8 && j0 + t < n_out; ++t) {
      const float w = (float)o.Wt[(size_t)n * Kpad + o.idx[j0 + t]] * step;
      out[t >> 1] |= rounded_float_to_half_bits(w) << (16 * (t & 1));
    }
    *reinterpret_cast<v4u*>(o.Wo + (size_t)n * kOutlierSlab + j0) = v4u{out[0], out[1], out[2], out[3]};
  }
}

__global__ __launch_bounds__(kThreads) void k_pack(const uint16_t* __restrict__ X, int M, int K, int ldx,
                                                   const uint8_t* __restrict__ flag,
                                                   const float* __restrict__ r, int8_t* __restrict__ Xq,
                                                   int Kpad, int8_t* __restrict__ tap_xq, int pack_blocks_y,
                                                   const PackOutliers o) {
  if ((int)blockIdx.y >= pack_blocks_y) {                         // the extra blocks prepare the slab
    const int b = ((int)blockIdx.y - pack_blocks_y) * gridDim.x + blockIdx.x;
    gather_outlier_slab(X, M, ldx, Kpad, o, b * kThreads + threadIdx.x);
    return;
  }
  const int k0 = (blockIdx.x * kThreads + threadIdx.x) * 16;
  if (k0 >= Kpad) return;
  const int m0 = blockIdx.y * kPackRows;
  uint32_t keep[4] = {0, 0, 0, 0};                    // 0xff per kept byte
  if (k0 < K) {                                       // K % 16 == 0: a group is all inside or all padding
    const v4u f = *reinterpret_cast<const v4u*>(flag + k0);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      // bytes are 0 or 1: (1 - f) * 0xff per byte, no carries between bytes
      keep[w] = (0x01010101u - f[w]) * 0xffu;
    }
  }
#pragma unroll
  for (int i = 0; i < kPackRows; ++i) {
    const int m = m0 + i;
    if (m >= M) break;
    uint32_t out[4] = {0, 0, 0, 0};
    if (k0 < K) {
      const float rm = r[m];
      const float scale = (rm == 0.0f) ? 0.0f : 127.0f / rm;       // IEEE division
      const v4u a = *reinterpret_cast<const v4u*>(X + (size_t)m * ldx + k0);
      const v4u b = *reinterpret_cast<const v4u*>(X + (size_t)m * ldx + k0 + 8);
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        out[w] = to_code_byte(half_lo_to_float(a[2 * w]), scale) |
                 (to_code_byte(half_hi_to_float(a[2 * w]), scale) << 8) |
                 (to_code_byte(half_lo_to_float(a[2 * w + 1]), scale) << 16) |
                 (to_code_byte(half_hi_to_float(a[2 * w + 1]), scale) << 24);
        out[2 + w] = to_code_byte(half_lo_to_float(b[2 * w]), scale) |
                     (to_code_byte(half_hi_to_float(b[2 * w]), scale) << 8) |
                     (to_code_byte(half_lo_to_float(b[2 * w + 1]), scale) << 16) |
                     (to_code_byte(half_hi_to_float(b[2 * w + 1]), scale) << 24);
      }
#pragma unroll
      for (int w = 0; w < 4; ++w) out[w] &= keep[w];
    }
    const v4u o = v4u{out[0], out[1], out[2], out[3]};
    *reinterpret_cast<v4u*>(Xq + (size_t)m * Kpad + k0) = o;
    if (tap_xq && k0 < K) *reinterpret_cast<v4u*>(tap_xq + (size_t)m * K + k0) = o;
  }
}

// ------------------------------------------------------------------ launchers
hipError_t launch_fill_u32(uint32_t* p, uint32_t v, int n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_fill_u32, dim3(ceil_div(n, 256)), dim3(256), 0, stream, p, v, n);
  return hipGetLastError();
}

hipError_t launch_scan(const uint16_t* X, int M, int K, int ldx, uint32_t th, uint8_t* flag, float* r,
                       hipStream_t stream) {
  hipLaunchKernelGGL(k_scan, dim3(ceil_div(M, kScanRows)), dim3(kThreads), 0, stream, X, M, K, ldx, th, flag, r);
  return hipGetLastError();
}

hipError_t launch_compact(const uint8_t* flag, int K, int32_t* idx, int32_t* n_out, uint8_t* tap_mask,
                          int32_t* tap_idx, int32_t* tap_n, hipStream_t stream) {
  hipLaunchKernelGGL(k_compact, dim3(1), dim3(kCompactThreads), 0, stream, flag, K, idx, n_out, tap_mask, tap_idx,
                     tap_n);
  return hipGetLastError();
}

hipError_t launch_pack(const uint16_t* X, int M, int K, int ldx, const uint8_t* flag, const float* r, int8_t* Xq,
                       int Kpad, int8_t* tap_xq, const PackOutliers& o, hipStream_t stream) {
  const int gx = ceil_div(Kpad / 16, kThreads), pack_y = ceil_div(M, kPackRows);
  const int slab_items = (M + o.N) * (kOutlierSlab / 8);
  const int slab_y = ceil_div(ceil_div(slab_items, kThreads), gx);
  const dim3 grid(gx, pack_y + slab_y);
  hipLaunchKernelGGL(k_pack, grid, dim3(kThreads), 0, stream, X, M, K, ldx, flag, r, Xq, Kpad, tap_xq, pack_y, o);
  return hipGetLastError();
}

}  // namespace mmd8
