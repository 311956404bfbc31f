// Weight pre-quantization ("Compression techniques", item 2): per-column absmax, int8 codes,
// and the packed layout the GEMM streams.
//
// The codes are written transposed (Wt[n][k]: both GEMM operands are then K-contiguous, which is
// what the int8 MFMA fragments want, 16 consecutive k per lane) in the blocked order described in
// operand_layout.h; padding is zero.
#include "common.h"
#include "launchers.h"
#include "operand_layout.h"

namespace mmd8 {

// c[n] = max_k |W[k,n]| via atomicMax on the bit pattern of the non-negative float; c must be
// zero on entry.  Thread = 8 columns (16 bytes), workgroup = 32 column groups x 8 row lanes.
__global__ __launch_bounds__(256) void k_col_absmax(const uint16_t* __restrict__ W, int K, int N, int ldw,
                                                    uint32_t* __restrict__ c_bits) {
  const int cg = threadIdx.x & 31, rl = threadIdx.x >> 5;
  const int n0 = (blockIdx.x * 32 + cg) * 8;
  const bool live = n0 < N;
  uint32_t m[4] = {0, 0, 0, 0};
  typedef unsigned short us2 __attribute__((ext_vector_type(2)));
  // four rows in flight per thread (rows past K read as zeros)
  const int stride = gridDim.y * 8;
  for (int k = blockIdx.y * 8 + rl; k < K; k += 4 * stride) {
    v4u raw[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      raw[u] = v4u{0, 0, 0, 0};
      if (live && k + u * stride < K) raw[u] = *reinterpret_cast<const v4u*>(W + (size_t)(k + u * stride) * ldw + n0);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const us2 a = __builtin_bit_cast(us2, raw[u][w] & 0x7fff7fffu);
        m[w] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(us2, m[w]), a));
      }
  }
  // the 8 row lanes of a column group meet in LDS: one atomic per column and workgroup
  __shared__ uint32_t s_m[8][32][4];
#pragma unroll
  for (int w = 0; w < 4; ++w) s_m[rl][cg][w] = m[w];
  __syncthreads();
  if (rl == 0 && live) {
#pragma unroll
    for (int r = 1; r < 8; ++r)
#pragma unroll
      for (int w = 0; w < 4; ++w)
        m[w] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(us2, m[w]), __builtin_bit_cast(us2, s_m[r][cg][w])));
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      atomicMax(c_bits + n0 + 2 * w, __float_as_uint(half_lo_to_float(m[w])));
      atomicMax(c_bits + n0 + 2 * w + 1, __float_as_uint(half_hi_to_float(m[w])));
    }
  }
}

// One workgroup converts a tile of 128 k x 64 n and writes it transposed through LDS.
constexpr int kTileK = 128, kTileN = 64;
__device__ inline uint32_t weight_code(float w, float scale) {
  float q = __builtin_rintf(w * scale);
  q = fminf(fmaxf(q, -127.0f), 127.0f);
  return (uint32_t)((int)q) & 0xffu;
}
__global__ __launch_bounds__(256) void k_weight_quant_pack(const uint16_t* __restrict__ W, int K, int N, int ldw,
                                                           const float* __restrict__ c,
                                                           int8_t* __restrict__ Wt, int n_slabs) {
  // the transposed tile: row n holds its 128 codes as eight 16-byte chunks, chunk q stored at place q ^ (n / 8).
  // A thread has the codes of 8 columns n for 4 neighbouring k: one dword per column.  The 8 column groups of a
  // wave are 8 rows apart, which is a whole number of bank cycles for any 16-byte aligned row length, so
  // without the exchange of chunks they would all write to the same banks.
  constexpr int kRowBytes = kTileK + 16;
  __shared__ __attribute__((aligned(16))) uint8_t s_tile[kTileN][kRowBytes];
  const int kt0 = blockIdx.x * kTileK, nt0 = blockIdx.y * kTileN;
  const int cg = threadIdx.x & 7, rl = threadIdx.x >> 3;          // 8 column groups x 32 groups of 4 rows (k)
  const int n0 = nt0 + cg * 8;
  float scale[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const float cn = (n0 + t < N) ? c[n0 + t] : 0.0f;
    scale[t] = (cn == 0.0f) ? 0.0f : 127.0f / cn;                  // IEEE division
  }
  v4u raw[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int k = kt0 + 4 * rl + i;
    // unconditional loads (all four in flight together); rows and columns outside W re-read its first element
    // and are masked
    const bool ok = k < K && n0 < N;
    raw[i] = *reinterpret_cast<const v4u*>(W + (ok ? (size_t)k * ldw + n0 : (size_t)0));
    if (!ok) raw[i] = v4u{0, 0, 0, 0};
  }
  uint32_t col[8] = {0, 0, 0, 0, 0, 0, 0, 0};                       // column t: the codes of k .. k + 3, lowest byte first
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      col[2 * w] |= weight_code(half_lo_to_float(raw[i][w]), scale[2 * w]) << (8 * i);
      col[2 * w + 1] |= weight_code(half_hi_to_float(raw[i][w]), scale[2 * w + 1]) << (8 * i);
    }
  // dword rl of the row = chunk rl / 4, dword rl % 4 inside it
#pragma unroll
  for (int t = 0; t < 8; ++t)
    *reinterpret_cast<uint32_t*>(&s_tile[cg * 8 + t][(((rl >> 2) ^ cg) << 4) + ((rl & 3) << 2)]) = col[t];
  __syncthreads();
  // one 64-byte slab of the 64 rows per pass: 4 KB contiguous in the packed layout
  static_assert(kTileK / kSlabBytes == 2 && kTileN * (kSlabBytes / 16) == 256, "write-out mapping");
#pragma unroll
  for (int pass = 0; pass < kTileK / kSlabBytes; ++pass) {
    const int nl = threadIdx.x >> 2, ch = threadIdx.x & 3;
    const v4u v = *reinterpret_cast<const v4u*>(&s_tile[nl][((pass * 4 + ch) ^ (nl >> 3)) << 4]);
    *reinterpret_cast<v4u*>(Wt + packed_chunk_offset(nt0 + nl, kt0 / kSlabBytes + pass, ch, n_slabs)) = v;
  }
}

__global__ void k_weight_unpack(const int8_t* __restrict__ Wt, int K, int N, int n_slabs,
                                int8_t* __restrict__ Wq) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)K * N) return;
  const int k = (int)(i / N), n = (int)(i % N);
  Wq[i] = Wt[packed_offset(n, k, n_slabs)];
}

hipError_t launch_col_absmax(const uint16_t* W, int K, int N, int ldw, float* c, hipStream_t stream) {
  const int ysplit = max(1, min(ceil_div(K, 32), 2048 / max(1, ceil_div(N, 256))));
  hipLaunchKernelGGL(k_col_absmax, dim3(ceil_div(N, 256), ysplit), dim3(256), 0, stream, W, K, N, ldw,
                     reinterpret_cast<uint32_t*>(c));
  return hipGetLastError();
}

hipError_t launch_weight_quant_pack(const uint16_t* W, int K, int N, int ldw, const float* c, int8_t* Wt,
                                    hipStream_t stream) {
  const int Kpad = packed_k(K), Npad = packed_n(N);
  hipLaunchKernelGGL(k_weight_quant_pack, dim3(Kpad / kTileK, Npad / kTileN), dim3(256), 0, stream, W, K, N, ldw,
                     c, Wt, Kpad / kSlabBytes);
  return hipGetLastError();
}

hipError_t launch_weight_unpack(const int8_t* Wt, int K, int N, int8_t* Wq, hipStream_t stream) {
  const size_t total = (size_t)K * N;
  hipLaunchKernelGGL(k_weight_unpack, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, Wt, K, N,
                     packed_k(K) / kSlabBytes, Wq);
  return hipGetLastError();
}

}  // namespace mmd8
