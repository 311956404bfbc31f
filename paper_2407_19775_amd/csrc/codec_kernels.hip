// Dynamic blockwise 8-bit codec kernels ("Compression techniques", item 1).
//
// Both directions are streaming kernels bound by HBM traffic (3 + 4/B bytes per element).
// A workgroup of 256 threads works on a span of whole quantization blocks of at most 4096
// elements, 16 bytes of fp16 per thread per load; workgroups stride over the spans so the
// lookup tables are staged into LDS once per workgroup, not once per span.
#include "common.h"
#include "dynamic_code.h"
#include "codec_device.h"
#include "launchers.h"

namespace mmd8 {

static constexpr DynamicCode kCodeHost = make_dynamic_code();
static_assert(kCodeHost.one_midpoint_per_cell, "a lookup cell holds more than one midpoint");
static_assert(sizeof(CodeCell) == 8, "cell is read with one 64-bit LDS load");
__device__ const DynamicCode kCodeDev = make_dynamic_code();

const float* code_table_host() { return kCodeHost.T; }
const float* code_midpoints_host() { return kCodeHost.Mid; }

constexpr int kThreads = kCodecThreads;
constexpr int kChunk = kCodecChunk;               // fp16 elements per 16-byte load
constexpr int kSpanMax = kCodecSpanMax;           // elements per span: 2 chunks per thread

// the tensor itself as the source of the generic encoder
struct GlobalHalves {
  const uint16_t* x;
  __device__ v4u chunk(size_t e0, int valid) const {
    if (valid == kChunk) return *reinterpret_cast<const v4u*>(x + e0);
    uint32_t tmp[4] = {0, 0, 0, 0};              // ragged end of the tensor: element loads
    for (int t = 0; t < valid; ++t) tmp[t >> 1] |= (uint32_t)x[e0 + t] << (16 * (t & 1));
    return v4u{tmp[0], tmp[1], tmp[2], tmp[3]};
  }
};

// Generic kernel: any block size that is a multiple of 64, any n (ragged end included).
template <class Scale>
__global__ __launch_bounds__(kThreads) void k_quantize_blockwise(
    const uint16_t* __restrict__ x, size_t n, int block, uint8_t* __restrict__ codes,
    Scale* __restrict__ absmax, int blocks_per_span, size_t n_spans) {
  encode_spans(GlobalHalves{x}, n, block, codes, absmax, blocks_per_span, n_spans, kCodeDev);
}

// ------------------------------------------------------------------------------------------------
// Fast path: block sizes that are powers of two.  The unit of work is what one wave encodes on its own: 1024
// elements (two 16-byte loads per lane, 1 KB per wave instruction) holding whole blocks of up to 1024, or one
// whole block of 2048 / 4096 elements (four / eight loads per lane).  A block never leaves its wave, so every
// absmax is a cross-lane reduction (DPP / swizzle): no LDS memory, no barrier.  (The per-element encoding is in
// codec_device.h.)
//
// Launch shape: a fixed number of workgroups per compute unit (kEncodeGroupsPerCu, fewer for small tensors); a
// wave walks its units with the loads of the next one already in flight while the current one is encoded and
// stored, so reads and writes overlap inside every wave instead of the launch being one burst of reads
// followed by one burst of writes.  (Measured on the [8192, 8192] hidden state, blocks of 256: two 4096-element
// spans per short workgroup with all loads first 41.5 us; this form with 4 / 6 / 8 / 12 / 16 workgroups per
// compute unit 39.2 / 38.4 / 37.5 / 39.8 / 38.7 us; plain instead of nontemporal accesses 41.0 us.)
// ------------------------------------------------------------------------------------------------
constexpr int kEncodeGroupsPerCu = 8;
constexpr int kWavesPerGroup = kThreads / kWave;
template <int kLogBlock>
constexpr int encode_unit() { return (1 << kLogBlock) > 1024 ? (1 << kLogBlock) : 1024; }

template <int kLogBlock, class Scale>
__global__ __launch_bounds__(kThreads) void k_quantize_pow2(const uint16_t* __restrict__ x, size_t n_units,
                                                            uint8_t* __restrict__ codes,
                                                            Scale* __restrict__ absmax) {
  static_assert(kLogBlock >= 6 && kLogBlock <= 12, "64 .. 4096");
  __shared__ v2u s_cells[DynamicCode::kCells];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  constexpr int kBlock = 1 << kLogBlock;
  constexpr int kUnit = encode_unit<kLogBlock>();
  constexpr int kLoads = kUnit / (kWave * kChunk);                 // 16-byte loads per lane and unit: 2, 4 or 8
  constexpr int kLanesPerBlock = kBlock / kChunk;                  // lanes of one load that share a block (small blocks)

  auto load_unit = [&](size_t u, v4u (&r)[kLoads]) {
    const uint16_t* base = x + u * kUnit + lane * kChunk;
#pragma unroll
    for (int c = 0; c < kLoads; ++c) r[c] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(base + c * (kWave * kChunk)));
  };
  const size_t stride = (size_t)gridDim.x * kWavesPerGroup;
  size_t u = (size_t)blockIdx.x * kWavesPerGroup + wave;
  v4u raw[kLoads], ahead[kLoads];
  if (u < n_units) load_unit(u, raw);
  for (int i = threadIdx.x; i < DynamicCode::kCells; i += kThreads) {
    const CodeCell c = kCodeDev.cell[i];
    s_cells[i] = v2u{c.threshold == kNoThreshold ? kNoThreshold : c.threshold * 2u, c.base};
  }
  __syncthreads();                                                 // the only barrier: every wave passes it once
  const uint32_t cells_biased = (uint32_t)(uintptr_t)s_cells - (uint32_t)DynamicCode::kCellLo * 8u;

  for (; u < n_units; u += stride) {
    const size_t u_next = u + stride;
    if (u_next < n_units) load_unit(u_next, ahead);                // (uniform over the wave; nothing is fetched twice)
    const size_t e0 = u * kUnit;                                   // first element of the unit
    uint32_t m[kLoads];
#pragma unroll
    for (int c = 0; c < kLoads; ++c) m[c] = chunk_absmax_pattern(raw[c]);
    if constexpr (kLogBlock <= 9) {
#pragma unroll
      for (int c = 0; c < kLoads; ++c) {
        m[c] = group_max<kLanesPerBlock>(m[c]);
        if ((lane & (kLanesPerBlock - 1)) == 0) store_scale(absmax, (e0 + c * (kWave * kChunk) + lane * kChunk) >> kLogBlock, m[c]);
      }
    } else {
      uint32_t mm = m[0];
#pragma unroll
      for (int c = 1; c < kLoads; ++c) mm = max(mm, m[c]);
      mm = group_max<kWave>(mm);                                   // the unit is one block
      if (lane == 0) store_scale(absmax, e0 >> kLogBlock, mm);
#pragma unroll
      for (int c = 0; c < kLoads; ++c) m[c] = mm;
    }
    uint8_t* out = codes + e0 + lane * kChunk;
    float inv = 0.0f;
#pragma unroll
    for (int c = 0; c < kLoads; ++c) {
      if (kLogBlock <= 9 || c == 0) {
        const float a = half_lo_to_float(m[c]);
        inv = (a == 0.0f) ? 0.0f : 1.0f / a;                       // IEEE division
      }
      __builtin_nontemporal_store(encode_chunk(raw[c], inv, cells_biased), reinterpret_cast<v2u*>(out + c * (kWave * kChunk)));
    }
#pragma unroll
    for (int c = 0; c < kLoads; ++c) raw[c] = ahead[c];
  }
}

// Decoder.  A group is 8 codes: 8 bytes in, 16 bytes out per lane, so that every load instruction of
// a wave reads 512 and every store instruction writes 1024 consecutive bytes.  The block index of a
// group is unique because every block size is a multiple of 64.
constexpr int kDeqGroup = 8;
__device__ inline v4u decode_group(const v2u& c, float a, const float* s_T) {
  uint32_t o[4];
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    const uint32_t cw = c[w];
    const float f0 = s_T[cw & 0xffu] * a;
    const float f1 = s_T[(cw >> 8) & 0xffu] * a;
    const float f2 = s_T[(cw >> 16) & 0xffu] * a;
    const float f3 = s_T[cw >> 24] * a;
    o[2 * w] = rounded_float_to_half_bits(f0) | (rounded_float_to_half_bits(f1) << 16);
    o[2 * w + 1] = rounded_float_to_half_bits(f2) | (rounded_float_to_half_bits(f3) << 16);
  }
  return v4u{o[0], o[1], o[2], o[3]};
}

// Whole groups only.  A thread decodes kDeqPerThread groups that lie an eighth of the tensor apart,
// all loads first (same launch shape as the encoder).
constexpr int kDeqPerThread = 8;
// kPow2: the block size is 1 << log_block (otherwise log_block is unused: the block index is a 64-bit division,
// which must not sit in front of the loads of the common case).
template <class Scale, bool kPow2>
__global__ __launch_bounds__(kThreads) void k_dequantize_blockwise(
    const uint8_t* __restrict__ codes, const Scale* __restrict__ absmax, int block,
    int log_block, uint16_t* __restrict__ out, size_t n_groups) {
  __shared__ float s_T[256];
  const size_t stride = (size_t)gridDim.x * kThreads;
  const size_t g0 = (size_t)blockIdx.x * kThreads + threadIdx.x;
  v2u c[kDeqPerThread];
  float a[kDeqPerThread];
#pragma unroll
  for (int j = 0; j < kDeqPerThread; ++j) {
    const size_t g = g0 + j * stride;
    const size_t e0 = (g < n_groups ? g : n_groups - 1) * kDeqGroup;   // a missing group re-reads the last one
    c[j] = __builtin_nontemporal_load(reinterpret_cast<const v2u*>(codes + e0));
    a[j] = load_scale(absmax, kPow2 ? (e0 >> log_block) : (e0 / (size_t)block));
  }
  s_T[threadIdx.x] = kCodeDev.T[threadIdx.x];
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kDeqPerThread; ++j) {
    const size_t g = g0 + j * stride;
    if (g >= n_groups) break;
    __builtin_nontemporal_store(decode_group(c[j], a[j], s_T), reinterpret_cast<v4u*>(out + g * kDeqGroup));
  }
}

// The last, short group of a tensor whose length is not a multiple of 8: one thread.
template <class Scale>
__global__ void k_dequantize_tail(const uint8_t* __restrict__ codes, const Scale* __restrict__ absmax, size_t e0, int valid,
                                  int block, uint16_t* __restrict__ out) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const float a = load_scale(absmax, e0 / (size_t)block);
  for (int t = 0; t < valid; ++t)
    out[e0 + t] = (uint16_t)rounded_float_to_half_bits(kCodeDev.T[codes[e0 + t]] * a);
}

// ------------------------------------------------------------------ launchers
static int log2_exact(int v) {
  for (int l = 0; l < 31; ++l)
    if ((1 << l) == v) return l;
  return -1;
}

template <class Scale>
static hipError_t launch_quantize_generic(const uint16_t* x, size_t n, int block, uint8_t* codes, Scale* absmax,
                                          hipStream_t stream) {
  const int blocks_per_span = kSpanMax / block;                  // >= 1
  const size_t span_elems = (size_t)blocks_per_span * block;
  const size_t n_spans = (n + span_elems - 1) / span_elems;
  const size_t max_grid = (size_t)device_cu_count() * 8;
  const dim3 grid((unsigned)(n_spans < max_grid ? n_spans : max_grid));
  hipLaunchKernelGGL(k_quantize_blockwise<Scale>, grid, dim3(kThreads), 0, stream, x, n, block, codes, absmax,
                     blocks_per_span, n_spans);
  return hipGetLastError();
}

template <class Scale>
static hipError_t launch_quantize_any(const uint16_t* x, size_t n, int block, uint8_t* codes, Scale* absmax,
                                      hipStream_t stream) {
  const int log_block = log2_exact(block);
  if (log_block < 0) return launch_quantize_generic(x, n, block, codes, absmax, stream);
  // whole units on the fast path (1024 elements, or one block of 2048 / 4096), the ragged end (whole blocks plus a
  // short one) through the generic kernel
  const size_t unit = block > 1024 ? (size_t)block : 1024;
  const size_t n_units = n / unit;
  if (n_units > 0) {
    // (a 4096-element unit keeps 16 loads per lane in flight and needs more registers: fewer workgroups per compute
    // unit, so that all of them are resident together)
    const size_t per_cu = log_block >= 12 ? kEncodeGroupsPerCu / 2 : kEncodeGroupsPerCu;
    const size_t want = (n_units + kWavesPerGroup - 1) / kWavesPerGroup, max_groups = (size_t)device_cu_count() * per_cu;
    const dim3 grid((unsigned)(want < max_groups ? want : max_groups));
#define MMD8_Q(L) hipLaunchKernelGGL((k_quantize_pow2<L, Scale>), grid, dim3(kThreads), 0, stream, x, n_units, codes, absmax)
    switch (log_block) {
      case 6: MMD8_Q(6); break;
      case 7: MMD8_Q(7); break;
      case 8: MMD8_Q(8); break;
      case 9: MMD8_Q(9); break;
      case 10: MMD8_Q(10); break;
      case 11: MMD8_Q(11); break;
      default: MMD8_Q(12); break;
    }
#undef MMD8_Q
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const size_t done = n_units * unit;
  if (done < n)
    return launch_quantize_generic(x + done, n - done, block, codes + done, absmax + done / block, stream);
  return hipSuccess;
}

hipError_t launch_quantize_blockwise(const uint16_t* x, size_t n, int block, uint8_t* codes, float* absmax,
                                     hipStream_t stream) {
  return launch_quantize_any(x, n, block, codes, absmax, stream);
}
hipError_t launch_quantize_blockwise_h(const uint16_t* x, size_t n, int block, uint8_t* codes, uint16_t* absmax,
                                       hipStream_t stream) {
  return launch_quantize_any(x, n, block, codes, absmax, stream);
}

template <class Scale>
static hipError_t launch_dequantize_any(const uint8_t* codes, const Scale* absmax, size_t n, int block,
                                        uint16_t* out, hipStream_t stream) {
  const size_t n_groups = n / kDeqGroup;                         // whole groups
  if (n_groups > 0) {
    const size_t per_wg = (size_t)kThreads * kDeqPerThread;
    const dim3 grid((unsigned)((n_groups + per_wg - 1) / per_wg));
    const int log_block = log2_exact(block);
    if (log_block >= 0)
      hipLaunchKernelGGL((k_dequantize_blockwise<Scale, true>), grid, dim3(kThreads), 0, stream, codes, absmax, block, log_block,
                         out, n_groups);
    else
      hipLaunchKernelGGL((k_dequantize_blockwise<Scale, false>), grid, dim3(kThreads), 0, stream, codes, absmax, block, 0, out,
                         n_groups);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const int rest = (int)(n - n_groups * kDeqGroup);
  if (rest > 0) {
    hipLaunchKernelGGL(k_dequantize_tail<Scale>, dim3(1), dim3(64), 0, stream, codes, absmax, n_groups * kDeqGroup, rest, block,
                       out);
    return hipGetLastError();
  }
  return hipSuccess;
}
hipError_t launch_dequantize_blockwise(const uint8_t* codes, const float* absmax, size_t n, int block,
                                       uint16_t* out, hipStream_t stream) {
  return launch_dequantize_any(codes, absmax, n, block, out, stream);
}
hipError_t launch_dequantize_blockwise_h(const uint8_t* codes, const uint16_t* absmax, size_t n, int block,
                                         uint16_t* out, hipStream_t stream) {
  return launch_dequantize_any(codes, absmax, n, block, out, stream);
}

}  // namespace mmd8
