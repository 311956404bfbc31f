// Device-side pieces of the blockwise encoder ("Compression techniques", item 1) that more than one kernel
// file uses: the per-element code lookup, the 8-values-at-a-time encoder of the streaming kernel, and the
// span loop of the generic kernel with the source of its fp16 values left open (global memory for the
// codec itself; the summed partial outputs of a decode-shaped linear when the layer's result leaves coded).
// Each kernel file that encodes defines its own `__device__ const DynamicCode` from make_dynamic_code().
#pragma once
#include "common.h"
#include "dynamic_code.h"

namespace mmd8 {

// A block scale is the magnitude of an fp16 element.  It is stored either as fp32 (4 bytes per block, the
// default) or as the fp16 number it is (2 bytes per block): both are exact, the codes are the same.
__device__ inline void store_scale(float* p, size_t i, uint32_t fp16_pattern) { p[i] = half_lo_to_float(fp16_pattern); }
__device__ inline void store_scale(uint16_t* p, size_t i, uint32_t fp16_pattern) { p[i] = (uint16_t)fp16_pattern; }
__device__ inline float load_scale(const float* p, size_t i) { return p[i]; }
__device__ inline float load_scale(const uint16_t* p, size_t i) { return half_lo_to_float(p[i]); }

constexpr int kCodecThreads = 256;
constexpr int kCodecChunk = 8;                          // fp16 elements per 16-byte load
constexpr int kCodecSpanMax = 4096;                     // elements per span: 2 chunks per thread
constexpr int kCodecChunksPerThread = kCodecSpanMax / (kCodecThreads * kCodecChunk);
constexpr int kCodecSpanChunks = kCodecSpanMax / kCodecChunk;    // 512

// count of midpoints strictly below v, from the cell table in LDS
__device__ inline uint32_t encode_one(float v, const CodeCell* __restrict__ cells) {
  const uint32_t bits = __float_as_uint(v);
  const uint32_t sign = (uint32_t)((int32_t)bits >> 31);          // 0 or 0xffffffff
  const uint32_t u = (bits & 0x7fffffffu) - sign;                  // |v| bits, +1 for negatives (>= becomes >)
  uint32_t c = u >> kCellShift;
  c = min(max(c, (uint32_t)DynamicCode::kCellLo), (uint32_t)DynamicCode::kCellHi) - DynamicCode::kCellLo;
  const CodeCell cell = cells[c];
  uint32_t cnt = cell.base + (u > cell.threshold ? 1u : 0u);
  cnt = min(cnt, 128u + sign);                                     // negatives count P[0..126] only
  return 127u + ((cnt ^ sign) - sign);
}

// The generic encoder: any block size that is a multiple of 64, any n (ragged end included).  A workgroup
// of kCodecThreads threads walks spans of blocks_per_span whole blocks (at most kCodecSpanMax elements).
// src.chunk(e0, valid) returns the eight fp16 values that start at element e0 (a multiple of 8), of which
// `valid` (1..8) lie inside the tensor; the others must come back as zeros.
template <class Source, class Scale = float>
__device__ inline void encode_spans(const Source& src, size_t n, int block, uint8_t* __restrict__ codes,
                                    Scale* __restrict__ absmax, int blocks_per_span, size_t n_spans,
                                    const DynamicCode& code) {
  constexpr int kThreads = kCodecThreads, kChunk = kCodecChunk, kChunksPerThread = kCodecChunksPerThread;
  __shared__ CodeCell s_cells[DynamicCode::kCells];
  __shared__ uint32_t s_chunk_max[kCodecSpanChunks];    // |x| bit pattern maxima, one per 8-element chunk
  __shared__ uint32_t s_block_max[kCodecSpanMax / 64];

  for (int i = threadIdx.x; i < DynamicCode::kCells; i += kThreads) s_cells[i] = code.cell[i];

  const int chunks_per_block = block >> 3;
  const int span_elems = blocks_per_span * block;
  const int span_chunks = span_elems >> 3;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;

  for (size_t span = blockIdx.x; span < n_spans; span += gridDim.x) {
    const size_t span_base = span * (size_t)span_elems;
    v4u raw[kChunksPerThread];
    bool live[kChunksPerThread];
    int valid[kChunksPerThread];                   // elements of the chunk inside the tensor (0..8)
#pragma unroll
    for (int j = 0; j < kChunksPerThread; ++j) {
      const int ch = j * kThreads + threadIdx.x;
      const size_t e0 = span_base + (size_t)ch * kChunk;
      live[j] = ch < span_chunks && e0 < n;
      valid[j] = live[j] ? (int)min((size_t)kChunk, n - e0) : 0;
      raw[j] = v4u{0, 0, 0, 0};
      if (valid[j] > 0) raw[j] = src.chunk(e0, valid[j]);
    }
    // chunk maxima of |x| (fp16 magnitudes order like their 15-bit patterns)
#pragma unroll
    for (int j = 0; j < kChunksPerThread; ++j) {
      uint32_t m = 0;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t a = raw[j][w] & 0x7fff7fffu;
        m = max(m, max(a & 0xffffu, a >> 16));
      }
      const int ch = j * kThreads + threadIdx.x;
      if (ch < span_chunks) s_chunk_max[ch] = m;
    }
    __syncthreads();
    // block maxima: one wave per block, lanes stride over the block's chunks
    for (int b = wave; b < blocks_per_span; b += kThreads / kWave) {
      uint32_t m = 0;
      for (int c = lane; c < chunks_per_block; c += kWave) m = max(m, s_chunk_max[b * chunks_per_block + c]);
      m = wave_max_u32(m);
      if (lane == 0) {
        s_block_max[b] = m;
        const size_t gb = span * (size_t)blocks_per_span + b;
        if (gb * (size_t)block < n) store_scale(absmax, gb, m);
      }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kChunksPerThread; ++j) {
      if (!live[j]) continue;
      const int ch = j * kThreads + threadIdx.x;
      const int b = ch / chunks_per_block;
      const float a = half_lo_to_float(s_block_max[b]);
      const float inv = (a == 0.0f) ? 0.0f : 1.0f / a;            // IEEE division, once per chunk
      uint32_t out[2];
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        const uint32_t w0 = raw[j][2 * w], w1 = raw[j][2 * w + 1];
        const uint32_t c0 = encode_one(half_lo_to_float(w0) * inv, s_cells);
        const uint32_t c1 = encode_one(half_hi_to_float(w0) * inv, s_cells);
        const uint32_t c2 = encode_one(half_lo_to_float(w1) * inv, s_cells);
        const uint32_t c3 = encode_one(half_hi_to_float(w1) * inv, s_cells);
        out[w] = c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
      }
      const size_t e0 = span_base + (size_t)ch * kChunk;
      if (valid[j] == kChunk) {
        *reinterpret_cast<v2u*>(codes + e0) = v2u{out[0], out[1]};
      } else {
        for (int t = 0; t < valid[j]; ++t) codes[e0 + t] = (uint8_t)(out[t >> 2] >> (8 * (t & 3)));
      }
    }
    __syncthreads();                                // s_chunk_max / s_block_max are reused by the next span
  }
}

// ------------------------------------------------------------------------------------------------
// Fast encoder: eight values at a time.
//
// Encoding, per element: r = rotate_left(bits(v), 1) = 2 |v|bits + (v < 0), so that
// "|v| > P" for v >= 0 and "|v| >= P" for v < 0 are both  r > 2 bits(P);  cell = r >> 18;
// count = base[cell] + (r > threshold2[cell]).  The sign is applied afterwards on two counts at a
// time with packed 16-bit operations, taking the sign bits from the fp16 inputs.
// ------------------------------------------------------------------------------------------------
typedef unsigned short us2 __attribute__((ext_vector_type(2)));
typedef short ss2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) const v2u* lds_cell_ptr;

template <int kCtrl>
__device__ inline uint32_t dpp_max(uint32_t v) {
  return max(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, kCtrl, 0xf, 0xf, false));
}
// max over aligned groups of kLanes lanes, result in every lane of the group
template <int kLanes>
__device__ inline uint32_t group_max(uint32_t v) {
  if constexpr (kLanes >= 2) v = dpp_max<0xB1>(v);      // quad_perm [1,0,3,2]
  if constexpr (kLanes >= 4) v = dpp_max<0x4E>(v);      // quad_perm [2,3,0,1]
  if constexpr (kLanes >= 8) v = dpp_max<0x141>(v);     // row_half_mirror
  if constexpr (kLanes >= 16) v = dpp_max<0x140>(v);    // row_mirror
  if constexpr (kLanes >= 32) v = max(v, (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x401f));   // lane ^ 16
  if constexpr (kLanes >= 64)
    v = max((uint32_t)__builtin_amdgcn_readlane((int)v, 0), (uint32_t)__builtin_amdgcn_readlane((int)v, 32));
  return v;
}

__device__ inline uint32_t chunk_absmax_pattern(const v4u& raw) {
  us2 m = __builtin_bit_cast(us2, raw[0] & 0x7fff7fffu);
#pragma unroll
  for (int w = 1; w < 4; ++w) m = __builtin_elementwise_max(m, __builtin_bit_cast(us2, raw[w] & 0x7fff7fffu));
  const uint32_t both = __builtin_bit_cast(uint32_t, m);
  return max(both & 0xffffu, both >> 16);
}

__device__ inline uint32_t midpoints_below(float v, uint32_t cells_biased) {
  const uint32_t r = __builtin_amdgcn_alignbit(__float_as_uint(v), __float_as_uint(v), 31);
  const uint32_t c = min(max(r >> (kCellShift + 1), (uint32_t)DynamicCode::kCellLo), (uint32_t)DynamicCode::kCellHi);
  const v2u cell = *(lds_cell_ptr)(uintptr_t)(cells_biased + (c << 3));
  return cell[1] + (r > cell[0] ? 1u : 0u);
}

// f32(low or high fp16 half of `word`) * inv as one instruction: a fused multiply-add that reads the
// half directly, with addend +0.  Same rounding as a multiplication; a zero product may come out
// as +0 instead of -0, which lands in the same lookup cell with the same count.
template <bool kHigh>
__device__ inline float half_times(uint32_t word, float inv) {
  float v;
  if constexpr (kHigh)
    asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(v) : "v"(word), "v"(inv));
  else
    asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(v) : "v"(word), "v"(inv));
  return v;
}

// eight fp16 values (one 16-byte chunk) -> eight codes (8 bytes)
__device__ inline v2u encode_chunk(const v4u& raw, float inv, uint32_t cells_biased) {
  uint32_t pair[4];
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const uint32_t word = raw[w];
    const uint32_t n0 = midpoints_below(half_times<false>(word, inv), cells_biased);
    const uint32_t n1 = midpoints_below(half_times<true>(word, inv), cells_biased);
    const us2 cnt = __builtin_bit_cast(us2, n0 | (n1 << 16));
    // 0xffff in the halves where x < 0 (arithmetic shift of each half; written out because the
    // compiler turns the vector shift into compares and selects)
    uint32_t neg_bits;
    // (op_sel_hi: both halves take the shift count from the low half of the constant)
    asm("v_pk_ashrrev_i16 %0, 15, %1 op_sel_hi:[0,1]" : "=v"(neg_bits) : "v"(word));
    const us2 neg = __builtin_bit_cast(us2, neg_bits);
    // x >= 0: 127 + n ;  x < 0: 127 - min(n, 127) = a saturating 127 - n (n <= 128)
    const us2 up = (cnt & ~neg) + (unsigned short)127;
    pair[w] = __builtin_bit_cast(uint32_t, __builtin_elementwise_sub_sat(up, (us2)(cnt & neg)));
  }
  // pair[w] holds two codes in its 16-bit halves: gather the low bytes
  return v2u{__builtin_amdgcn_perm(pair[1], pair[0], 0x06040200u), __builtin_amdgcn_perm(pair[3], pair[2], 0x06040200u)};
}

// the cell table in the form midpoints_below reads it: {2 x threshold, base}
__device__ inline void stage_code_cells(v2u* s_cells, const DynamicCode& code, int tid, int n_threads) {
  for (int i = tid; i < DynamicCode::kCells; i += n_threads) {
    const CodeCell c = code.cell[i];
    s_cells[i] = v2u{c.threshold == kNoThreshold ? kNoThreshold : c.threshold * 2u, c.base};
  }
}
__device__ inline uint32_t biased_cell_base(const v2u* s_cells) {
  return (uint32_t)(uintptr_t)s_cells - (uint32_t)DynamicCode::kCellLo * 8u;
}

}  // namespace mmd8
