// Activation-side kernels of the mixed int8 linear layer ("Compression techniques", item 2):
// outlier scan + row absmax, compaction of the critical feature dimensions, int8 packing.
//
// fp16 magnitudes order like their 15-bit patterns, so the scan works on packed 16-bit integers:
// with th = the smallest fp16 pattern whose value is >= tau, |x| >= tau is  a >= th  on patterns,
// and  t = a - th  (mod 2^16) has its top bit set exactly for the sub-threshold entries while
// keeping their order; a single unsigned max of t therefore yields the row scale.
#include "common.h"
#include "dynamic_code.h"
#include "gemm.h"
#include "launchers.h"
#include "operand_layout.h"
#include "skinny.h"

namespace mmd8 {

constexpr int kThreads = 256;

// the 256 values of the dynamic code, for the preparation kernel that takes coded activations
struct CodeValues {
  float v[256];
};
constexpr CodeValues make_code_values() {
  CodeValues c{};
  const DynamicCode d = make_dynamic_code();
  for (int i = 0; i < 256; ++i) c.v[i] = d.T[i];
  return c;
}
__device__ const CodeValues kCodeValuesDev = make_code_values();

__global__ void k_fill_u32(uint32_t* __restrict__ p, uint32_t v, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// ------------------------------------------------------------------ scan
// One workgroup owns kRows consecutive rows over all K columns: row scales need no atomics.
// kRows is 4 for tall inputs and smaller for short ones, so that there are always enough
// workgroups to keep the memory system busy.
// A column is flagged by a plain byte store of 1 into a byte-per-column flag array that is zero
// when the kernel starts: every writer stores the same value and the readers are later kernels,
// so no atomics and no waiting are needed.  The flags are part of the workspace's standing state:
// zeroed once when the workspace is set up, read by the kernels that follow the scan, and zeroed
// again by the GEMM kernel that ends the call.
typedef unsigned short us2 __attribute__((ext_vector_type(2)));
__device__ inline us2 as_us2(uint32_t v) { return __builtin_bit_cast(us2, v); }
__device__ inline uint32_t as_u32(us2 v) { return __builtin_bit_cast(uint32_t, v); }
// 16 column flags (bytes 0 / 1) starting at column k0
__device__ inline v4u flags16(const uint8_t* __restrict__ flag, int k0) {
  return *reinterpret_cast<const v4u*>(flag + k0) & 0x01010101u;
}

template <int kScanRows>
__global__ __launch_bounds__(kThreads) void k_scan(const uint16_t* __restrict__ X, int M, int K, int ldx,
                                                   uint32_t th, int Kpad, uint8_t* __restrict__ flag, float* __restrict__ r_out) {
  __shared__ uint32_t s_part[kScanRows][kThreads / kWave];
  const int m0 = blockIdx.x * kScanRows;
  const us2 th2 = as_us2(th | (th << 16));
  us2 rowt[kScanRows];
#pragma unroll
  for (int i = 0; i < kScanRows; ++i) rowt[i] = as_us2(0u);

  // two column groups per pass: eight 16-byte loads in flight per thread
  for (int kk = threadIdx.x * 8; kk < K; kk += 2 * kThreads * 8) {
    v4u raw2[2][kScanRows];
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
      for (int i = 0; i < kScanRows; ++i) {
        // rows past M (and a missing second group) read as zeros: sub-threshold for tau > 0, and
        // for tau <= 0 every column is flagged by the real rows anyway
        raw2[g][i] = v4u{0, 0, 0, 0};
        const int kc = kk + g * kThreads * 8;
        if (m0 + i < M && kc < K) raw2[g][i] = *reinterpret_cast<const v4u*>(X + (size_t)(m0 + i) * ldx + kc);
      }
#pragma unroll
    for (int g = 0; g < 2; ++g) {
    const int k0 = kk + g * kThreads * 8;
    if (k0 >= K) break;
    const v4u (&raw)[kScanRows] = raw2[g];
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
    r_out[m0 + threadIdx.x] = (m & 0x8000u) ? half_lo_to_float((m + th) & 0xffffu) : 0.0f;
  }
}

// ------------------------------------------------------------------ row scale over the non-critical columns
// The alternative reading of the row scale: r[m] = max |X[m,k]| over the columns whose flag is 0.  It needs the
// flags of every row, so it is a pass of its own between the scan and the pack kernel: one wave per row, the
// row's 16-column pieces strided over the lanes, flags read 16 bytes at a time.
__global__ __launch_bounds__(kThreads) void k_row_absmax_noncritical(const uint16_t* __restrict__ X, int M, int K, int ldx,
                                                                     const uint8_t* __restrict__ flag,
                                                                     float* __restrict__ r_out) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int m = blockIdx.x * (kThreads / kWave) + wave;
  if (m >= M) return;
  uint32_t mx = 0;
  for (int k0 = lane * 16; k0 < K; k0 += kWave * 16) {               // K % 16 == 0: whole pieces
    const v4u f = flags16(flag, k0);
    const v4u a = *reinterpret_cast<const v4u*>(X + (size_t)m * ldx + k0);
    const v4u b = *reinterpret_cast<const v4u*>(X + (size_t)m * ldx + k0 + 8);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      // flag bytes 2 w' and 2 w' + 1 of the piece belong to the two halves of word w' (a: columns 0..7, b: 8..15)
      const uint32_t fa = f[w >> 1] >> (16 * (w & 1)), fb = f[2 + (w >> 1)] >> (16 * (w & 1));
      const uint32_t keep_a = ((fa & 1u) ? 0u : 0x7fffu) | ((fa & 0x100u) ? 0u : 0x7fff0000u);
      const uint32_t keep_b = ((fb & 1u) ? 0u : 0x7fffu) | ((fb & 0x100u) ? 0u : 0x7fff0000u);
      const uint32_t va = a[w] & keep_a, vb = b[w] & keep_b;
      mx = max(mx, max(max(va & 0xffffu, va >> 16), max(vb & 0xffffu, vb >> 16)));
    }
  }
  mx = wave_max_u32(mx);
  if (lane == 0) r_out[m] = half_lo_to_float(mx);                    // fp16 magnitudes order like their patterns
}

// ------------------------------------------------------------------ pack
// Xq in the blocked operand layout (operand_layout.h): codes of the non-critical columns, zeros
// in the critical columns and in the K padding.  A wave converts 32 rows x one 64-byte slab per
// step and writes it as two runs of 1 KB (the two half slabs, fragment-major): lane = (row, 16-byte
// piece of the half slab).  Its input per half slab is 32 bytes of one row of X; the two lanes of a
// row read 64 contiguous bytes, and the two half slabs make up one 128-byte line.  The lane's
// column flags are turned into byte masks once and reused for kPackRowSteps groups of 32 rows.
constexpr int kPackRowSteps = 2;
constexpr int kPackRows = 32 * kPackRowSteps;          // rows per workgroup
constexpr int kPackSlabs = kThreads / kWave;            // slabs per workgroup (one per wave)

constexpr int kListedColumns = kOutlierSlab * kCriticalSlabs + kGatherMax;   // critical columns a workgroup keeps in LDS

// The ascending list of critical columns and their count, computed by one whole workgroup from
// the flags (every workgroup that needs the list recomputes it: a few KB of flags from L2 are
// cheaper than a serial step between two kernels).  The first kOutlierSlab indices and the count
// land in LDS; the workgroup with `publish` also writes the list, the count, the byte mask and
// the taps to global memory.  Each thread owns a contiguous run of 16-column units.
template <int kMaxUnits>   // units a thread may own: ceil(Kpad / 16 / kThreads) at most
__device__ __forceinline__ void compact_critical_columns_n(const uint8_t* __restrict__ flag, int K, int Kpad,
                                                           const PackOutliers& o, bool publish,
                                                           int* s_idx /*[kListedColumns]*/, int* s_n_out,
                                                           int* s_wave_total /*[kThreads / kWave]*/) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int units = Kpad / 16;
  const int per = ceil_div(units, kThreads);
  const int u_begin = min(units, (int)threadIdx.x * per);
  v4u f[kMaxUnits];
  int cnt = 0;
#pragma unroll
  for (int i = 0; i < kMaxUnits; ++i) {
    // unconditional loads (a unit past the thread's run re-reads unit 0 and is masked): all in flight together
    const bool mine = i < per && u_begin + i < units;
    f[i] = flags16(flag, mine ? 16 * (u_begin + i) : 0) & (mine ? 0xffffffffu : 0u);
  }
#pragma unroll
  for (int i = 0; i < kMaxUnits; ++i) {
#pragma unroll
    for (int w = 0; w < 4; ++w) cnt += __builtin_popcount(f[i][w]);
  }
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
#pragma unroll
  for (int i = 0; i < kMaxUnits; ++i) {
    if (i < per && u_begin + i < units) {
      const int u = u_begin + i;
      if (publish) reinterpret_cast<v4u*>(o.mask)[u] = f[i];
      if ((f[i][0] | f[i][1] | f[i][2] | f[i][3]) || (publish && o.tap_mask)) {
        for (int t = 0; t < 16; ++t) {
          const int k = 16 * u + t;
          const bool set = (f[i][t >> 2] >> (8 * (t & 3))) & 1u;
          if (publish && o.tap_mask && k < K) o.tap_mask[k] = set ? 1 : 0;
          if (set) {
            if (pos < kOutlierSlab * (o.crit_slabs + (o.Xg ? o.g_slabs : 0))) s_idx[pos] = k;
            if (publish) {
              o.idx[pos] = k;
              if (o.tap_idx) o.tap_idx[pos] = k;
            }
            ++pos;
          }
        }
      }
    }
  }
  if (threadIdx.x == kThreads - 1) {
    *s_n_out = before + incl;
    if (publish) {
      *o.n_out = before + incl;
      if (o.tap_n) *o.tap_n = before + incl;
    }
  }
  __syncthreads();
}

// (a thread's loads are all issued whether it owns that many units or not, so the count is a template argument)
__device__ __forceinline__ void compact_critical_columns(const uint8_t* __restrict__ flag, int K, int Kpad,
                                                         const PackOutliers& o, bool publish, int* s_idx, int* s_n_out,
                                                         int* s_wave_total) {
  static_assert(MMD8_MAX_K / 16 / kThreads == 16, "largest number of units per thread");
  const int per = ceil_div(Kpad / 16, kThreads);
  if (per <= 2) compact_critical_columns_n<2>(flag, K, Kpad, o, publish, s_idx, s_n_out, s_wave_total);
  else if (per <= 8) compact_critical_columns_n<8>(flag, K, Kpad, o, publish, s_idx, s_n_out, s_wave_total);
  else compact_critical_columns_n<16>(flag, K, Kpad, o, publish, s_idx, s_n_out, s_wave_total);
}

// Rows of the critical-column slabs, 8 columns (16 bytes) per thread and slab: Xo[m][j] = X[m, O_j] for
// the first kOutlierSlab * crit_slabs critical columns and Wo[n][j] = f16(Wt[n, O_j] c[n] / 127); zero for
// j >= n_out.  The weights are dequantized with two roundings (fp32 product, then fp16).  Each group of 32
// columns is stored like one slab of a packed operand; slab 0 is always written (zeros without critical
// columns), slab s > 0 only when more than 32 s columns are critical (the GEMM reads no other).
// (slab `slab` of the list goes to slab `dst_slab` of dstX / dstW, which hold dst_slabs slabs per panel)
__device__ inline void gather_outlier_slab_one(const uint16_t* __restrict__ X, int M, int ldx, int n_slabs,
                                               const PackOutliers& o, int row, int ch, int slab, const int* s_idx,
                                               int n_out, uint16_t* dstX, uint16_t* dstW, int dst_slabs, int dst_slab);
__device__ inline void gather_outlier_slab(const uint16_t* __restrict__ X, int M, int ldx, int n_slabs,
                                           const PackOutliers& o, int item, const int* s_idx, int n_out_all) {
  const int row = item / (kOutlierSlab / 8), ch = item % (kOutlierSlab / 8);
  if (row >= M + o.N) return;
  if (dense_critical_path(n_out_all, o.crit_slabs, o.dense_from, o.W_master != nullptr)) return;   // the GEMM reads no slab then
  const int n_out = min(n_out_all, kOutlierSlab * o.crit_slabs);
  const int used = max(1, ceil_div(n_out, kOutlierSlab));
  for (int slab = 0; slab < used; ++slab)
    gather_outlier_slab_one(X, M, ldx, n_slabs, o, row, ch, slab, s_idx, n_out, o.Xo, o.Wo, o.f_slabs, slab);
}
// The critical columns beyond those slabs, as further slabs of the same layout in Xg / Wg (gemm.h): the slabs in use
// shared out over all the threads that build slabs.  Nothing to do in the usual case (no such column), and nothing
// when the GEMM takes the dense pass.
__device__ inline void gather_further_slabs(const uint16_t* __restrict__ X, int M, int ldx, int n_slabs,
                                            const PackOutliers& o, int first, int stride, const int* s_idx, int n_out_all) {
  if (o.Xg == nullptr || dense_critical_path(n_out_all, o.crit_slabs, o.dense_from, o.W_master != nullptr)) return;
  const int n_out = min(n_out_all, kOutlierSlab * (o.crit_slabs + o.g_slabs));
  const int more = ceil_div(n_out, kOutlierSlab) - o.crit_slabs;
  if (more <= 0) return;
  const int per_slab = (M + o.N) * (kOutlierSlab / 8);
  for (int item = first; item < more * per_slab; item += stride) {
    const int g = item / per_slab, rest = item % per_slab;
    gather_outlier_slab_one(X, M, ldx, n_slabs, o, rest / (kOutlierSlab / 8), rest % (kOutlierSlab / 8), o.crit_slabs + g, s_idx,
                            n_out, o.Xg, o.Wg, o.g_slabs, g);
  }
}
__device__ inline void gather_outlier_slab_one(const uint16_t* __restrict__ X, int M, int ldx, int n_slabs,
                                               const PackOutliers& o, int row, int ch, int slab, const int* s_idx,
                                               int n_out, uint16_t* dstX, uint16_t* dstW, int dst_slabs, int dst_slab) {
  const int j0 = slab * kOutlierSlab + ch * 8;
  // all eight loads of a thread are issued together: a missing column re-reads column 0 and is masked
  int kcol[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) kcol[t] = (j0 + t < n_out) ? s_idx[j0 + t] : -1;
  uint32_t out[4] = {0, 0, 0, 0};
  if (row < M) {
    uint16_t v[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = X[(size_t)row * ldx + max(kcol[t], 0)];
#pragma unroll
    for (int t = 0; t < 8; ++t) out[t >> 1] |= (kcol[t] >= 0 ? (uint32_t)v[t] : 0u) << (16 * (t & 1));
    *reinterpret_cast<v4u*>(reinterpret_cast<int8_t*>(dstX) + packed_chunk_offset(row, dst_slab, ch, dst_slabs)) =
        v4u{out[0], out[1], out[2], out[3]};
  } else {
    const int n = row - M;
    if (o.W_master) {
      // the original 16-bit rows of the critical dimensions, as they are
      uint16_t w[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) w[t] = o.W_master[(size_t)max(kcol[t], 0) * o.ldw + n];
#pragma unroll
      for (int t = 0; t < 8; ++t) out[t >> 1] |= (kcol[t] >= 0 ? (uint32_t)w[t] : 0u) << (16 * (t & 1));
    } else {
      const float step = o.c[n] / 127.0f;
      int8_t q[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) q[t] = o.Wt[packed_offset(n, max(kcol[t], 0), n_slabs)];
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const uint32_t h = rounded_float_to_half_bits((float)q[t] * step);
        out[t >> 1] |= (kcol[t] >= 0 ? h : 0u) << (16 * (t & 1));
      }
    }
    *reinterpret_cast<v4u*>(reinterpret_cast<int8_t*>(dstW) + packed_chunk_offset(n, dst_slab, ch, dst_slabs)) =
        v4u{out[0], out[1], out[2], out[3]};
  }
}

__global__ __launch_bounds__(kThreads) void k_pack(const uint16_t* __restrict__ X, int M, int K, int ldx,
                                                   const uint8_t* __restrict__ flag,
                                                   const float* __restrict__ r, int8_t* __restrict__ Xq,
                                                   int n_slabs, int8_t* __restrict__ tap_xq, int pack_blocks_y,
                                                   uint16_t* __restrict__ Xf, const PackOutliers o) {
  if ((int)blockIdx.y >= pack_blocks_y) {
    // the extra blocks list the critical columns and prepare their slab; the first one publishes
    __shared__ int s_idx[kListedColumns];
    __shared__ int s_n_out;
    __shared__ int s_wave_total[kThreads / kWave];
    const int b = ((int)blockIdx.y - pack_blocks_y) * gridDim.x + blockIdx.x;
    compact_critical_columns(flag, K, n_slabs * kSlabBytes, o, b == 0, s_idx, &s_n_out, s_wave_total);
    if (!Xf) {
      gather_outlier_slab(X, M, ldx, n_slabs, o, b * kThreads + threadIdx.x, s_idx, s_n_out);
      gather_further_slabs(X, M, ldx, n_slabs, o, b * kThreads + threadIdx.x,
                             ((int)gridDim.y - pack_blocks_y) * (int)gridDim.x * kThreads, s_idx, s_n_out);
    }
    return;
  }
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int slab = blockIdx.x * kPackSlabs + wave;
  if (slab >= n_slabs) return;
  const int rl = lane & 31, g = lane >> 5;
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int ch = 2 * ks + g;
    const int k0 = slab * kSlabBytes + ch * 16;
    const bool in_k = k0 < K;                         // K % 16 == 0: a piece is all inside or all padding
    uint32_t keep[4] = {0, 0, 0, 0};                  // 0xff per kept byte
    if (in_k) {
      const v4u f = flags16(flag, k0);
#pragma unroll
      for (int w = 0; w < 4; ++w) keep[w] = (0x01010101u - f[w]) * 0xffu;   // bytes are 0 or 1: no carries
    }
    const int m0 = blockIdx.y * kPackRows + rl;
    v4u a[kPackRowSteps], b[kPackRowSteps];
    float rm[kPackRowSteps];
#pragma unroll
    for (int i = 0; i < kPackRowSteps; ++i) {
      const int m = m0 + i * 32;
      a[i] = b[i] = v4u{0, 0, 0, 0};
      rm[i] = 0.0f;
      if (m < M && in_k) {
        a[i] = *reinterpret_cast<const v4u*>(X + (size_t)m * ldx + k0);
        b[i] = *reinterpret_cast<const v4u*>(X + (size_t)m * ldx + k0 + 8);
        rm[i] = r[m];
      }
    }
#pragma unroll
    for (int i = 0; i < kPackRowSteps; ++i) {
      const int m = m0 + i * 32;
      if (m >= M) break;
      const float scale = (rm[i] == 0.0f) ? 0.0f : 127.0f / rm[i];   // IEEE division
      uint32_t out[4];
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        out[w] = to_code_byte(half_lo_to_float(a[i][2 * w]), scale) |
                 (to_code_byte(half_hi_to_float(a[i][2 * w]), scale) << 8) |
                 (to_code_byte(half_lo_to_float(a[i][2 * w + 1]), scale) << 16) |
                 (to_code_byte(half_hi_to_float(a[i][2 * w + 1]), scale) << 24);
        out[2 + w] = to_code_byte(half_lo_to_float(b[i][2 * w]), scale) |
                     (to_code_byte(half_hi_to_float(b[i][2 * w]), scale) << 8) |
                     (to_code_byte(half_lo_to_float(b[i][2 * w + 1]), scale) << 16) |
                     (to_code_byte(half_hi_to_float(b[i][2 * w + 1]), scale) << 24);
      }
#pragma unroll
      for (int w = 0; w < 4; ++w) out[w] &= keep[w];
      const v4u v = v4u{out[0], out[1], out[2], out[3]};
      *reinterpret_cast<v4u*>(Xq + packed_chunk_offset(m, slab, ch, n_slabs)) = v;
      if (tap_xq && in_k) *reinterpret_cast<v4u*>(tap_xq + (size_t)m * K + k0) = v;
      if (Xf) {
        // decode path: the critical columns of X as fp16, everything else (K padding included) zero
        uint32_t fa[4], fb[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          // ~keep[] has 0xff per critical column byte; the fp16 pair w of a[] covers columns 2w, 2w+1
          const uint32_t ca = (~keep[w >> 1]) >> (16 * (w & 1)), cb = (~keep[2 + (w >> 1)]) >> (16 * (w & 1));
          const uint32_t ma = ((ca & 0xffu) * 0x0101u) | (((ca >> 8) & 0xffu) * 0x01010000u);
          const uint32_t mb = ((cb & 0xffu) * 0x0101u) | (((cb >> 8) & 0xffu) * 0x01010000u);
          fa[w] = in_k ? (a[i][w] & ma) : 0u;
          fb[w] = in_k ? (b[i][w] & mb) : 0u;
        }
        int8_t* xf_bytes = reinterpret_cast<int8_t*>(Xf);
        *reinterpret_cast<v4u*>(xf_bytes + xf_group_offset(m, k0)) = v4u{fa[0], fa[1], fa[2], fa[3]};
        *reinterpret_cast<v4u*>(xf_bytes + xf_group_offset(m, k0 + 8)) = v4u{fb[0], fb[1], fb[2], fb[3]};
      }
    }
  }
}

// ------------------------------------------------------------------ one-pass preparation (tall inputs)
// Scan and quantization in a single pass over X: a workgroup holds four whole rows in registers,
// finds their scales and the columns that reach the threshold, and writes the codes of every
// column straight away.  Which columns are critical is only known once every row has been seen,
// so the codes of critical columns are cleared afterwards by k_outlier_columns (a few bytes per
// row); X is read once and the codes written once: 3 bytes per element instead of 5.
//
// Lane l of a wave owns row (l % 4) of the workgroup's four rows and, in pass q, the 16-column
// piece 16 (q kWaves + wave) + l / 4 of that row: a load instruction reads 512 contiguous bytes of
// each of four rows, and a store instruction writes 64-byte runs (the four rows of a piece are
// neighbours in the blocked layout).
//
// kFromCodes: the activations arrive as a blockwise-coded hidden state ("Compression techniques",
// item 1: codes + per-block absmax, contiguous [M][K]).  The kernel decodes them first, exactly as
// the decoder does (f16(T[code] * absmax), fp32 product, then round), writes the fp16 values to X
// (which is then an output: the decoded hidden state, ldx = K) and carries on with them.
//
// Workgroups go to the eight XCDs in turn (workgroup b to XCD b % 8), each with an L2 of its own, and the 16-byte
// pieces of 32 neighbouring rows are 512 contiguous bytes of the blocked codes: the eight row quads of such a
// group are given to one XCD (workgroups b, b + 8, ..., b + 56, dispatched one after the other), so that its L2
// sees whole 128-byte lines instead of halves that two XCDs write separately.
__device__ inline int row_quad_of_block(int b, int n_blocks) {
  if (b >= (n_blocks & ~63)) return b;                      // a last partial chunk of 64 keeps its order
  return (b & ~63) | ((b & 7) << 3) | ((b >> 3) & 7);
}

template <int kWaves, int kPasses, bool kFromCodes>
__global__ __launch_bounds__(kWaves * kWave) void k_prep(uint16_t* __restrict__ X, int M, int K, int ldx, uint32_t th,
                                                         int n_slabs, uint8_t* __restrict__ flag,
                                                         float* __restrict__ r_out, int8_t* __restrict__ Xq,
                                                         int8_t* __restrict__ tap_xq, const CodedInput coded) {
  __shared__ uint32_t s_part[kWaves][4];
  __shared__ float s_T[kFromCodes ? 256 : 1];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int j = lane & 3, i = lane >> 2;
  const int m = row_quad_of_block(blockIdx.x, gridDim.x) * 4 + j;
  const bool row_ok = m < M;
  const int Kpad = n_slabs * kSlabBytes;
  const int n_pieces = Kpad / 16, k_pieces = K / 16;
  const us2 th2 = as_us2(th | (th << 16));

  // every load is unconditional (a lane without data re-reads the first piece of row 0, and what
  // it derives from that is discarded), so that all of them are in flight together
  v4u a[kPasses], b[kPasses];
  if constexpr (!kFromCodes) {
#pragma unroll
    for (int q = 0; q < kPasses; ++q) {
      const int piece = (q * kWaves + wave) * 16 + i;
      const bool ok = row_ok && piece < k_pieces;
      const uint16_t* src = X + (ok ? (size_t)m * ldx + piece * 16 : (size_t)0);
      a[q] = *reinterpret_cast<const v4u*>(src);
      b[q] = *reinterpret_cast<const v4u*>(src + 8);
    }
  } else {
    v4u cq[kPasses];
    float sc[kPasses];
#pragma unroll
    for (int q = 0; q < kPasses; ++q) {
      const int piece = (q * kWaves + wave) * 16 + i;
      const bool ok = row_ok && piece < k_pieces;
      const uint32_t e0 = ok ? (uint32_t)m * (uint32_t)K + piece * 16 : 0u;   // a piece lies inside one block
      cq[q] = *reinterpret_cast<const v4u*>(coded.codes + e0);
      sc[q] = coded.absmax[e0 / (uint32_t)coded.block];
    }
    for (int t = threadIdx.x; t < 256; t += kWaves * kWave) s_T[t] = kCodeValuesDev.v[t];
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kPasses; ++q) {
      const int piece = (q * kWaves + wave) * 16 + i;
      uint32_t h[8];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t cw = cq[q][w];
        h[2 * w] = rounded_float_to_half_bits(s_T[cw & 0xffu] * sc[q]) | (rounded_float_to_half_bits(s_T[(cw >> 8) & 0xffu] * sc[q]) << 16);
        h[2 * w + 1] = rounded_float_to_half_bits(s_T[(cw >> 16) & 0xffu] * sc[q]) | (rounded_float_to_half_bits(s_T[cw >> 24] * sc[q]) << 16);
      }
      a[q] = v4u{h[0], h[1], h[2], h[3]};
      b[q] = v4u{h[4], h[5], h[6], h[7]};
      if (row_ok && piece < k_pieces) {
        uint16_t* dst = X + (size_t)m * ldx + piece * 16;
        *reinterpret_cast<v4u*>(dst) = a[q];
        *reinterpret_cast<v4u*>(dst + 8) = b[q];
      }
    }
  }

  // ---- row scale and column flags (packed 16-bit compares, see the top of the file)
  us2 rowt = as_us2(0u);
#pragma unroll
  for (int q = 0; q < kPasses; ++q) {
    const int piece = (q * kWaves + wave) * 16 + i;
    uint32_t t_and = 0xffffffffu;
    us2 t_max = as_us2(0u);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const us2 t0 = as_us2(a[q][w] & 0x7fff7fffu) - th2, t1 = as_us2(b[q][w] & 0x7fff7fffu) - th2;
      t_max = __builtin_elementwise_max(t_max, __builtin_elementwise_max(t0, t1));
      t_and &= as_u32(t0) & as_u32(t1);
    }
    if (row_ok && piece < k_pieces) rowt = __builtin_elementwise_max(rowt, t_max);
    {
      // evaluate now: left alone, the compiler keeps all differences of every piece until after the loop
      uint32_t pin = as_u32(rowt);
      asm volatile("" : "+v"(pin));
      rowt = as_us2(pin);
    }
    const bool hit = row_ok && piece < k_pieces && ((~t_and) & 0x80008000u);
    if (__builtin_amdgcn_ballot_w64(hit)) {                 // rare for prefill-like inputs
      // one bit per column of the piece that reaches the threshold in this row, then over the
      // four rows of the quad; the quad's first lane publishes what is not yet known
      uint32_t bits = 0;
      if (hit) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          // plain magnitude compares here: sharing the packed differences of the common path with
          // this rare one would keep them in registers for every piece
          bits |= (uint32_t)((a[q][w] & 0x7fffu) >= th) << (2 * w) | (uint32_t)(((a[q][w] >> 16) & 0x7fffu) >= th) << (2 * w + 1);
          bits |= (uint32_t)((b[q][w] & 0x7fffu) >= th) << (8 + 2 * w) | (uint32_t)(((b[q][w] >> 16) & 0x7fffu) >= th) << (9 + 2 * w);
        }
      }
      bits |= (uint32_t)__builtin_amdgcn_mov_dpp((int)bits, 0xb1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]
      bits |= (uint32_t)__builtin_amdgcn_mov_dpp((int)bits, 0x4e, 0xf, 0xf, true);   // quad_perm [2,3,0,1]
      if (j == 0) {
        // plain byte stores of 1: every writer stores the same value, nobody reads before the
        // kernel ends, and nothing is waited for
        uint8_t* fb = flag + piece * 16;
        while (bits) {
          fb[__builtin_ctz(bits)] = 1;
          bits &= bits - 1;
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);                    // one piece at a time: bounded registers
  }
  uint32_t mx = max(as_u32(rowt) & 0xffffu, as_u32(rowt) >> 16);
#pragma unroll
  for (int d = 4; d < kWave; d <<= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, d, kWave));
  if (lane < 4) s_part[wave][lane] = mx;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kWaves; ++w) mx = max(mx, s_part[w][j]);
  // top bit set: a sub-threshold entry exists and its pattern is mx + th (mod 2^16)
  const float r = (mx & 0x8000u) ? half_lo_to_float((mx + th) & 0xffffu) : 0.0f;
  if (threadIdx.x < 4 && row_ok) r_out[m] = r;
  const float scale = (r == 0.0f) ? 0.0f : 127.0f / r;            // IEEE division

  // ---- codes of every column (critical ones are cleared later); K padding gets zeros
  if (!row_ok) return;
#pragma unroll
  for (int q = 0; q < kPasses; ++q) {
    int piece = (q * kWaves + wave) * 16 + i;
    // keeps the address arithmetic and the fp16 -> fp32 conversions of this piece here (hoisted above
    // the barrier they would double the registers)
    asm volatile("" : "+v"(piece), "+v"(a[q]), "+v"(b[q]));
    if (piece >= n_pieces) break;
    uint32_t out[4];
#pragma unroll
    for (int w = 0; w < 2; ++w) {
      out[w] = to_code_byte(half_lo_to_float(a[q][2 * w]), scale) | (to_code_byte(half_hi_to_float(a[q][2 * w]), scale) << 8) |
               (to_code_byte(half_lo_to_float(a[q][2 * w + 1]), scale) << 16) |
               (to_code_byte(half_hi_to_float(a[q][2 * w + 1]), scale) << 24);
      out[2 + w] = to_code_byte(half_lo_to_float(b[q][2 * w]), scale) | (to_code_byte(half_hi_to_float(b[q][2 * w]), scale) << 8) |
                   (to_code_byte(half_lo_to_float(b[q][2 * w + 1]), scale) << 16) |
                   (to_code_byte(half_hi_to_float(b[q][2 * w + 1]), scale) << 24);
    }
    const uint32_t in_k = piece < k_pieces ? 0xffffffffu : 0u;     // the K padding holds zeros
    const v4u v = v4u{out[0] & in_k, out[1] & in_k, out[2] & in_k, out[3] & in_k};
    *reinterpret_cast<v4u*>(Xq + packed_chunk_offset(m, piece >> 2, piece & 3, n_slabs)) = v;
    if (tap_xq && piece < k_pieces) *reinterpret_cast<v4u*>(tap_xq + (size_t)m * K + piece * 16) = v;
    __builtin_amdgcn_sched_barrier(0);                    // one piece at a time: bounded registers
  }
}

// After k_prep: the first `slab_blocks` workgroups list the critical columns (the first one
// publishes the list, the count and the byte mask) and build the fp16 slab of the first
// kOutlierSlab of them; each of the remaining workgroups owns 64 rows (lane = row) and 4096 columns or a multiple
// and clears the codes of the critical columns in those rows with byte stores of zero.  Driven by the
// flags themselves, so any number of critical columns is handled the same way.
__global__ __launch_bounds__(kThreads) void k_outlier_columns(const uint16_t* __restrict__ X, int M, int K, int ldx,
                                                              const uint8_t* __restrict__ flag, int8_t* __restrict__ Xq,
                                                              int n_slabs, int8_t* __restrict__ tap_xq, int slab_blocks,
                                                              int clear_units, const PackOutliers o) {
  const int Kpad = n_slabs * kSlabBytes;
  if ((int)blockIdx.x < slab_blocks) {
    __shared__ int s_idx[kListedColumns];
    __shared__ int s_n_out;
    __shared__ int s_wave_total[kThreads / kWave];
    compact_critical_columns(flag, K, Kpad, o, blockIdx.x == 0, s_idx, &s_n_out, s_wave_total);
    gather_outlier_slab(X, M, ldx, n_slabs, o, blockIdx.x * kThreads + threadIdx.x, s_idx, s_n_out);
    gather_further_slabs(X, M, ldx, n_slabs, o, blockIdx.x * kThreads + threadIdx.x, slab_blocks * kThreads, s_idx, s_n_out);
    return;
  }
  // A clearing workgroup owns 64 rows (lane = row) and clear_units units of 16 columns (a multiple of 64), a quarter
  // of them per wave, taken 64 at a time: lane l of a wave looks at unit u0 + l.  (With input whose columns are
  // nearly all critical the clearing is the longest part of the preparation unless many waves share a row.)
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int units = Kpad / 16;
  const int unit_groups = ceil_div(units, clear_units);
  const int cb = (int)blockIdx.x - slab_blocks;
  const int m = (cb / unit_groups) * kWave + lane;
  const int wave_units = clear_units / (kThreads / kWave);
  const int u_begin = (cb % unit_groups) * clear_units + wave * wave_units;
  const int u_end = min(units, u_begin + wave_units);
  for (int u0 = u_begin; u0 < u_end; u0 += kWave) {
    const v4u f = u0 + lane < u_end ? flags16(flag, 16 * (u0 + lane)) : v4u{0, 0, 0, 0};
    uint64_t todo = __builtin_amdgcn_ballot_w64((f[0] | f[1] | f[2] | f[3]) != 0);
    while (todo) {
      const int t = __builtin_ctzll(todo);
      todo &= todo - 1;
      const int unit = u0 + t;
      // the flagged columns of this unit, one bit each (the same for every lane)
      uint32_t cols = 0;
      v4u keep;                                                       // 0xff per column that stays
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t fw = (uint32_t)__builtin_amdgcn_readlane((int)f[w], t);
        cols |= ((fw & 1u) | ((fw >> 7) & 2u) | ((fw >> 14) & 4u) | ((fw >> 21) & 8u)) << (4 * w);
        keep[w] = (0x01010101u - fw) * 0xffu;                         // flag bytes are 0 or 1: no carries
      }
      if (m < M) {
        int8_t* p = Xq + packed_chunk_offset(m, unit >> 2, unit & 3, n_slabs);
        int8_t* tp = tap_xq ? tap_xq + (size_t)m * K + unit * 16 : nullptr;
        if (__builtin_popcount(cols) >= 4) {
          // many of the unit's 16 columns (heavy-tailed input): the row's 16 bytes are read, masked and written back
          // (they are this lane's alone) instead of a byte store per column
          *reinterpret_cast<v4u*>(p) = *reinterpret_cast<const v4u*>(p) & keep;
          if (tp) *reinterpret_cast<v4u*>(tp) = *reinterpret_cast<const v4u*>(tp) & keep;
          continue;
        }
        while (cols) {
          const int c = __builtin_ctz(cols);
          cols &= cols - 1;
          p[c] = 0;
          if (tp) tp[c] = 0;
        }
      }
    }
  }
}

// ------------------------------------------------------------------ launchers
hipError_t launch_fill_u32(uint32_t* p, uint32_t v, int n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_fill_u32, dim3(ceil_div(n, 256)), dim3(256), 0, stream, p, v, n);
  return hipGetLastError();
}

hipError_t launch_scan(const uint16_t* X, int M, int K, int ldx, uint32_t th, int Kpad, uint8_t* flag, float* r,
                       hipStream_t stream) {
  const int want = 2 * device_cu_count();                // workgroups
  if (M >= 4 * want)
    hipLaunchKernelGGL(k_scan<4>, dim3(ceil_div(M, 4)), dim3(kThreads), 0, stream, X, M, K, ldx, th, Kpad, flag, r);
  else if (M >= 2 * want)
    hipLaunchKernelGGL(k_scan<2>, dim3(ceil_div(M, 2)), dim3(kThreads), 0, stream, X, M, K, ldx, th, Kpad, flag, r);
  else
    hipLaunchKernelGGL(k_scan<1>, dim3(M), dim3(kThreads), 0, stream, X, M, K, ldx, th, Kpad, flag, r);
  return hipGetLastError();
}

hipError_t launch_row_absmax_noncritical(const uint16_t* X, int M, int K, int ldx, const uint8_t* flag, float* r,
                                         hipStream_t stream) {
  hipLaunchKernelGGL(k_row_absmax_noncritical, dim3(ceil_div(M, kThreads / kWave)), dim3(kThreads), 0, stream, X, M, K, ldx, flag, r);
  return hipGetLastError();
}

hipError_t launch_pack(const uint16_t* X, int M, int K, int ldx, const uint8_t* flag, const float* r, int8_t* Xq,
                       int Kpad, int8_t* tap_xq, uint16_t* Xf, const PackOutliers& o, hipStream_t stream, bool list_columns) {
  const int n_slabs = Kpad / kSlabBytes;
  const int gx = ceil_div(n_slabs, kPackSlabs), pack_y = ceil_div(M, kPackRows);
  // the slabs of critical columns are for the tiled GEMM kernels; the decode kernel reads Xf instead
  // (one extra block still lists the critical columns)
  const int slab_items = Xf ? 0 : (M + o.N) * (kOutlierSlab / 8);
  // (the list is a chain of dependent steps over all of K in one workgroup: the longest part of this kernel at
  // decode sizes; the decode kernels can read the flags themselves)
  if (!list_columns && !Xf) return hipErrorInvalidValue;
  const int slab_y = list_columns ? max(1, ceil_div(ceil_div(slab_items, kThreads), gx)) : 0;
  const dim3 grid(gx, pack_y + slab_y);
  hipLaunchKernelGGL(k_pack, grid, dim3(kThreads), 0, stream, X, M, K, ldx, flag, r, Xq, n_slabs, tap_xq, pack_y, Xf, o);
  return hipGetLastError();
}

bool prep_fits(int K) { return packed_k(K) / 16 <= 16 * 16 * 8; }
// the variant that decodes coded activations holds more per lane: rows up to 16384 columns without spilling
bool prep_from_codes_fits(int K) { return packed_k(K) / 16 <= 16 * 16 * 4; }

hipError_t launch_prep(uint16_t* X, int M, int K, int ldx, uint32_t th, int Kpad, uint8_t* flag, float* r,
                       int8_t* Xq, int8_t* tap_xq, const PackOutliers& o, const CodedInput* coded, void* event_mid,
                       hipStream_t stream) {
  const int n_slabs = Kpad / kSlabBytes, n_pieces = Kpad / 16;
  const dim3 grid(ceil_div(M, 4));
  const CodedInput ci = coded ? *coded : CodedInput{};
#define MMD8_PREP(W_, P_)                                                                                                \
  do {                                                                                                                   \
    if (coded)                                                                                                           \
      hipLaunchKernelGGL((k_prep<W_, P_, true>), grid, dim3(W_ * kWave), 0, stream, X, M, K, ldx, th, n_slabs, flag, r, \
                         Xq, tap_xq, ci);                                                                                \
    else                                                                                                                 \
      hipLaunchKernelGGL((k_prep<W_, P_, false>), grid, dim3(W_ * kWave), 0, stream, X, M, K, ldx, th, n_slabs, flag, r, \
                         Xq, tap_xq, ci);                                                                                \
  } while (0)
  if (n_pieces <= 64) MMD8_PREP(4, 1);
  else if (n_pieces <= 128) MMD8_PREP(4, 2);
  else if (n_pieces <= 256) MMD8_PREP(4, 4);
  else if (n_pieces <= 512) MMD8_PREP(8, 4);
  else if (n_pieces <= 1024) MMD8_PREP(16, 4);
  else if (coded) return hipErrorInvalidValue;                     // the caller decodes first (prep_from_codes_fits)
  else hipLaunchKernelGGL((k_prep<16, 8, false>), grid, dim3(16 * kWave), 0, stream, X, M, K, ldx, th, n_slabs, flag, r, Xq,
                          tap_xq, ci);
#undef MMD8_PREP
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (event_mid && (e = hipEventRecord(static_cast<hipEvent_t>(event_mid), stream)) != hipSuccess) return e;
  const int slab_blocks = max(1, ceil_div((M + o.N) * (kOutlierSlab / 8), kThreads));
  // clearing workgroups: 64 rows x 4096 columns each, more columns each once that would be more than one per four
  // CUs (with few critical columns, the usual case, a workgroup has next to nothing to do and their number is the
  // cost: 17.1 us with 256 of them against 12.7 us with 16 on a 4096 x 28672 input)
  const int row_groups = ceil_div(M, kWave), units = n_slabs * (kSlabBytes / 16);
  const int groups_256 = row_groups * ceil_div(units, kThreads);
  const int merge = max(1, ceil_div(groups_256, max(1, device_cu_count() / 4)));
  // (a few hundred rows: a quarter of that per workgroup, 16 units per wave, so that heavy-tailed input, where every
  // unit has columns to clear, does not leave the clearing to four workgroups)
  const int clear_units = groups_256 <= 16 ? kThreads / 4 : kThreads * merge;
  const int clear_blocks = row_groups * ceil_div(units, clear_units);
  hipLaunchKernelGGL(k_outlier_columns, dim3(slab_blocks + clear_blocks), dim3(kThreads), 0, stream, X, M, K, ldx, flag, Xq,
                     n_slabs, tap_xq, slab_blocks, clear_units, o);
  return hipGetLastError();
}

}  // namespace mmd8
