// Shared host/device helpers for the mmd8 library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/mmd8.h"

namespace mmd8 {

constexpr int kWave = 64;

typedef int      v4i  __attribute__((ext_vector_type(4)));
typedef int      v2i  __attribute__((ext_vector_type(2)));
typedef int      v16i __attribute__((ext_vector_type(16)));
typedef float    v16f __attribute__((ext_vector_type(16)));
typedef float    v4f  __attribute__((ext_vector_type(4)));
typedef _Float16 v8h  __attribute__((ext_vector_type(8)));
typedef _Float16 v2h  __attribute__((ext_vector_type(2)));
typedef uint32_t v4u  __attribute__((ext_vector_type(4)));
typedef uint32_t v2u  __attribute__((ext_vector_type(2)));

__host__ __device__ constexpr inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ constexpr inline int round_up(int a, int b) { return ceil_div(a, b) * b; }
__host__ __device__ constexpr inline size_t round_up_sz(size_t a, size_t b) { return (a + b - 1) / b * b; }

// fp16 bit pattern -> fp32 (exact).  The low/high halves of a packed dword.
__device__ inline float half_lo_to_float(uint32_t w) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu));
}
__device__ inline float half_hi_to_float(uint32_t w) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
}
// fp32 -> fp16 bit pattern, round to nearest even.
__device__ inline uint32_t float_to_half_bits(float f) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
}
// Same, for a value that must first exist as a rounded fp32 number.  Without the empty asm the
// compiler folds "multiply, then convert" into v_fma_mixlo_f16, which rounds the exact product
// once; the definition of the codec and of the fp16 weights rounds twice (fp32, then fp16).
__device__ inline uint32_t rounded_float_to_half_bits(float f) {
  asm("" : "+v"(f));
  return float_to_half_bits(f);
}

// activation value -> int8 code (as an unsigned byte) with the row's scale 127 / r: round to nearest even, clamp
__device__ inline uint32_t to_code_byte(float x, float scale) {
  float q = __builtin_rintf(x * scale);
  q = fminf(fmaxf(q, -127.0f), 127.0f);
  return (uint32_t)((int)q) & 0xffu;
}

// Exact GELU, x Phi(x), of an fp16 value given as fp32; fp16 bit pattern of the result.  Branch-free:
//   Phi(-|x|) = erfc(z) / 2, z = |x| / sqrt 2,   erfc(z) = t exp(-z^2 + g(t)), t = 1 / (1 + z / 2),
// with g a degree-8 polynomial fitted to ln(exp(z^2) erfc(z) / t) on the t range of |x| <= 13.5 (beyond that the
// result is below the smallest fp16 number); Phi(|x|) = 1 - Phi(-|x|).  Relative error of Phi(-|x|) in this
// fp32 evaluation: about 3e-6 for |x| < 5.5 (a least-squares fit; a host test re-evaluates these coefficients against erfc).  The complementary
// form keeps the negative tail accurate, where x Phi(x) is tiny but not zero.
__device__ inline uint32_t gelu_to_half_bits(float x) {
  const float z = __builtin_fabsf(x) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.5f, z, 1.0f));
  float g = 8.510084172e-02f;                                        // Horner, fused multiply-adds
  g = __builtin_fmaf(g, t, -5.867012528e-01f);
  g = __builtin_fmaf(g, t, 1.540184314e+00f);
  g = __builtin_fmaf(g, t, -1.856008460e+00f);
  g = __builtin_fmaf(g, t, 9.031074855e-01f);
  g = __builtin_fmaf(g, t, -2.573335189e-01f);
  g = __builtin_fmaf(g, t, 4.445369191e-01f);
  g = __builtin_fmaf(g, t, 9.922661813e-01f);
  g = __builtin_fmaf(g, t, -1.265152659e+00f);
  const float q = 0.5f * t * __builtin_amdgcn_exp2f(__builtin_fmaf(-z, z, g) * 1.4426950408889634f);   // Phi(-|x|)
  return float_to_half_bits(x * (x < 0.0f ? q : 1.0f - q));
}
__device__ inline uint32_t gelu_half_pair(uint32_t w) {
  return gelu_to_half_bits(half_lo_to_float(w)) | (gelu_to_half_bits(half_hi_to_float(w)) << 16);
}

// ---- wave-wide max of a u32 held by every lane (DPP row shifts + row broadcasts); result valid in lane 63
template <int kCtrl>
__device__ inline uint32_t dpp_mov(uint32_t v) {
  // lanes without a source keep their own value (old = v, bound_ctrl off)
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, kCtrl, 0xf, 0xf, false);
}
__device__ inline uint32_t wave_max_u32_to_lane63(uint32_t v) {
  v = max(v, dpp_mov<0x111>(v));   // row_shr:1
  v = max(v, dpp_mov<0x112>(v));   // row_shr:2
  v = max(v, dpp_mov<0x114>(v));   // row_shr:4
  v = max(v, dpp_mov<0x118>(v));   // row_shr:8   -> lane 15 of each row of 16 holds the row max
  v = max(v, dpp_mov<0x142>(v));   // row_bcast:15 -> lanes 31 and 63 hold the max of their 32
  v = max(v, dpp_mov<0x143>(v));   // row_bcast:31 -> lane 63 holds the wave max
  return v;
}
__device__ inline uint32_t wave_max_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_readlane((int)wave_max_u32_to_lane63(v), 63);
}

// One 16-byte-per-lane global -> LDS copy (no registers in between).  Lane i's 16 bytes land at
// lds_addr + 16 i.  Issued through asm so that the compiler does not serialise later LDS reads
// behind it: completion is tracked by hand with vmcnt.
__device__ __forceinline__ void dma16(const void* src, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(src), "s"(lds_addr)
               : "memory");
}

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

int device_cu_count();   // compute units of the current device (cached per device)

}  // namespace mmd8
