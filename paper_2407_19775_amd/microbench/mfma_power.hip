// Sustained rate of a register-only v_mfma_i32_32x32x32_i8 loop as a function of the operand data
// (constant, uniform random, Gaussian int8 codes): the chip is power-limited, so this is the
// ceiling an int8 GEMM on realistic data can approach.  Stand-alone: hipcc --offload-arch=gfx950 -O3 mfma_power.hip
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <stdint.h>
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)
__device__ inline uint32_t hash32(uint32_t i, uint32_t seed) { uint32_t h = i * 2654435761u + seed; h ^= h >> 15; h *= 2246822519u; h ^= h >> 13; h *= 3266489917u; h ^= h >> 16; return h; }
__device__ inline int gauss_byte(uint32_t h) { int s = (int)(h & 31) + (int)((h >> 5) & 31) + (int)((h >> 10) & 31) + (int)((h >> 15) & 31) - 62; return s & 0xff; }   // sigma ~ 18
// MODE 0: constant operands; 1: uniform random bytes; 2: Gaussian-like small int8 (as quantized activations/weights)
template <int MODE, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void k_pow(int iters, unsigned long long* out, int* sink) {
  v16i acc[8];
  for (int t = 0; t < 8; ++t) for (int e = 0; e < 16; ++e) acc[t][e] = 0;
  v4i a[4], b[4];
  for (int f = 0; f < 4; ++f) for (int w = 0; w < 4; ++w) {
    uint32_t ha = hash32(threadIdx.x * 64 + f * 4 + w, 1 + blockIdx.x), hb = hash32(threadIdx.x * 64 + f * 4 + w, 77 + blockIdx.x);
    if (MODE == 0) { a[f][w] = 0x01010101; b[f][w] = 0x02020202; }
    else if (MODE == 1) { a[f][w] = (int)ha; b[f][w] = (int)hb; }
    else {
      a[f][w] = gauss_byte(ha) | (gauss_byte(hash32(ha, 3)) << 8) | (gauss_byte(hash32(ha, 4)) << 16) | (gauss_byte(hash32(ha, 5)) << 24);
      b[f][w] = gauss_byte(hb) | (gauss_byte(hash32(hb, 3)) << 8) | (gauss_byte(hash32(hb, 4)) << 16) | (gauss_byte(hash32(hb, 5)) << 24);
    }
  }
  const unsigned long long t0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[t & 3], b[(t >> 1) & 3], acc[t], 0, 0, 0);
    if ((it & 63) == 63) for (int t = 0; t < 8; ++t) for (int e = 0; e < 16; ++e) acc[t][e] &= 0xffff;   // keep the sums bounded
  }
  const unsigned long long t1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  int s = 0;
  for (int t = 0; t < 8; ++t) for (int e = 0; e < 16; ++e) s += acc[t][e];
  if (s == 0x12345678) sink[0] = s;
  if (threadIdx.x == 0) { out[2 * blockIdx.x] = t1 - t0; out[2 * blockIdx.x + 1] = r1 - r0; }
}
template <int MODE, int WAVES>
void run(const char* name, unsigned long long* out, int* sink) {
  const int iters = 20000, wgs = 256;
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  hipLaunchKernelGGL((k_pow<MODE, WAVES>), dim3(wgs), dim3(WAVES * 64), 0, 0, iters, out, sink); CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  hipLaunchKernelGGL((k_pow<MODE, WAVES>), dim3(wgs), dim3(WAVES * 64), 0, 0, iters, out, sink);
  CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  unsigned long long h[2]; CK(hipMemcpy(h, out, 16, hipMemcpyDeviceToHost));
  const double ops = 2.0 * 32768 * 8 * iters * WAVES * wgs;
  printf("%-44s %7.3f ms  %7.1f TOPS   shader clock %.3f GHz  %.1f clk/MFMA/SIMD\n", name, ms, ops / (ms * 1e-3) / 1e12, (double)h[0] / h[1] * 0.1, (double)h[0] / (8.0 * iters * (WAVES / 4)));
  fflush(stdout);
}
int main() {
  unsigned long long* out; int* sink; CK(hipMalloc(&out, 16 * 4096)); CK(hipMalloc(&sink, 64));
  for (int rep = 0; rep < 2; ++rep) {
    run<0, 4>("constant operands, 4 waves/CU", out, sink);
    run<1, 4>("uniform random bytes, 4 waves/CU", out, sink);
    run<2, 4>("Gaussian int8 (sigma 18), 4 waves/CU", out, sink);
    run<0, 8>("constant operands, 8 waves/CU", out, sink);
    run<1, 8>("uniform random bytes, 8 waves/CU", out, sink);
    run<2, 8>("Gaussian int8 (sigma 18), 8 waves/CU", out, sink);
  }
  return 0;
}
