// Streaming ceilings of the HBM of one MI355X for the access patterns of the memory-bound kernels:
// read only (scan), write only, copy 2 B -> 2 B, and the codec's shapes (read 2 B / write 1 B per
// element and the reverse).  16 bytes per lane per access, buffers far larger than the 256 MB
// last-level cache, several launch shapes.  Stand-alone:
//   hipcc --offload-arch=gfx950 -O3 hbm_stream.hip -o hbm_stream && ./hbm_stream
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <stdint.h>
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)

// kUnroll independent 16-byte accesses per lane and loop trip; n16 = number of 16-byte items
template <int kUnroll, bool kNt>
__global__ __launch_bounds__(256) void k_read(const v4u* __restrict__ src, size_t n16, uint32_t* sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  uint32_t s = 0;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride * kUnroll) {
    v4u v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const size_t j = i + u * stride;
      v[u] = v4u{0, 0, 0, 0};
      if (j < n16) v[u] = kNt ? __builtin_nontemporal_load(src + j) : src[j];
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) s += v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
  }
  if (s == 0x9e3779b9u) sink[0] = s;
}
template <int kUnroll, bool kNt>
__global__ __launch_bounds__(256) void k_write(v4u* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride * kUnroll) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const size_t j = i + u * stride;
      const v4u v = v4u{(uint32_t)j, 1, 2, 3};
      if (j < n16) { if (kNt) __builtin_nontemporal_store(v, dst + j); else dst[j] = v; }
    }
  }
}
template <int kUnroll, bool kNt>
__global__ __launch_bounds__(256) void k_copy(const v4u* __restrict__ src, v4u* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride * kUnroll) {
    v4u v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const size_t j = i + u * stride;
      v[u] = v4u{0, 0, 0, 0};
      if (j < n16) v[u] = kNt ? __builtin_nontemporal_load(src + j) : src[j];
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const size_t j = i + u * stride;
      if (j < n16) { if (kNt) __builtin_nontemporal_store(v[u], dst + j); else dst[j] = v[u]; }
    }
  }
}
// read 16 bytes, write 8 (the encoder's traffic shape) and the reverse (the decoder's)
template <int kUnroll>
__global__ __launch_bounds__(256) void k_narrow(const v4u* __restrict__ src, v2u* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride * kUnroll) {
    v4u v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const size_t j = i + u * stride;
      v[u] = v4u{0, 0, 0, 0};
      if (j < n16) v[u] = __builtin_nontemporal_load(src + j);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const size_t j = i + u * stride;
      if (j < n16) __builtin_nontemporal_store(v2u{v[u][0] ^ v[u][1], v[u][2] ^ v[u][3]}, dst + j);
    }
  }
}
template <int kUnroll>
__global__ __launch_bounds__(256) void k_widen(const v2u* __restrict__ src, v4u* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride * kUnroll) {
    v2u v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const size_t j = i + u * stride;
      v[u] = v2u{0, 0};
      if (j < n16) v[u] = __builtin_nontemporal_load(src + j);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const size_t j = i + u * stride;
      if (j < n16) __builtin_nontemporal_store(v4u{v[u][0], v[u][1], v[u][0] + 1, v[u][1] + 1}, dst + j);
    }
  }
}

template <class F>
static void timed(const char* name, double bytes, F launch) {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  launch(0); CK(hipDeviceSynchronize());
  const int reps = 6;
  CK(hipEventRecord(e0));
  for (int r = 0; r < reps; ++r) launch(r + 1);
  CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  ms /= reps;
  printf("%-58s %8.1f us  %7.0f GB/s  (%4.1f %% of 8 TB/s)\n", name, ms * 1e3, bytes / (ms * 1e-3) / 1e9, bytes / (ms * 1e-3) / 8e10);
  fflush(stdout);
}

int main() {
  // four rotating 512 MiB buffers: every launch touches memory that has left the last-level cache
  const size_t bytes = 512ull << 20, n16 = bytes / 16;
  const int NB = 4;
  v4u* buf[NB];
  for (int b = 0; b < NB; ++b) { CK(hipMalloc(&buf[b], bytes)); CK(hipMemset(buf[b], 1 + b, bytes)); }
  uint32_t* sink; CK(hipMalloc(&sink, 64));
  int cus = 256; CK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
  printf("compute units: %d\n", cus);
  const int oneshot4 = (int)((n16 + 256 * 4 - 1) / (256 * 4));
  char name[128];
  for (int per_cu : {4, 8, 16, 0}) {
    const int grid = per_cu ? cus * per_cu : oneshot4;
    snprintf(name, sizeof name, "read  x4 plain, %d workgroups", grid);
    timed(name, (double)bytes, [&](int r) { hipLaunchKernelGGL((k_read<4, false>), dim3(grid), dim3(256), 0, 0, buf[r % NB], n16, sink); });
    snprintf(name, sizeof name, "read  x4 nontemporal, %d workgroups", grid);
    timed(name, (double)bytes, [&](int r) { hipLaunchKernelGGL((k_read<4, true>), dim3(grid), dim3(256), 0, 0, buf[r % NB], n16, sink); });
    snprintf(name, sizeof name, "write x4 plain, %d workgroups", grid);
    timed(name, (double)bytes, [&](int r) { hipLaunchKernelGGL((k_write<4, false>), dim3(grid), dim3(256), 0, 0, buf[r % NB], n16); });
    snprintf(name, sizeof name, "write x4 nontemporal, %d workgroups", grid);
    timed(name, (double)bytes, [&](int r) { hipLaunchKernelGGL((k_write<4, true>), dim3(grid), dim3(256), 0, 0, buf[r % NB], n16); });
    snprintf(name, sizeof name, "copy  x4 plain, %d workgroups", grid);
    timed(name, 2.0 * bytes, [&](int r) { hipLaunchKernelGGL((k_copy<4, false>), dim3(grid), dim3(256), 0, 0, buf[r % NB], buf[(r + 2) % NB], n16); });
    snprintf(name, sizeof name, "copy  x4 nontemporal, %d workgroups", grid);
    timed(name, 2.0 * bytes, [&](int r) { hipLaunchKernelGGL((k_copy<4, true>), dim3(grid), dim3(256), 0, 0, buf[r % NB], buf[(r + 2) % NB], n16); });
    snprintf(name, sizeof name, "read 16 B write 8 B (encoder shape) x4, %d workgroups", grid);
    timed(name, 1.5 * bytes, [&](int r) { hipLaunchKernelGGL((k_narrow<4>), dim3(grid), dim3(256), 0, 0, buf[r % NB], (v2u*)buf[(r + 2) % NB], n16); });
    snprintf(name, sizeof name, "read 8 B write 16 B (decoder shape) x4, %d workgroups", grid);
    timed(name, 1.5 * bytes, [&](int r) { hipLaunchKernelGGL((k_widen<4>), dim3(grid), dim3(256), 0, 0, (const v2u*)buf[r % NB], buf[(r + 2) % NB], n16); });
  }
  {
    const int grid = cus * 8;
    timed("read  x8 nontemporal, 2048 workgroups", (double)bytes, [&](int r) { hipLaunchKernelGGL((k_read<8, true>), dim3(grid), dim3(256), 0, 0, buf[r % NB], n16, sink); });
    timed("copy  x8 nontemporal, 2048 workgroups", 2.0 * bytes, [&](int r) { hipLaunchKernelGGL((k_copy<8, true>), dim3(grid), dim3(256), 0, 0, buf[r % NB], buf[(r + 2) % NB], n16); });
    timed("copy  x2 nontemporal, 2048 workgroups", 2.0 * bytes, [&](int r) { hipLaunchKernelGGL((k_copy<2, true>), dim3(grid), dim3(256), 0, 0, buf[r % NB], buf[(r + 2) % NB], n16); });
  }
  {
    // the library copy for comparison
    timed("hipMemcpyDtoD (runtime's own copy)", 2.0 * bytes, [&](int r) { CK(hipMemcpyAsync(buf[(r + 2) % NB], buf[r % NB], bytes, hipMemcpyDeviceToDevice, 0)); });
  }
  return 0;
}
