// What this GPU reaches on the access patterns the step kernels are made of: streaming read /
// write / copy, random row gathers, random and same-address atomics.  The figures are the
// practical ceilings that the kernel durations are read against (next to the 8 TB/s vendor peak).
// Usage: hbm_ceilings            (prints one line per pattern; about two seconds)
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define HIP_OK(x)                                                                              \
  do {                                                                                         \
    hipError_t e_ = (x);                                                                       \
    if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(2); } \
  } while (0)

typedef float vf4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint64_t mix(uint64_t x) {
  x ^= x >> 33; x *= 0xff51afd7ed558ccdULL; x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ULL; x ^= x >> 33;
  return x;
}

// each thread moves four 16-byte chunks, 4 KiB apart within its block's 16 KiB
__global__ __launch_bounds__(256) void k_read(const float4* __restrict__ a, size_t n, float* sink) {
  const size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const size_t j = i + k * 256;
    if (j < n) { const float4 v = a[j]; s += v.x + v.y + v.z + v.w; }
  }
  if (s == 12345.678f) *sink = s;
}
__global__ __launch_bounds__(256) void k_write(float4* __restrict__ b, size_t n) {
  const size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
  const vf4 v = {1.f, 2.f, 3.f, 4.f};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const size_t j = i + k * 256;
    if (j < n) __builtin_nontemporal_store(v, (vf4*)&b[j]);
  }
}
__global__ __launch_bounds__(256) void k_copy(const float4* __restrict__ a, float4* __restrict__ b, size_t n) {
  const size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const size_t j = i + k * 256;
    if (j < n) __builtin_nontemporal_store(__builtin_nontemporal_load((const vf4*)&a[j]), (vf4*)&b[j]);
  }
}
// rows of d4 chunks in a pseudo-random order, one chunk per lane, four rows per thread in flight
__global__ __launch_bounds__(256) void k_gather(const float4* __restrict__ a, size_t rows, int d4, size_t chunks,
                                                float* sink) {
  const size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const size_t j = i + k * 256;
    if (j < chunks) {
      const size_t r = mix(j / d4) % rows;
      const float4 v = a[r * d4 + j % d4];
      s += v.x + v.y + v.z + v.w;
    }
  }
  if (s == 12345.678f) *sink = s;
}
// the mirror image: rows read in order, written to pseudo-random places (each row once)
__global__ __launch_bounds__(256) void k_scatter_rows(const float4* __restrict__ a, float4* __restrict__ b, size_t rows,
                                                      int d4, size_t chunks, uint64_t mul) {
  const size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const size_t j = i + k * 256;
    if (j < chunks) {
      const size_t r = ((j / d4) * mul) % rows;          // a bijection for odd mul and rows a power of two
      __builtin_nontemporal_store(*(const vf4*)&a[j], (vf4*)&b[r * d4 + j % d4]);
    }
  }
}
__global__ __launch_bounds__(256) void k_atomic(int* c, size_t words, size_t n, int same) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) atomicAdd(&c[same ? 0 : mix(i) % words], 1);
}

template <typename F>
static double best_ms(F launch) {
  hipEvent_t a, b;
  HIP_OK(hipEventCreate(&a)); HIP_OK(hipEventCreate(&b));
  double best = 1e30;
  for (int rep = 0; rep < 6; ++rep) {
    HIP_OK(hipEventRecord(a));
    launch();
    HIP_OK(hipEventRecord(b));
    HIP_OK(hipEventSynchronize(b));
    float ms;
    HIP_OK(hipEventElapsedTime(&ms, a, b));
    if (rep > 0 && ms < best) best = ms;
  }
  return best;
}

int main() {
  const size_t bytes = (size_t)1 << 30, n = bytes / 16;
  float4 *a, *b;
  float* sink;
  HIP_OK(hipMalloc(&a, bytes)); HIP_OK(hipMalloc(&b, bytes)); HIP_OK(hipMalloc(&sink, 4));
  HIP_OK(hipMemset(a, 1, bytes)); HIP_OK(hipMemset(b, 0, bytes));
  const dim3 blk(256), grd((unsigned)((n + 1023) / 1024));
  double ms;
  ms = best_ms([&] { hipLaunchKernelGGL(k_read, grd, blk, 0, 0, a, n, sink); });
  printf("stream read   1 GiB               %7.1f us  %6.2f TB/s\n", ms * 1e3, bytes / ms / 1e9);
  ms = best_ms([&] { hipLaunchKernelGGL(k_write, grd, blk, 0, 0, b, n); });
  printf("stream write  1 GiB (nt stores)   %7.1f us  %6.2f TB/s\n", ms * 1e3, bytes / ms / 1e9);
  ms = best_ms([&] { hipLaunchKernelGGL(k_copy, grd, blk, 0, 0, a, b, n); });
  printf("copy          1 GiB -> 1 GiB      %7.1f us  %6.2f TB/s (read + written)\n", ms * 1e3, 2.0 * bytes / ms / 1e9);
  for (int d4 : {4, 8, 16}) {
    const size_t rows = n / d4;
    ms = best_ms([&] { hipLaunchKernelGGL(k_gather, grd, blk, 0, 0, a, rows, d4, n, sink); });
    printf("random gather of %3d-byte rows     %7.1f us  %6.2f TB/s\n", d4 * 16, ms * 1e3, bytes / ms / 1e9);
  }
  for (int d4 : {8}) {
    const size_t rows = n / d4;
    ms = best_ms([&] { hipLaunchKernelGGL(k_scatter_rows, grd, blk, 0, 0, a, b, rows, d4, n, 2654435761ull); });
    printf("copy with random %3d-byte row writes %5.1f us  %6.2f TB/s (read + written)\n", d4 * 16, ms * 1e3, 2.0 * bytes / ms / 1e9);
  }
  int* c = (int*)b;
  const size_t na = (size_t)1 << 24;
  ms = best_ms([&] { hipLaunchKernelGGL(k_atomic, dim3((unsigned)(na / 256)), blk, 0, 0, c, bytes / 4, na, 0); });
  printf("random atomics over 1 GiB, 2^24    %7.1f us  %6.2f G/s\n", ms * 1e3, na / ms / 1e6);
  const size_t ns = (size_t)1 << 16;
  ms = best_ms([&] { hipLaunchKernelGGL(k_atomic, dim3((unsigned)(ns / 256)), blk, 0, 0, c, bytes / 4, ns, 1); });
  printf("same-address atomics, 2^16         %7.1f us  %6.1f ns each\n", ms * 1e3, ms * 1e6 / ns);
  return 0;
}
