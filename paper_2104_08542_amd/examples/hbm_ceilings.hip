// What this GPU reaches on the access patterns the step kernels are made of: streaming read /
// write / copy, random row gathers, random and same-address atomics.  The figures are the
// practical ceilings that the kernel durations are read against (next to the 8 TB/s vendor peak).
// A second part runs two patterns side by side on two streams, and each pattern beside a small
// kernel that moves 256-byte rows to and from pinned host memory: how much of a pipeline's overlap
// this GPU turns into time saved.
// Usage: hbm_ceilings            (prints one line per pattern; a few seconds)
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

// 256-byte rows between pinned host memory and HBM, zero-copy: reads (mode & 1), writes (mode & 2)
__global__ __launch_bounds__(256) void k_host_rows(float4* host, size_t host_rows, float4* dev, int rows, int mode) {
  const size_t total = (size_t)rows * 16;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const size_t k = i / 16, c = i % 16;
    float4 v = dev[i];
    if (mode & 2) host[(mix(2 * k + 1) % host_rows) * 16 + c] = v;
    if (mode & 1) v = host[(mix(2 * k) % host_rows) * 16 + c];
    dev[i] = v;
  }
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

  // ---- two streams -------------------------------------------------------------------------
  hipStream_t s1, s2;
  HIP_OK(hipStreamCreateWithFlags(&s1, hipStreamNonBlocking));
  HIP_OK(hipStreamCreateWithFlags(&s2, hipStreamNonBlocking));
  const size_t q = n / 4, qrows = q / 8;              // 256 MiB per launch
  auto pattern = [&](int which, hipStream_t st) {
    const dim3 g((unsigned)((q + 1023) / 1024));
    if (which == 0) hipLaunchKernelGGL(k_copy, g, blk, 0, st, a, b, q);
    if (which == 1) hipLaunchKernelGGL(k_gather, g, blk, 0, st, a + q, qrows, 8, q, sink);
    if (which == 2) hipLaunchKernelGGL(k_atomic, dim3((unsigned)(na / 4 / 256)), blk, 0, st, (int*)(b + 2 * q), bytes / 16, na / 4, 0);
  };
  const char* pname[3] = {"copy 256 MiB", "gather 128-byte rows, 256 MiB", "random atomics, 2^22"};
  hipEvent_t e0, e1, e2;
  HIP_OK(hipEventCreate(&e0)); HIP_OK(hipEventCreate(&e1)); HIP_OK(hipEventCreate(&e2));
  double alone[3];
  for (int w = 0; w < 3; ++w) {
    alone[w] = best_ms([&] { pattern(w, 0); });
    printf("alone: %-30s %7.1f us\n", pname[w], alone[w] * 1e3);
  }
  const int reps = 10;
  const int pairs[3][2] = {{0, 1}, {1, 2}, {0, 2}};
  for (auto& pr : pairs) {
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipEventRecord(e0, s1)); HIP_OK(hipStreamWaitEvent(s2, e0, 0));
    for (int r = 0; r < reps; ++r) { pattern(pr[0], s1); pattern(pr[1], s2); }
    HIP_OK(hipEventRecord(e1, s1)); HIP_OK(hipEventRecord(e2, s2));
    HIP_OK(hipDeviceSynchronize());
    float m1, m2;
    HIP_OK(hipEventElapsedTime(&m1, e0, e1)); HIP_OK(hipEventElapsedTime(&m2, e0, e2));
    const double both = (m1 > m2 ? m1 : m2) / reps, serial = alone[pr[0]] + alone[pr[1]];
    printf("side by side: %s + %s: %.1f us per pair, %.1f us one after the other (%.2f)\n", pname[pr[0]],
           pname[pr[1]], both * 1e3, serial * 1e3, both / serial);
  }
  // each pattern beside zero-copy host traffic: 55000 rows of 256 bytes per launch on 32 blocks
  const size_t host_rows = (size_t)1 << 24;           // 4 GiB of pinned host memory
  float4 *host, *host_d, *stage;
  HIP_OK(hipHostMalloc((void**)&host, host_rows * 256, hipHostMallocMapped));
  for (size_t o = 0; o < host_rows * 256; o += 4096) ((volatile char*)host)[o] = 0;
  HIP_OK(hipHostGetDevicePointer((void**)&host_d, host, 0));
  const int hrows = 55000;
  HIP_OK(hipMalloc(&stage, (size_t)hrows * 256));
  HIP_OK(hipMemset(stage, 0, (size_t)hrows * 256));
  const char* hname[4] = {"", "host reads", "host writes", "host reads + writes"};
  for (int mode = 1; mode <= 3; ++mode) {
    const double hm = best_ms([&] { hipLaunchKernelGGL(k_host_rows, dim3(32), blk, 0, 0, host_d, host_rows, stage, hrows, mode); });
    printf("alone: %-20s %7.1f us  %5.1f GB/s\n", hname[mode], hm * 1e3, hrows * 256.0 * (mode == 3 ? 2 : 1) / hm / 1e6);
    for (int w = 0; w < 3; ++w) {
      HIP_OK(hipDeviceSynchronize());
      const int cover = (int)(alone[w] * reps * 2 / hm) + 2;     // host traffic outlasts the timed launches
      HIP_OK(hipEventRecord(e0, s1)); HIP_OK(hipStreamWaitEvent(s2, e0, 0));
      for (int r = 0; r < cover; ++r) hipLaunchKernelGGL(k_host_rows, dim3(32), blk, 0, s1, host_d, host_rows, stage, hrows, mode);
      HIP_OK(hipEventRecord(e1, s2));
      for (int r = 0; r < reps; ++r) pattern(w, s2);
      HIP_OK(hipEventRecord(e2, s2));
      HIP_OK(hipDeviceSynchronize());
      float m;
      HIP_OK(hipEventElapsedTime(&m, e1, e2));
      printf("beside %-20s %-30s %7.1f us (%.2f of alone)\n", hname[mode], pname[w], m * 1e3 / reps, m / reps / alone[w]);
    }
  }
  HIP_OK(hipGetLastError());
  return 0;
}
