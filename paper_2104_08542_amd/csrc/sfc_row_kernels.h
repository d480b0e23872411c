// Row-moving kernels: Host<->cache copies, the forward gather, the gradient segment-sum and
// the Adagrad update.  A row is D fp32 = D/4 chunks of 16 bytes; consecutive lanes take
// consecutive chunks, so a wavefront moves 1 KiB of contiguous output per instruction and a
// 128-byte row (D = 32) is one request of 8 lanes.
#pragma once
#include <hip/amd_detail/amd_hip_unsafe_atomics.h>
#include "sfc_device.h"

namespace sfc {

typedef float vf4 __attribute__((ext_vector_type(4)));

// streaming (non-temporal) 16-byte accesses for data that is touched once per step
__device__ __forceinline__ float4 ld_stream(const float4* p) {
  const vf4 v = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st_stream(float4* p, float4 v) {
  vf4 x; x.x = v.x; x.y = v.y; x.z = v.z; x.w = v.w;
  __builtin_nontemporal_store(x, reinterpret_cast<vf4*>(p));
}

// ---------------------------------------------------------------------------------------------
// Host link (Algorithm 1 lines 5-6).  The Host table is pinned, device-mapped memory; the
// kernels read / write it directly, 16 bytes per lane, rows contiguous.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_writeback_victims(const int* __restrict__ victim_slot,
                                                            const int64_t* __restrict__ victim_id,
                                                            const float4* __restrict__ cw,
                                                            const float4* __restrict__ ca,
                                                            float4* __restrict__ hw,
                                                            float4* __restrict__ ha, int d4,
                                                            const Ctr* ctr) {
  const int64_t total = (int64_t)ctr->K * d4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int k = (int)(i / d4), c = (int)(i % d4);
    const int64_t src = (int64_t)victim_slot[k] * d4 + c, dst = victim_id[k] * d4 + c;
    hw[dst] = cw[src];
    ha[dst] = ca[src];
  }
}

__global__ __launch_bounds__(256) void k_fetch_misses(const int* __restrict__ miss_vids,
                                                       const int64_t* __restrict__ unique_ids,
                                                       const int* __restrict__ slot,
                                                       const float4* __restrict__ hw,
                                                       const float4* __restrict__ ha,
                                                       float4* __restrict__ cw,
                                                       float4* __restrict__ ca, int d4,
                                                       const Ctr* ctr) {
  const int64_t total = (int64_t)ctr->M * d4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int k = (int)(i / d4), c = (int)(i % d4);
    const int v = miss_vids[k];
    const int64_t src = unique_ids[v] * d4 + c, dst = (int64_t)slot[v] * d4 + c;
    cw[dst] = hw[src];
    ca[dst] = ha[src];
  }
}

// Bypass rows (misses that found no slot) go back to Host after the update.
__global__ __launch_bounds__(256) void k_writeback_bypass(const int* __restrict__ miss_vids,
                                                           const int64_t* __restrict__ unique_ids,
                                                           const int* __restrict__ slot,
                                                           const float4* __restrict__ cw,
                                                           const float4* __restrict__ ca,
                                                           float4* __restrict__ hw,
                                                           float4* __restrict__ ha, int d4,
                                                           const Ctr* ctr) {
  const int M = ctr->M, nb = ctr->n_bypass;
  const int64_t total = (int64_t)nb * d4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int k = M - nb + (int)(i / d4), c = (int)(i % d4);
    const int v = miss_vids[k];
    const int64_t src = (int64_t)slot[v] * d4 + c, dst = unique_ids[v] * d4 + c;
    hw[dst] = cw[src];
    ha[dst] = ca[src];
  }
}

__global__ __launch_bounds__(256) void k_flush(const int64_t* __restrict__ slot_id,
                                                const float4* __restrict__ cw,
                                                const float4* __restrict__ ca,
                                                float4* __restrict__ hw, float4* __restrict__ ha,
                                                int d4, const Ctr* ctr) {
  const int64_t total = (int64_t)ctr->f * d4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t s = i / d4;
    const int c = (int)(i % d4);
    const int64_t id = slot_id[s];
    if (id < 0) continue;
    hw[id * d4 + c] = cw[i];
    ha[id * d4 + c] = ca[i];
  }
}

// ---------------------------------------------------------------------------------------------
// Forward gather (Algorithm 1 lines 9 and 11 fused): out[b] = cache row of slot[inverse[b]].
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_lookup_onehot(const int* __restrict__ inverse,
                                                        const int* __restrict__ slot,
                                                        const float4* __restrict__ cw,
                                                        float4* __restrict__ out, int64_t total,
                                                        int d4) {
  const int64_t base = (int64_t)blockIdx.x * 1024 + threadIdx.x;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int64_t i = base + k * 256;
    if (i < total) {
      const int b = (int)(i / d4), c = (int)(i % d4);
      const int s = slot[inverse[b]];
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (s >= 0) v = cw[(int64_t)s * d4 + c];
      st_stream(&out[i], v);
    }
  }
}

__global__ __launch_bounds__(256) void k_lookup_bags(const int64_t* __restrict__ offsets,
                                                      const int* __restrict__ inverse,
                                                      const int* __restrict__ slot,
                                                      const float4* __restrict__ cw,
                                                      float4* __restrict__ out, int64_t total,
                                                      int d4) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int64_t b = i / d4;
  const int c = (int)(i % d4);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int64_t q = offsets[b], e = offsets[b + 1]; q < e; ++q) {
    const int s = slot[inverse[q]];
    if (s >= 0) {
      const float4 v = cw[(int64_t)s * d4 + c];
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
  }
  st_stream(&out[i], acc);
}

// ---------------------------------------------------------------------------------------------
// Gradient segment-sum (GPU-Worker / Backward): common[v] = sum of grad rows whose position has
// virtual id v, accumulated in fp64 in a [U, D] scratch that is all zero between uses.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void add4(double* dst, float4 g) {
  unsafeAtomicAdd(dst + 0, (double)g.x);
  unsafeAtomicAdd(dst + 1, (double)g.y);
  unsafeAtomicAdd(dst + 2, (double)g.z);
  unsafeAtomicAdd(dst + 3, (double)g.w);
}

__global__ __launch_bounds__(256) void k_accum_onehot(const float4* __restrict__ grad,
                                                       const int* __restrict__ inverse,
                                                       double* g64, int64_t total, int d4) {
  const int64_t base = (int64_t)blockIdx.x * 1024 + threadIdx.x;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int64_t i = base + k * 256;
    if (i < total) {
      const int b = (int)(i / d4), c = (int)(i % d4);
      const float4 g = ld_stream(&grad[i]);
      add4(g64 + ((int64_t)inverse[b] * d4 + c) * 4, g);
    }
  }
}

__global__ __launch_bounds__(256) void k_accum_bags(const float4* __restrict__ grad,
                                                     const int64_t* __restrict__ offsets,
                                                     const int* __restrict__ inverse, double* g64,
                                                     int64_t total, int d4) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int64_t b = i / d4;
  const int c = (int)(i % d4);
  const float4 g = ld_stream(&grad[i]);
  for (int64_t q = offsets[b], e = offsets[b + 1]; q < e; ++q)
    add4(g64 + ((int64_t)inverse[q] * d4 + c) * 4, g);
}

// common_grad[v] = (float) g64[v]; the scratch returns to zero.
__global__ __launch_bounds__(256) void k_emit_common(double* g64, float4* __restrict__ common,
                                                      int d4, const Ctr* ctr) {
  const int64_t total = (int64_t)ctr->U * d4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    double4* p = reinterpret_cast<double4*>(g64) + i;
    const double4 g = *p;
    *p = make_double4(0., 0., 0., 0.);
    common[i] = make_float4((float)g.x, (float)g.y, (float)g.z, (float)g.w);
  }
}

// ---------------------------------------------------------------------------------------------
// Sparse Adagrad (Algorithm 1 line 14), once per unique row:
//   acc += g*g ; w -= lr * g / (sqrt(acc) + eps)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void adagrad1(float& w, float& a, float g, float lr, float eps) {
  a = a + g * g;
  w = w - lr * g / (sqrtf(a) + eps);
}

__global__ __launch_bounds__(256) void k_adagrad(double* g64, const int* __restrict__ slot,
                                                  float4* __restrict__ cw, float4* __restrict__ ca,
                                                  float lr, float eps, int d4, const Ctr* ctr) {
  const int64_t total = (int64_t)ctr->U * d4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int v = (int)(i / d4), c = (int)(i % d4);
    double4* p = reinterpret_cast<double4*>(g64) + i;
    const double4 gd = *p;
    *p = make_double4(0., 0., 0., 0.);
    const int s = slot[v];
    if (s < 0) continue;
    const int64_t r = (int64_t)s * d4 + c;
    float4 w = cw[r], a = ca[r];
    adagrad1(w.x, a.x, (float)gd.x, lr, eps);
    adagrad1(w.y, a.y, (float)gd.y, lr, eps);
    adagrad1(w.z, a.z, (float)gd.z, lr, eps);
    adagrad1(w.w, a.w, (float)gd.w, lr, eps);
    cw[r] = w;
    ca[r] = a;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void k_fill(T* p, int64_t n, T v) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = v;
}

}  // namespace sfc
