// Row-moving kernels: Host<->cache copies, the forward gather, the gradient segment-sum and
// the Adagrad update.  A row is D fp32 = D/4 chunks of 16 bytes; consecutive lanes take
// consecutive chunks, so a wavefront moves 1 KiB of contiguous output per instruction and a
// 128-byte row (D = 32) is one request of 8 lanes.
#pragma once
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
// Host link (Algorithm 1 lines 5-6).  The Host table is pinned, device-mapped memory; the kernel
// reads / writes it directly, 16 bytes per lane, rows contiguous.  The k-th miss takes the slot
// of the k-th victim (both lists are in ascending order of the assignment), so one thread group
// does both directions for that slot: it loads the victim's row from HBM and the missed row
// from Host, then stores each on the other side.  Reads and writes cross the link at the same
// time instead of one after the other.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_swap_rows(const int* __restrict__ miss_vids,
                                                    const int64_t* __restrict__ unique_ids,
                                                    const int* __restrict__ slot,
                                                    const int64_t* __restrict__ victim_id,
                                                    float4* __restrict__ cw, float4* __restrict__ ca,
                                                    float4* __restrict__ hw, float4* __restrict__ ha,
                                                    int d4, const Ctr* ctr) {
  const int K = ctr->K;
  const int64_t total = (int64_t)ctr->M * d4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int k = (int)(i / d4), c = (int)(i % d4);
    const int v = miss_vids[k];
    const int64_t src = unique_ids[v] * d4 + c, dst = (int64_t)slot[v] * d4 + c;
    const float4 nw = hw[src], na = ha[src];
    if (k < K) {
      const int64_t back = victim_id[k] * d4 + c;
      const float4 ow = cw[dst], oa = ca[dst];
      hw[back] = ow;
      ha[back] = oa;
    }
    cw[dst] = nw;
    ca[dst] = na;
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
// Gradient segment-sum fused with the sparse Adagrad update (GPU-Worker / Backward; Algorithm 1
// line 14).  Input: perm64, the batch's positions grouped by virtual id, entry = (vid << 32) |
// row of grad.  A block takes B consecutive entries (B * D = 4096 floats, 16 KiB):
//   1. gathers their grad rows into LDS, all loads in flight at once;
//   2. splits the B rows into ranges of 16; thread (range, column) sums runs of equal vid in
//      fp64.  A run that begins and ends inside the range is complete: its sum replaces the
//      run's first row in LDS.  A run cut by a range edge leaves an fp64 partial;
//   3. the first D threads chain the partials across ranges; runs closed inside the block are
//      complete as well, runs cut by the block edge go to bp[block][0 = head, 1 = tail] in HBM;
//   4. complete runs are compacted and each gets its Adagrad update (or is emitted as a row of
//      the common-gradient matrix), D/4 lanes per row.
// k_seg_finish then chains the block-edge partials of the few long groups.  No atomics, and
// the summation tree depends only on perm64.
// A whole-range (whole-block) run stores its sum in the head slot and a zero in the tail slot
// under the same vid, so equal vids are always adjacent in the partial lists.
// ---------------------------------------------------------------------------------------------
constexpr int kSegRows = 16;        // rows per range
constexpr int kSegFloats = 4096;    // floats of grad per block in LDS

struct SegGeom { int ranges, B; };
__host__ __device__ inline SegGeom seg_geom(int D) {
  int r = 256 / D;
  if (r < 1) r = 1;
  if (r > 16) r = 16;
  SegGeom g; g.ranges = r; g.B = r * kSegRows;
  return g;
}

__device__ __forceinline__ void adagrad1(float& w, float& a, float g, float lr, float eps) {
  a = a + g * g;
  w = w - lr * g / (sqrtf(a) + eps);
}
__device__ __forceinline__ void adagrad4(float4* cw, float4* ca, int64_t r, float4 g, float lr,
                                         float eps) {
  float4 w = cw[r], a = ca[r];
  adagrad1(w.x, a.x, g.x, lr, eps);
  adagrad1(w.y, a.y, g.y, lr, eps);
  adagrad1(w.z, a.z, g.z, lr, eps);
  adagrad1(w.w, a.w, g.w, lr, eps);
  cw[r] = w;
  ca[r] = a;
}

template <bool EMIT>
__global__ __launch_bounds__(256) void k_seg_reduce(const float4* __restrict__ grad,
                                                     const int64_t* __restrict__ perm64, int n,
                                                     int D, const int* __restrict__ slot,
                                                     float4* __restrict__ cw,
                                                     float4* __restrict__ ca, float lr, float eps,
                                                     float4* __restrict__ common,
                                                     double* __restrict__ bp,
                                                     int* __restrict__ bp_vid) {
  __shared__ float tile[kSegFloats];            // [B][D] grad rows; later the complete sums
  __shared__ double part[2 * 256];              // [ranges][2][D] range-edge partials (ranges*D <= 256)
  __shared__ int lvid[16 * kSegRows + 2];       // vid of entries e0-1 .. e0+B
  __shared__ int lrow[16 * kSegRows];           // grad row of each entry
  __shared__ int pvid[32], pstart[32];          // per partial slot: vid (-1 = none), first row
  __shared__ int head[16 * kSegRows];           // 1 = complete run starts at this row; later: list
  __shared__ int smem[20];
  const SegGeom g = seg_geom(D);
  const int B = g.B, ranges = g.ranges, d4 = D / 4;
  const int tid = (int)threadIdx.x;
  const int64_t e0 = (int64_t)blockIdx.x * B;

  for (int i = tid; i < B + 2; i += 256) {
    const int64_t e = e0 - 1 + i;
    const int64_t pv = (e >= 0 && e < n) ? perm64[e] : (int64_t)-1;
    lvid[i] = (int)(pv >> 32);
    if (i >= 1 && i <= B) { lrow[i - 1] = (int)(uint32_t)pv; head[i - 1] = 0; }
  }
  if (tid < 32) pvid[tid] = -1;
  __syncthreads();

  // 1. gather (B * d4 = 1024 chunks of 16 bytes for the power-of-two dims: 4 per thread)
  {
    const int chunks = B * d4;
    float4* tile4 = reinterpret_cast<float4*>(tile);
    for (int base = 0; base < chunks; base += 256 * 4) {
      float4 v[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int ch = base + k * 256 + tid;
        v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ch < chunks) {
          const int i = ch / d4;
          if (lvid[i + 1] >= 0) v[k] = ld_stream(&grad[(int64_t)lrow[i] * d4 + (ch - i * d4)]);
        }
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int ch = base + k * 256 + tid;
        if (ch < chunks) tile4[ch] = v[k];
      }
    }
  }
  __syncthreads();

  // 2. runs inside each range
  {
    const int r = tid / D, c = tid - r * D;
    if (r < ranges) {
      const int i0 = r * kSegRows;
      double acc = 0.0;
      int cur = lvid[i0 + 1], start = i0;
      for (int i = i0; i <= i0 + kSegRows; ++i) {
        const int v = i < i0 + kSegRows ? lvid[i + 1] : -2;     // -2 closes the last run
        if (v != cur || i == i0 + kSegRows) {
          if (cur >= 0) {
            const bool begins = lvid[start] != cur;      // entry before the run differs
            const bool ends = lvid[i + 1] != cur;        // entry after the run differs
            if (begins && ends) {
              tile[start * D + c] = (float)acc;
              if (c == 0) head[start] = 1;
            } else if (!begins) {
              part[(2 * r) * D + c] = acc;
              if (c == 0) { pvid[2 * r] = cur; pstart[2 * r] = start; }
              if (!ends) {
                part[(2 * r + 1) * D + c] = 0.0;
                if (c == 0) { pvid[2 * r + 1] = cur; pstart[2 * r + 1] = start; }
              }
            } else {
              part[(2 * r + 1) * D + c] = acc;
              if (c == 0) { pvid[2 * r + 1] = cur; pstart[2 * r + 1] = start; }
            }
          }
          cur = v; start = i; acc = 0.0;
        }
        if (i < i0 + kSegRows) acc += (double)tile[i * D + c];
      }
    }
  }
  __syncthreads();

  // 3. chain the range-edge partials (slot order = range order; odd = tail, even = head)
  if (tid < D) {
    const int c = tid;
    int bv0 = -1, bv1 = -1;
    double b0 = 0.0, b1 = 0.0;
    double run = 0.0;
    int rv = -1, rstart = 0;
    bool begun = false;
    const int nslots = 2 * ranges;
    for (int j = 0; j <= nslots; ++j) {
      const int v = j < nslots ? pvid[j] : -1;
      if (v != rv) {
        if (rv >= 0) {
          // the run's last slot is j-1: an even (head) slot means it ended inside the block
          const bool ended = ((j - 1) & 1) == 0;
          if (begun && ended) {
            tile[rstart * D + c] = (float)run;
            if (c == 0) head[rstart] = 1;
          } else if (!begun) {
            bv0 = rv; b0 = run;
            if (!ended) { bv1 = rv; b1 = 0.0; }
          } else {
            bv1 = rv; b1 = run;
          }
        }
        rv = v; run = 0.0;
        if (v >= 0) { begun = (j & 1) == 1; rstart = pstart[j]; }
      }
      if (v >= 0) run += part[j * D + c];
    }
    const int64_t o = (int64_t)blockIdx.x * 2;
    bp[(o + 0) * D + c] = b0;
    bp[(o + 1) * D + c] = b1;
    if (c == 0) { bp_vid[o] = bv0; bp_vid[o + 1] = bv1; }
  }
  __syncthreads();

  // 4. compact the complete runs, then update / emit them D/4 lanes per row
  int nl = 0;
  {
    int f0 = 0, f1 = 0;
    const int i0 = 2 * tid, i1 = 2 * tid + 1;       // B <= 256
    if (i0 < B) f0 = head[i0];
    if (i1 < B) f1 = head[i1];
    const int k = block_excl_scan(f0 + f1, nl, smem);
    __syncthreads();                                  // all flags read before the list overwrites them
    if (f0) head[k] = i0;
    if (f1) head[k + f0] = i1;
  }
  __syncthreads();
  {
    const int groups = 256 / d4, gi = tid / d4, c4 = tid - gi * d4;
    const float4* tile4 = reinterpret_cast<const float4*>(tile);
    if (gi < groups) {
      // four rows per pass: all row loads are issued before the first update is computed
      for (int k0 = gi; k0 < nl; k0 += 4 * groups) {
        float4 gs[4], w[4], a[4];
        int64_t r[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int k = k0 + u * groups;
          r[u] = -1;
          if (k < nl) {
            const int row = head[k];
            const int v = lvid[row + 1];
            gs[u] = tile4[row * d4 + c4];
            if (EMIT) {
              common[(int64_t)v * d4 + c4] = gs[u];
            } else {
              const int s = slot[v];
              if (s >= 0) { r[u] = (int64_t)s * d4 + c4; w[u] = cw[r[u]]; a[u] = ca[r[u]]; }
            }
          }
        }
        if (!EMIT) {
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            if (r[u] >= 0) {
              adagrad1(w[u].x, a[u].x, gs[u].x, lr, eps);
              adagrad1(w[u].y, a[u].y, gs[u].y, lr, eps);
              adagrad1(w[u].z, a[u].z, gs[u].z, lr, eps);
              adagrad1(w[u].w, a[u].w, gs[u].w, lr, eps);
              cw[r[u]] = w[u];
              ca[r[u]] = a[u];
            }
          }
        }
      }
    }
  }
}

// Chains the block-edge partials: slot j = 2 * block + (0 head | 1 tail); equal vids are adjacent
// and a long group (the hottest id spans thousands of blocks) is one long run of slots.  One
// thread block per slot; only the first slot of a run works: it finds the run's end by binary
// search (the predicate "same vid" is true on the run and false after it), its 256 threads sum
// the run's partials in a strided, fixed order and combine through LDS.
template <bool EMIT>
__global__ __launch_bounds__(256) void k_seg_finish(const double* __restrict__ bp,
                                                     const int* __restrict__ bp_vid, int nslots,
                                                     int D, const int* __restrict__ slot,
                                                     float4* __restrict__ cw,
                                                     float4* __restrict__ ca, float lr, float eps,
                                                     float4* __restrict__ common) {
  __shared__ double red[256 * 4];
  const int j = (int)blockIdx.x;
  const int v = bp_vid[j];
  if (v < 0 || (j > 0 && bp_vid[j - 1] == v)) return;     // not the first slot of its run
  int lo = j, hi = nslots;                                 // bp_vid[lo] == v, run ends in (lo, hi]
  while (hi - lo > 1) {
    const int mid = lo + (hi - lo) / 2;
    if (bp_vid[mid] == v) lo = mid; else hi = mid;
  }
  const int end = hi;
  const int d4 = D / 4, tid = (int)threadIdx.x;
  const int lanes = 256 / d4, q = tid / d4, c4 = tid - q * d4;
  double s0 = 0., s1 = 0., s2 = 0., s3 = 0.;
  if (q < lanes) {
    for (int k = j + q; k < end; k += lanes) {
      const double4 x = *reinterpret_cast<const double4*>(&bp[(int64_t)k * D + 4 * c4]);
      s0 += x.x; s1 += x.y; s2 += x.z; s3 += x.w;
    }
  }
  red[tid * 4 + 0] = s0; red[tid * 4 + 1] = s1; red[tid * 4 + 2] = s2; red[tid * 4 + 3] = s3;
  __syncthreads();
  if (q == 0) {
    for (int o = 1; o < lanes; ++o) {
      const double* r = &red[(o * d4 + c4) * 4];
      s0 += r[0]; s1 += r[1]; s2 += r[2]; s3 += r[3];
    }
    const float4 gs = make_float4((float)s0, (float)s1, (float)s2, (float)s3);
    if (EMIT) {
      common[(int64_t)v * d4 + c4] = gs;
    } else {
      const int s = slot[v];
      if (s >= 0) adagrad4(cw, ca, (int64_t)s * d4 + c4, gs, lr, eps);
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void k_fill(T* p, int64_t n, T v) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = v;
}

}  // namespace sfc
