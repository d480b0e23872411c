// Row-moving kernels: Host<->cache copies, the forward gather, the gradient segment-sum and
// the optimizer updates (Adagrad, Adam, row-wise Adagrad).  A row is D fp32 = D/4 chunks of 16 bytes; consecutive lanes take
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
// kStream: the datum is read once per step (streamed); otherwise it is read again by other lanes
// later in the same kernel and should stay cached
template <bool kStream>
__device__ __forceinline__ float4 ld_row(const float4* p) { return kStream ? ld_stream(p) : *p; }
template <bool kStream>
__device__ __forceinline__ void st_row(float4* p, float4 v) { if (kStream) st_stream(p, v); else *p = v; }

// ---------------------------------------------------------------------------------------------
// Host link (Algorithm 1 lines 5-6).  The Host table is pinned, device-mapped memory; the kernels
// read / write it directly, 16 bytes per lane.  A row moves as (D + S)/4 chunks: its weights, then
// its S floats of optimizer state; hs4 / has4 are the Host row strides in 16-byte units.  When the
// caller interleaves the two Host arrays (h_acc = h_weights + D, both strides D + S) the lanes of
// a row touch one contiguous 4*(D+S)-byte block of Host memory, which the link moves measurably
// faster than two separate blocks (55 vs 41 GB/s Host->device for D = S = 32).
// The k-th miss takes the slot of the k-th victim (both lists are in ascending order of the
// assignment), so one lane group does both directions for that slot: it loads the victim's row
// from HBM and the missed row from Host, then stores each on the other side.  Reads and writes
// cross the link at the same time instead of one after the other.
//
// Pipelined steps: a row that bypassed the cache in an older step still in flight reaches the
// Host table only with that step's update, so this step's copies must then run behind it.  The
// host cannot know whether that happened without waiting, so it launches the kernel twice: once
// on the side stream right away and once on the main stream behind the older steps' updates; the
// device counters decide which of the two launches does the work (on_main below), the other one
// returns at once.  `chain` extends the rule to "the previous step's copies ran on the main
// stream and that launch was not yet enqueued when this one was issued".
// ---------------------------------------------------------------------------------------------
struct HostRows {
  float4* w;      // device view of h_weights
  float4* a;      // device view of h_acc (the optimizer state, s4 chunks per row)
  int64_t hs4;    // row stride of w in float4
  int64_t has4;   // row stride of a in float4
};

__global__ __launch_bounds__(256) void k_swap_rows(const int* __restrict__ miss_row,
                                                    const int64_t* __restrict__ miss_id,
                                                    const int64_t* __restrict__ victim_id,
                                                    float4* __restrict__ cw, float4* __restrict__ ca,
                                                    HostRows h, int d4, int s4, Ctr* ctr,
                                                    const Ctr* older1, const Ctr* older2,
                                                    const Ctr* older3, int chain, int main_variant) {
  const bool on_main = (older1 && older1->n_bypass != 0) || (older2 && older2->n_bypass != 0) ||
                       (older3 && older3->n_bypass != 0) ||
                       (chain && older1 && older1->fetch_on_main != 0);
  if (blockIdx.x == 0 && threadIdx.x == 0) ctr->fetch_on_main = on_main;   // same value from both launches
  if (on_main != (main_variant != 0)) return;
  __builtin_amdgcn_s_setprio(3);            // few waves, long round trips: issue ahead of the kernels beside them
  const int K = ctr->K;
  const int w2 = d4 + s4;                   // chunks of a row and of its optimizer state
  const int64_t total = (int64_t)ctr->M * w2;
  const int64_t stride = (int64_t)gridDim.x * 256;
  // A thread's chunks are a serial chain, and with few blocks (see the launch) the chain is long:
  // the list entries of the next chunk are fetched while this chunk's Host read is in flight, so
  // that the chain is one Host round trip per chunk and nothing that waits on HBM.
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  int row = 0;
  int64_t id = 0, vic = 0;
  if (i < total) {
    const int k = (int)(i / w2);
    row = miss_row[k]; id = miss_id[k]; vic = k < K ? victim_id[k] : -1;
  }
  while (i < total) {
    const int k = (int)(i / w2);
    int c = (int)(i - (int64_t)k * w2);
    const bool acc = c >= d4;
    if (acc) c -= d4;
    float4* hb = acc ? h.a : h.w;
    float4* cb = acc ? ca : cw;
    const int64_t hst = acc ? h.has4 : h.hs4;
    const int cst = acc ? s4 : d4;
    const int64_t dst = (int64_t)row * cst + c;
    const float4 nv = hb[id * hst + c];
    const int64_t vnow = vic;
    const int64_t inext = i + stride;
    if (inext < total) {
      const int kn = (int)(inext / w2);
      row = miss_row[kn]; id = miss_id[kn]; vic = kn < K ? victim_id[kn] : -1;
    }
    if (vnow >= 0) hb[vnow * hst + c] = cb[dst];
    cb[dst] = nv;
    i = inext;
  }
}

__global__ __launch_bounds__(256) void k_flush(const int64_t* __restrict__ slot_id,
                                                const float4* __restrict__ cw,
                                                const float4* __restrict__ ca, HostRows h, int d4,
                                                int s4, const Ctr* ctr) {
  const int w2 = d4 + s4;
  const int64_t total = (int64_t)ctr->f * w2;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t s = i / w2;
    int c = (int)(i - s * w2);
    const bool acc = c >= d4;
    if (acc) c -= d4;
    const int64_t id = slot_id[s];
    if (id < 0) continue;
    if (acc) h.a[id * h.has4 + c] = ca[s * s4 + c];
    else h.w[id * h.hs4 + c] = cw[s * d4 + c];
  }
}

// ---------------------------------------------------------------------------------------------
// Forward gather (Algorithm 1 lines 9 and 11 fused): out[b] = cache row of the slot of position b.
// pos_slot[p] = slot[inverse[p]] is written by the prepare step, so the gather is one level of
// indirection.  A block stages the slots of its bags in LDS with one coalesced load, then every
// thread has its 16-byte row chunks (up to eight) in flight before the first store; a
// wavefront's stores are 1 KiB contiguous and non-temporal: the output is consumed by the model,
// and keeping it out of L2 keeps the hot rows in (plain stores measured 50 % slower).
// What bounds it on MI355X: with the rows resident in the memory-side cache the kernel runs at
// the write rate of HBM (52-58 us for 327 MB); in the training loop the other kernels of the step
// have evicted them, the ~59 MB of row reads mix into the write stream and the same kernel takes
// 79-85 us, which is what k_warm_rows below is for.  Variants without LDS staging or with
// persistent blocks measured within +-5 % of this one under those conditions.
// ---------------------------------------------------------------------------------------------
constexpr int kLookupBags = 256;      // most rows a block of the one-hot gather takes
// Rows per block of the one-hot gather: 512 16-byte chunks, two per thread.  With the rows
// waiting in the memory-side cache (k_warm_rows) small blocks win: 62.6 us at the target
// configuration against 69.7 with 256 rows (2048 chunks) per block; 32 rows: 66.4.
inline int lookup_rows_per_block(int d4) {
  int b = 512 / d4;
  if (b < 16) b = 16;
  if (b > kLookupBags) b = kLookupBags;
  return b;
}

// Before the gather: every row the batch needs is read once, by a kernel that does nothing else.
// The gather is sensitive to the latency of its slowest row: each wavefront holds eight rows per
// lane group in flight and stores nothing until the last has arrived, and a row that comes from
// HBM between the kernel's own writes takes several times as long as one that is cached.  This
// kernel has all its loads in flight at once and nothing to wait for; the 30 MB it reads at the
// target configuration stay in the memory-side cache for the microseconds until the gather asks
// for them.  Measured there: 9.6 us of warming take the gather from 80 to 60 us.
// It only pays while the rows fit that cache with room to spare: beyond kWarmMaxBytes of rows
// (decided on the device from the step's unique count) the kernel returns at once.
constexpr int64_t kWarmMaxBytes = (int64_t)96 << 20;
constexpr int kWarmGrid = 2048;

__global__ __launch_bounds__(256) void k_warm_rows(const int* __restrict__ slot,
                                                    const float4* __restrict__ cw, int d4, int C,
                                                    int boff, const Ctr* ctr, float* sink,
                                                    const int4* __restrict__ pos_slot4, int n4) {
  const int64_t total = (int64_t)ctr->U * d4;
  if (total * 16 > kWarmMaxBytes) return;
  const int64_t stride = (int64_t)gridDim.x * 256;
  float acc = 0.f;
  // the per-position slots as well: in a pipelined run they were written steps ago and have left
  // every cache, and each block of the gather starts with a load of them
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    const int4 q = pos_slot4[i];
    acc += (float)(q.x ^ q.y ^ q.z ^ q.w) * 1e-30f;
  }
  for (int64_t i0 = (int64_t)blockIdx.x * 256 + threadIdx.x; i0 < total; i0 += 8 * stride) {
    float4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int64_t i = i0 + u * stride;
      v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i < total) {
        const int vrow = (int)(i / d4);
        int s = slot[vrow];
        if (s >= C) s += boff;
        if (s >= 0) v[u] = cw[(int64_t)s * d4 + (i - (int64_t)vrow * d4)];
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u].x + v[u].y + v[u].z + v[u].w;
  }
  // the loads must not be optimised away; no finite sum of table values equals this
  if (acc == 1.2345678e30f) *sink = acc;
}

// d4 is a runtime value; when it is a power of two (sh >= 0) index math is shifts and masks
__device__ __forceinline__ void split_chunk(unsigned ch, int d4, int sh, unsigned& r, unsigned& c) {
  if (sh >= 0) { r = ch >> sh; c = ch & (unsigned)(d4 - 1); }
  else { r = ch / (unsigned)d4; c = ch - r * (unsigned)d4; }
}

__global__ __launch_bounds__(256) void k_lookup_onehot(const int* __restrict__ pos_slot,
                                                        const float4* __restrict__ cw,
                                                        float4* __restrict__ out, int n_bags,
                                                        int d4, int sh, int bpb) {
  __shared__ int ls[kLookupBags];
  const int b0 = (int)blockIdx.x * bpb;          // bpb <= kLookupBags = block size
  {
    const int b = b0 + (int)threadIdx.x;
    ls[threadIdx.x] = ((int)threadIdx.x < bpb && b < n_bags) ? pos_slot[b] : -1;
  }
  __syncthreads();
  int nb = n_bags - b0;
  if (nb > bpb) nb = bpb;
  const unsigned chunks = (unsigned)nb * (unsigned)d4;
  float4* dst = out + (int64_t)b0 * d4;
  for (unsigned base = 0; base < chunks; base += 256 * 8) {
    float4 v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const unsigned ch = base + k * 256 + threadIdx.x;
      v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (ch < chunks) {
        unsigned r, c;
        split_chunk(ch, d4, sh, r, c);
        const int s = ls[r];
        if (s >= 0) v[k] = cw[(int64_t)s * d4 + c];
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const unsigned ch = base + k * 256 + threadIdx.x;
      if (ch < chunks) st_stream(&dst[ch], v[k]);
    }
  }
}

// Multi-hot forward (sum pooling): out[b] = sum over the positions q of bag b of the cached row of
// position q, fp32 adds in bag order.  A row is d4 lanes of 16 bytes, so a wavefront holds
// G = 64 / d4 lane groups and each group owns one bag: its lanes read the bag's slots (one
// broadcast load per position), keep kBagUnroll row chunks in flight per lane and fetch the
// slots of the next kBagUnroll positions meanwhile, so that the chain offsets -> slot -> row is
// walked once per kBagUnroll rows instead of once per row.  The four bags of a wavefront are
// neighbours, so its stores are contiguous (G * d4 * 16 bytes) and non-temporal.
// Bags are short (1-20 ids in the benchmark's multi-hot configuration), so the lane groups of a
// wavefront finish at different times; the idle lanes cost nothing that matters here, the kernel
// is bound by the row traffic (every position reads a full row; only the rows that are hot
// enough to stay in an XCD's L2 are not fetched again).
// Malformed offsets are reported by the prepare step; here they only must not lead outside
// pos_slot, hence the clamp to [0, n_ids].
#ifndef SFC_BAG_UNROLL
#define SFC_BAG_UNROLL 8
#endif
constexpr int kBagUnroll = SFC_BAG_UNROLL;

__global__ __launch_bounds__(256) void k_lookup_bags(const int64_t* __restrict__ offsets,
                                                      const int* __restrict__ pos_slot,
                                                      const float4* __restrict__ cw,
                                                      float4* __restrict__ out, int n_bags,
                                                      int d4, int G, int64_t n_ids) {
  const int lane = lane_id();
  const int g = lane / d4, c = lane - g * d4;
  const int64_t b = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * G + g;
  if (g >= G || b >= n_bags) return;
  int64_t q = offsets[b], e = offsets[b + 1];
  if (q < 0) q = 0;
  if (e > n_ids) e = n_ids;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  int sl[kBagUnroll], sn[kBagUnroll];
#pragma unroll
  for (int k = 0; k < kBagUnroll; ++k) sl[k] = q + k < e ? pos_slot[q + k] : -1;
  for (; q < e; q += kBagUnroll) {
    float4 v[kBagUnroll];
#pragma unroll
    for (int k = 0; k < kBagUnroll; ++k) {
      v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (sl[k] >= 0) v[k] = cw[(int64_t)sl[k] * d4 + c];
    }
#pragma unroll
    for (int k = 0; k < kBagUnroll; ++k) {
      const int64_t qn = q + kBagUnroll + k;
      sn[k] = qn < e ? pos_slot[qn] : -1;
    }
#pragma unroll
    for (int k = 0; k < kBagUnroll; ++k) {
      acc.x += v[k].x; acc.y += v[k].y; acc.z += v[k].z; acc.w += v[k].w;
      sl[k] = sn[k];
    }
  }
  st_stream(&out[b * d4 + c], acc);
}

// ---------------------------------------------------------------------------------------------
// Gradient segment-sum (GPU-Worker / Backward): common[v] = sum of the grad rows of the positions
// with virtual id v.  Input: perm64, the batch's positions grouped by virtual id, entry =
// (vid << 32) | row of grad.  The kernel is a barrier-free stream over perm64:
//   - a row is D/4 lanes of 16 bytes, so a wavefront holds G = 64 / (D/4) lane groups; group g of
//     wavefront w owns the span of L consecutive entries starting at (w*G + g)*L;
//   - a group walks its span four entries at a time, the grad rows of the next four already in
//     flight, and sums runs of equal vid in fp64 registers.  A run that begins and ends inside
//     the span is complete when it closes: it is rounded to fp32 once and stored as row vid of
//     the common-gradient matrix;
//   - a run cut by the span's edge leaves an fp64 partial (head / tail).  The G groups of the
//     wavefront chain their partials through LDS once, at the end; runs cut by the wavefront's
//     edge are chained once more across the block's four wavefronts; what is cut by the
//     block's edge goes to bp[block][0 = head, 1 = tail] in HBM and k_seg_finish chains those.
// No atomics; the summation tree depends only on perm64, n and D.  perm64 itself lists a group's
// positions in the order the grouping pass ranked them, which its atomics decide, so the fp64 sum
// of a frequent id can differ in its last bits from run to run; rounded to fp32 once, the results
// of two runs are nearly always identical and never further apart than one unit in the last place
// of the sum (ids with at most kColdMax positions are added in a fixed order and are identical).
// A run that covers a whole span (wavefront) stores its sum in the head slot and a zero in the
// tail slot under the same vid, so equal vids are always adjacent in the partial lists.
//
// The Adagrad update is a separate kernel over the common-gradient matrix (k_adagrad_rows).
// Fusing it into the stream (update the cached row when its run closes) was measured slower on
// MI355X: the dependent chain entry -> slot -> cached row sits inside the streaming loop and
// the extra registers cost a wavefront of occupancy per SIMD, which outweighs the 60 MB of
// common-gradient traffic that fusion saves.
// ---------------------------------------------------------------------------------------------
#ifndef SFC_SEG_CHUNK
#define SFC_SEG_CHUNK 4
#endif
constexpr int kSegChunk = SFC_SEG_CHUNK;        // entries per group per loop iteration
// the stream never has more wavefronts than this: 48 per compute unit measured best at the target
// size (16: stream 82 us + finish 10; 48: 75 + 14; the finish pass grows with the number of blocks)
#ifndef SFC_SEG_WAVES
#define SFC_SEG_WAVES 48
#endif
constexpr int kSegTargetWaves = 256 * SFC_SEG_WAVES;

struct SegGeom { int G, L, waves; };
// L is chosen so that the stream has about kSegTargetWaves wavefronts.
inline SegGeom seg_geom(int D, int64_t n) {
  SegGeom g;
  g.G = 64 / (D / 4);
  if (g.G < 1) g.G = 1;
  const int64_t target_waves = kSegTargetWaves;
  int64_t L = (n + g.G * target_waves - 1) / (g.G * target_waves);
  // never below 32 entries per span, except for batches too small to fill the chip that way
  // (a 4e4-position batch: 13 against 21 us with spans of 8)
  const int64_t lmin = n < ((int64_t)1 << 18) ? 8 : 32;
  if (L < lmin) L = lmin;
  L = (L + kSegChunk - 1) / kSegChunk * kSegChunk;
  g.L = (int)L;
  g.waves = (int)((n + (int64_t)g.G * L - 1) / ((int64_t)g.G * L));
  return g;
}

struct D4 { double x, y, z, w; };
__device__ __forceinline__ void d4_zero(D4& a) { a.x = a.y = a.z = a.w = 0.0; }
__device__ __forceinline__ void d4_add(D4& a, float4 v) {
  a.x += (double)v.x; a.y += (double)v.y; a.z += (double)v.z; a.w += (double)v.w;
}
__device__ __forceinline__ float4 d4_round(const D4& a) {
  return make_float4((float)a.x, (float)a.y, (float)a.z, (float)a.w);
}

// Chains a list of partial slots (even = head of a span, odd = its tail; vid -1 = none).  Runs that
// begin at an odd slot and end at an even one lie inside the list: they are complete and stored.
// A run open at the left edge is returned as (bv0, b0), one open at the right edge as (bv1, b1);
// a run open at both edges returns its sum in b0 and a zero marker in b1.
__device__ __forceinline__ void chain_slots(int nslots, const int* __restrict__ vids,
                                            const double* __restrict__ sums, int D, int d4, int c4,
                                            float4* __restrict__ common, int& bv0, D4& b0, int& bv1,
                                            D4& b1) {
  bv0 = -1; bv1 = -1;
  d4_zero(b0); d4_zero(b1);
  D4 run; d4_zero(run);
  int rv = -1;
  bool rbegun = false;
  for (int j = 0; j <= nslots; ++j) {
    const int v = j < nslots ? vids[j] : -1;
    if (v != rv) {
      if (rv >= 0) {
        const bool ended = ((j - 1) & 1) == 0;      // the run's last slot was a head slot
        if (rbegun && ended) {
          common[(int64_t)rv * d4 + c4] = d4_round(run);
        } else if (!rbegun) {
          bv0 = rv; b0 = run;
          if (!ended) bv1 = rv;
        } else {
          bv1 = rv; b1 = run;
        }
      }
      rv = v; d4_zero(run);
      rbegun = (j & 1) == 1;
    }
    if (v >= 0) {
      const double* q = &sums[j * D + 4 * c4];
      run.x += q[0]; run.y += q[1]; run.z += q[2]; run.w += q[3];
    }
  }
}

// kOneHot: every gradient row is read exactly once (one position per bag): streamed with
// non-temporal loads (measured 75 against 96 us at the target one-hot configuration).  Multi-hot: a
// bag's row is read once per position of the bag, from all over the grouping: plain loads, so that
// the caches keep what they can (358 against 410 us at the multi-hot configuration).
// kSkipCold: entries of cold groups (see kColdBit) are passed over, their gradient rows are not
// read: sfc_backward_update with the Adagrad kernel, which sums those groups itself.  An entry
// that is passed over acts as a separator (key -1): it ends the run before it and begins none.
template <bool kSkipCold>
__device__ __forceinline__ int entry_key(int64_t e) {
  return (kSkipCold && entry_cold(e)) ? -1 : entry_vid(e);
}

// kSegChunk consecutive grouping entries from q on (q is a multiple of kSegChunk, the array is
// 256-byte aligned), -1 for those at or beyond se: 16-byte loads of two entries where both exist.
__device__ __forceinline__ void load_entries(const int64_t* __restrict__ perm64, int64_t q,
                                             int64_t se, int64_t (&e)[kSegChunk]) {
  static_assert(kSegChunk % 2 == 0, "entries are loaded in pairs");
#pragma unroll
  for (int k = 0; k < kSegChunk; k += 2) {
    if (q + k + 1 < se) {
      const longlong2 v = *reinterpret_cast<const longlong2*>(&perm64[q + k]);
      e[k] = v.x; e[k + 1] = v.y;
    } else {
      e[k] = q + k < se ? perm64[q + k] : (int64_t)-1;
      e[k + 1] = -1;
    }
  }
}

template <bool kOneHot, bool kSkipCold>
__global__ __launch_bounds__(256) void k_seg_stream(const float4* __restrict__ grad,
                                                     const int64_t* __restrict__ perm64, int n,
                                                     int d4, int G, int L,
                                                     float4* __restrict__ common,
                                                     double* __restrict__ bp,
                                                     int* __restrict__ bp_vid,
                                                     int* __restrict__ edge_mark) {
  // per wavefront: [2G slots][D] doubles (2*G*D <= 512) and the slots' vids
  __shared__ double part[4][512];
  __shared__ int pvid[4][128];
  __shared__ int wvid[8];
  // [4 wavefronts][2][D] (8 * D <= 2048 doubles): reuses part once every wavefront has chained its
  // own slots, which keeps the block at 18 KB of LDS and the kernel register-limited
  double* const wpart = &part[0][0];
  const int lane = lane_id(), wib = (int)(threadIdx.x >> 6);
  const int wave = (int)blockIdx.x * 4 + wib;
  const int g = lane / d4, c4 = lane - g * d4;
  const int D = d4 * 4;
  const bool active = g < G;
  const int64_t sb = ((int64_t)wave * G + g) * L;           // span of this group: [sb, se)
  int64_t se = sb + L;
  if (se > n) se = n;
  const bool nonempty = active && sb < n;

  int cur = -1;           // vid of the open run
  bool begun = false;     // the open run began inside this span
  D4 acc; d4_zero(acc);
  int head_v = -1; D4 head_s; d4_zero(head_s);     // run that continues from before the span
  int tail_v = -1; D4 tail_s; d4_zero(tail_s);     // run that continues past the span

  if (nonempty) {
    const int prev_v = sb > 0 ? entry_key<kSkipCold>(perm64[sb - 1]) : -1;
    // software pipeline: pe / x = entries and grad rows of the chunk being processed (issued one
    // iteration earlier), pn = the next chunk's entries
    int64_t pe[kSegChunk], pn[kSegChunk];
    float4 x[kSegChunk];
    load_entries(perm64, sb, se, pe);
#pragma unroll
    for (int k = 0; k < kSegChunk; ++k) {
      x[k] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (pe[k] >= 0 && entry_key<kSkipCold>(pe[k]) >= 0)
        x[k] = ld_row<kOneHot>(&grad[(int64_t)(uint32_t)pe[k] * d4 + c4]);
    }
    load_entries(perm64, sb + kSegChunk, se, pn);
    cur = entry_key<kSkipCold>(pe[0]);
    begun = prev_v != cur;

    for (int64_t e = sb; e < se; e += kSegChunk) {
      // issue the next chunk's rows and the chunk after that's entries
      float4 xn[kSegChunk];
      int64_t pnn[kSegChunk];
#pragma unroll
      for (int k = 0; k < kSegChunk; ++k) {
        xn[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (pn[k] >= 0 && entry_key<kSkipCold>(pn[k]) >= 0)
          xn[k] = ld_row<kOneHot>(&grad[(int64_t)(uint32_t)pn[k] * d4 + c4]);
      }
      load_entries(perm64, e + 2 * kSegChunk, se, pnn);
#pragma unroll
      for (int k = 0; k < kSegChunk; ++k) {
        if (pe[k] >= 0) {
          const int v = entry_key<kSkipCold>(pe[k]);
          if (v != cur) {
            if (begun) { if (cur >= 0) common[(int64_t)cur * d4 + c4] = d4_round(acc); }
            else { head_v = cur; head_s = acc; }
            cur = v; begun = true; d4_zero(acc);
          }
          d4_add(acc, x[k]);
        }
      }
#pragma unroll
      for (int k = 0; k < kSegChunk; ++k) { pe[k] = pn[k]; pn[k] = pnn[k]; x[k] = xn[k]; }
    }
    // close the span: the open run either ends here or continues into the next span
    const int next_v = se < n ? entry_key<kSkipCold>(perm64[se]) : -1;
    if (next_v != cur || cur < 0) {
      if (begun) { if (cur >= 0) common[(int64_t)cur * d4 + c4] = d4_round(acc); }
      else { head_v = cur; head_s = acc; }
    } else if (begun) {
      tail_v = cur; tail_s = acc;
    } else {
      head_v = cur; head_s = acc; tail_v = cur;          // whole span: zero marker in the tail
    }
  }

  // chain the 2G partial slots of this wavefront (slot order = span order; even = head, odd = tail)
  if (active) {
    double* ph = &part[wib][(2 * g) * D + 4 * c4];
    ph[0] = head_s.x; ph[1] = head_s.y; ph[2] = head_s.z; ph[3] = head_s.w;
    ph += D;
    ph[0] = tail_s.x; ph[1] = tail_s.y; ph[2] = tail_s.z; ph[3] = tail_s.w;
    if (c4 == 0) { pvid[wib][2 * g] = head_v; pvid[wib][2 * g + 1] = tail_v; }
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  int wbv0 = -1, wbv1 = -1;
  D4 wb0, wb1;
  d4_zero(wb0); d4_zero(wb1);
  if (lane < d4) chain_slots(2 * G, pvid[wib], part[wib], D, d4, c4, common, wbv0, wb0, wbv1, wb1);
  __syncthreads();                       // every wavefront has read its part of `part`
  if (lane < d4) {
    const int bv0 = wbv0, bv1 = wbv1;
    const D4 b0 = wb0, b1 = wb1;
    // the wavefront's own head / tail become slots 2*wib, 2*wib+1 of the block's chain
    double* o0 = &wpart[(2 * wib) * D + 4 * c4];
    o0[0] = b0.x; o0[1] = b0.y; o0[2] = b0.z; o0[3] = b0.w;
    double* o1 = o0 + D;
    o1[0] = b1.x; o1[1] = b1.y; o1[2] = b1.z; o1[3] = b1.w;
    if (c4 == 0) { wvid[2 * wib] = bv0; wvid[2 * wib + 1] = bv1; }
  }
  __syncthreads();
  if (threadIdx.x < (unsigned)d4) {
    int bv0, bv1;
    D4 b0, b1;
    chain_slots(8, wvid, wpart, D, d4, c4, common, bv0, b0, bv1, b1);
    const int64_t o = (int64_t)blockIdx.x * 2;
    double* o0 = &bp[(o + 0) * D + 4 * c4];
    o0[0] = b0.x; o0[1] = b0.y; o0[2] = b0.z; o0[3] = b0.w;
    double* o1 = &bp[(o + 1) * D + 4 * c4];
    o1[0] = b1.x; o1[1] = b1.y; o1[2] = b1.z; o1[3] = b1.w;
    if (c4 == 0) {
      bp_vid[o] = bv0; bp_vid[o + 1] = bv1;
      // a group cut by a block's edge: its sum is not in `common`, and the optimizer kernel that
      // chains the partials itself (k_adagrad_rows) must not take it from there (see kEdgeMark)
      if (edge_mark) {
        if (bv0 >= 0) edge_mark[2 * bv0] = kEdgeMark;
        if (bv1 >= 0) edge_mark[2 * bv1] = kEdgeMark;
      }
    }
  }
}

// Chains the block-edge partials: slot j = 2 * block + (0 head | 1 tail); equal vids are adjacent
// and a long group (the hottest id spans hundreds of blocks) is one long run of slots.  One
// thread block per slot; only the first slot of a run works: it finds the run's end by binary
// search (the predicate "same vid" is true on the run and false after it), its lane groups sum
// the run's partials in a strided, fixed order, four loads in flight, and combine through LDS.
// The work of one block on slot j of the block-edge partial lists: true (for the whole block) when
// j is the first slot of its run; then v is the run's virtual id and the threads tid < d4 hold the
// run's fp64 sum, chunk tid of the row, in s.
__device__ __forceinline__ bool edge_run_sum(const double* __restrict__ bp,
                                             const int* __restrict__ bp_vid, int nslots, int d4,
                                             int j, int& v, D4& s) {
  __shared__ double red[256 * 4];
  __shared__ int s_cnt[4];
  v = bp_vid[j];
  if (v < 0 || (j > 0 && bp_vid[j - 1] == v)) return false;     // not the first slot of its run
  // the run's end: "same vid" is true on the run and false after it, so the block probes 256
  // places at once and narrows the bracket by that factor per round (two rounds for thousands of
  // slots, where a bisection took a dozen dependent loads)
  const int tid = (int)threadIdx.x;
  int lo = j, hi = nslots;                                 // bp_vid[lo] == v, run ends in (lo, hi]
  while (hi - lo > 1) {
    const int step = (hi - lo + 255) / 256;
    const int probe = lo + (tid + 1) * step;
    const bool same = probe < hi && bp_vid[probe] == v;
    const uint64_t m = __ballot(same);
    if ((tid & 63) == 0) s_cnt[tid >> 6] = __popcll(m);
    __syncthreads();
    const int k = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];   // probes 1..k are on the run
    __syncthreads();
    const int nlo = lo + k * step;
    int nhi = lo + (k + 1) * step;
    if (nhi > hi) nhi = hi;
    lo = nlo; hi = nhi;
  }
  const int end = hi, D = d4 * 4;
  const int groups = 256 / d4, g = tid / d4, c4 = tid - g * d4;
  double s0 = 0., s1 = 0., s2 = 0., s3 = 0.;
  if (g < groups) {
    const double4 zero = make_double4(0., 0., 0., 0.);
    for (int k = j + g; k < end; k += 4 * groups) {
      double4 x[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int kk = k + u * groups;
        x[u] = kk < end ? *reinterpret_cast<const double4*>(&bp[(int64_t)kk * D + 4 * c4]) : zero;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) { s0 += x[u].x; s1 += x[u].y; s2 += x[u].z; s3 += x[u].w; }
    }
  }
  double* r = &red[tid * 4];
  r[0] = s0; r[1] = s1; r[2] = s2; r[3] = s3;
  __syncthreads();
  if (g == 0) {
    for (int o = 1; o < groups; ++o) {
      const double* q = &red[(o * d4 + c4) * 4];
      s0 += q[0]; s1 += q[1]; s2 += q[2]; s3 += q[3];
    }
  }
  s.x = s0; s.y = s1; s.z = s2; s.w = s3;
  return true;
}

__global__ __launch_bounds__(256) void k_seg_finish(const double* __restrict__ bp,
                                                     const int* __restrict__ bp_vid, int nslots,
                                                     int d4, float4* __restrict__ common) {
  int v;
  D4 s;
  if (!edge_run_sum(bp, bp_vid, nslots, d4, (int)blockIdx.x, v, s)) return;
  if ((int)threadIdx.x < d4) common[(int64_t)v * d4 + threadIdx.x] = d4_round(s);
}

// ---------------------------------------------------------------------------------------------
// Sparse Adagrad (Algorithm 1 line 14), once per unique row:
//   acc += g*g ; w -= lr * g / (sqrt(acc) + eps)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void adagrad1(float& w, float& a, float g, float lr, float eps) {
  a = a + g * g;
  w = w - lr * g / (sqrtf(a) + eps);
}
__device__ __forceinline__ void adagrad4v(float4& w, float4& a, float4 g, float lr, float eps) {
  adagrad1(w.x, a.x, g.x, lr, eps);
  adagrad1(w.y, a.y, g.y, lr, eps);
  adagrad1(w.z, a.z, g.z, lr, eps);
  adagrad1(w.w, a.w, g.w, lr, eps);
}

// The update kernels touch every row of the batch once.  When those rows (weights, state, summed
// gradient; read and written) exceed what the memory-side cache holds, keeping them cached only
// evicts what the next kernel could have used: they are then moved with non-temporal accesses
// (multi-hot configuration, 1.4e6 rows of 256 bytes: 305 against 400 us).  Below that size plain
// accesses are as fast or a little faster (target configuration: 32 us either way).
constexpr int64_t kStreamRowsBytes = (int64_t)256 << 20;
__device__ __forceinline__ bool stream_rows(int U, int d4, int s4) {
  return (int64_t)U * (3 * d4 + 2 * s4) * 16 > kStreamRowsBytes;
}

// ---------------------------------------------------------------------------------------------
// Adam (Experiment settings: the paper's optimizer), lazily on the rows of the batch, with the
// batch number t in the bias corrections bc = 1 - beta^t (computed by the host in double):
//   m = b1*m + c1*g ; v = b2*v + c2*g*g ; w -= lr * (m/bc1) / (sqrt(v/bc2) + eps)
// The state of a row is 2*d4 chunks: first moments, then second moments.
// ---------------------------------------------------------------------------------------------
struct AdamArgs {
  float b1, c1, b2, c2;   // beta1, 1-beta1, beta2, 1-beta2
  float bc1, bc2, lr, eps;
};
__device__ __forceinline__ void adam1(float& w, float& m, float& v, float g, const AdamArgs& k) {
  m = k.b1 * m + k.c1 * g;
  v = k.b2 * v + k.c2 * (g * g);
  const float mhat = m / k.bc1, vhat = v / k.bc2;
  w = w - k.lr * mhat / (sqrtf(vhat) + k.eps);
}

// The two element-wise optimizers as policies of one row kernel: kParts state chunks travel with
// each 16-byte chunk of a row (part p of chunk c of a row lies at row * kParts * d4 + p * d4 + c),
// kRows rows are in flight per thread.
struct AdagradOp {
  static constexpr int kParts = 1;
  static constexpr int kRows = 3;      // four cost a wavefront of occupancy: 33 against 28.5 us
  float lr, eps;
  __device__ __forceinline__ void apply(float4& w, float4 (&st)[1], float4 g) const {
    adagrad4v(w, st[0], g, lr, eps);
  }
};
struct AdamOp {
  static constexpr int kParts = 2;
  static constexpr int kRows = 2;
  AdamArgs k;
  __device__ __forceinline__ void apply(float4& w, float4 (&st)[2], float4 g) const {
    adam1(w.x, st[0].x, st[1].x, g.x, k);
    adam1(w.y, st[0].y, st[1].y, g.y, k);
    adam1(w.z, st[0].z, st[1].z, g.z, k);
    adam1(w.w, st[0].w, st[1].w, g.w, k);
  }
};

// The update over the rows of a batch (one row per virtual id), Op::kRows rows per thread in flight.
// A bypass row (slot >= C: a miss that found no cache slot) is also written to the Host table
// here: it lives for this step only.
// The gradient of a cold row (see kColdBit) is summed here from its at most kColdMax gradient rows
// (cold_pay[v] = their numbers, -1 = none; both -1 = not a cold row), in fp64, lower gradient row
// first (so the sum does not depend on the order in which the grouping pass happened to rank the
// group's positions); a row marked kEdgeMark is left to the block that chains its partials; every
// other row takes its sum from the common-gradient matrix.  kOneHot: a gradient row is read once
// per step.
template <class Op, bool kStream, bool kOneHot>
__device__ __forceinline__ void update_rows(const Op& op, const float4* __restrict__ common,
                                            const int* __restrict__ slot,
                                            const int64_t* __restrict__ unique_ids,
                                            float4* __restrict__ cw, float4* __restrict__ cs,
                                            const HostRows& h, int C, int boff, int d4, int U,
                                            const int2* __restrict__ cold_pay,
                                            const float4* __restrict__ grad, int blk, int nblk) {
  static_assert(kColdMax == 2, "the gather path below takes two gradient rows");
  constexpr int kR = Op::kRows, kP = Op::kParts;
  const int64_t total = (int64_t)U * d4;
  const int64_t stride = (int64_t)nblk * 256;
  for (int64_t i0 = (int64_t)blk * 256 + threadIdx.x; i0 < total; i0 += kR * stride) {
    float4 g[kR], w[kR], st[kR][kP], x1[kR];
    int64_t r[kR], rs[kR];
    int sl[kR], vrow[kR], cc[kR];
    int2 cp[kR];
    // two levels of indirection, kR rows in flight at each: slot and cold rows of the row, then
    // its weights, state and gradient (one row of the common matrix, or its own one or two rows)
#pragma unroll
    for (int u = 0; u < kR; ++u) {
      const int64_t i = i0 + u * stride;
      r[u] = -1; sl[u] = -1; cp[u] = make_int2(-1, -1);
      if (i < total) {
        vrow[u] = (int)(i / d4); cc[u] = (int)(i - (int64_t)vrow[u] * d4);
        sl[u] = slot[vrow[u]];
        cp[u] = cold_pay[vrow[u]];
      }
    }
#pragma unroll
    for (int u = 0; u < kR; ++u) {
      x1[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (cp[u].x == kEdgeMark) continue;     // updated by the block that chains its partials
      if (sl[u] < 0) continue;
      const int64_t row = sl[u] >= C ? sl[u] + boff : sl[u];
      r[u] = row * d4 + cc[u];
      rs[u] = row * (kP * d4) + cc[u];
      w[u] = ld_row<kStream>(&cw[r[u]]);
#pragma unroll
      for (int p = 0; p < kP; ++p) st[u][p] = ld_row<kStream>(&cs[rs[u] + p * d4]);
      if (cp[u].x >= 0) {
        // lower gradient row first
        const bool two = cp[u].y >= 0;
        const int q0 = two && cp[u].y < cp[u].x ? cp[u].y : cp[u].x;
        const int q1 = two && cp[u].y < cp[u].x ? cp[u].x : cp[u].y;
        g[u] = ld_row<kOneHot>(&grad[(int64_t)q0 * d4 + cc[u]]);
        if (two) x1[u] = ld_row<kOneHot>(&grad[(int64_t)q1 * d4 + cc[u]]);
      } else {
        g[u] = ld_row<kStream>(&common[(int64_t)vrow[u] * d4 + cc[u]]);
      }
    }
#pragma unroll
    for (int u = 0; u < kR; ++u)
      if (cp[u].x >= 0 && cp[u].y >= 0) {
        g[u].x = (float)((double)g[u].x + (double)x1[u].x);
        g[u].y = (float)((double)g[u].y + (double)x1[u].y);
        g[u].z = (float)((double)g[u].z + (double)x1[u].z);
        g[u].w = (float)((double)g[u].w + (double)x1[u].w);
      }
#pragma unroll
    for (int u = 0; u < kR; ++u)
      if (r[u] >= 0) {
        op.apply(w[u], st[u], g[u]);
        st_row<kStream>(&cw[r[u]], w[u]);
#pragma unroll
        for (int p = 0; p < kP; ++p) st_row<kStream>(&cs[rs[u] + p * d4], st[u][p]);
        if (sl[u] >= C) {
          const int64_t id = unique_ids[vrow[u]];
          h.w[id * h.hs4 + cc[u]] = w[u];
#pragma unroll
          for (int p = 0; p < kP; ++p) h.a[id * h.has4 + p * d4 + cc[u]] = st[u][p];
        }
      }
  }
}

// One update of row v, chunk c4 of it, with the summed gradient g (lanes c4 < d4 of a lane group).
template <class Op>
__device__ __forceinline__ void update_one_row(const Op& op, int v, int c4, float4 g,
                                               const int* __restrict__ slot,
                                               const int64_t* __restrict__ unique_ids,
                                               float4* __restrict__ cw, float4* __restrict__ cs,
                                               const HostRows& h, int C, int boff, int d4) {
  constexpr int kP = Op::kParts;
  const int sl = slot[v];
  if (sl < 0) return;
  const int64_t row = sl >= C ? sl + boff : sl;
  const int64_t r = row * d4 + c4, rs = row * (kP * d4) + c4;
  float4 w = cw[r], st[kP];
#pragma unroll
  for (int p = 0; p < kP; ++p) st[p] = cs[rs + p * d4];
  op.apply(w, st, g);
  cw[r] = w;
#pragma unroll
  for (int p = 0; p < kP; ++p) cs[rs + p * d4] = st[p];
  if (sl >= C) {
    const int64_t id = unique_ids[v];
    h.w[id * h.hs4 + c4] = w;
#pragma unroll
    for (int p = 0; p < kP; ++p) h.a[id * h.has4 + p * d4 + c4] = st[p];
  }
}

// Cold rows are summed here (the stream that ran before passed over them), and so are the groups
// that the stream left as block-edge partials: the first blocks of the grid do what k_seg_finish
// does and update the rows they have summed at once; the other blocks walk the rows and pass
// over the marked ones (kEdgeMark).  The two parts share nothing and wait for nothing: the chain of
// dependent loads that sums a run (ten microseconds as a kernel of its own) runs beside the row
// stream instead of before it.
// In an edge block every lane group takes one slot of the partial lists.  Nearly all runs are two
// slots long (the tail of one stream block and the head of the next): a group that finds the first
// slot of a run of at most kEdgeShort slots adds them up itself, in slot order.  The few long runs
// (an id with thousands of positions spans many stream blocks) are listed in LDS and summed by
// the whole block, one after the other, as in k_seg_finish; their first slots lie more than
// kEdgeShort slots apart, so a block meets only a few.
constexpr int kEdgeShort = 8;
inline int edge_blocks(int nslots, int d4) {
  const int per_block = 4 * (64 / d4 > 0 ? 64 / d4 : 1);
  return (nslots + per_block - 1) / per_block;
}

template <class Op, bool kOneHot>
__device__ __forceinline__ void update_kernel(const Op& op, const float4* __restrict__ common,
                                              const int* __restrict__ slot,
                                              const int64_t* __restrict__ unique_ids,
                                              float4* __restrict__ cw, float4* __restrict__ cs,
                                              const HostRows& h, int C, int boff, int d4,
                                              const Ctr* ctr, const int2* __restrict__ cold_pay,
                                              const float4* __restrict__ grad,
                                              const double* __restrict__ bp,
                                              const int* __restrict__ bp_vid, int nslots,
                                              int nedge) {
  if ((int)blockIdx.x < nedge) {
    __shared__ int n_long;
    __shared__ int long_at[256];
    if (threadIdx.x == 0) n_long = 0;
    __syncthreads();
    const int lane = lane_id(), G = 64 / d4 > 0 ? 64 / d4 : 1;
    const int g = lane / d4, c4 = lane - g * d4;
    const int j = ((int)blockIdx.x * 4 + (int)(threadIdx.x >> 6)) * G + g;
    if (g < G && j < nslots) {
      const int v = bp_vid[j];
      if (v >= 0 && (j == 0 || bp_vid[j - 1] != v)) {       // first slot of its run
        int len = 1;
        while (len <= kEdgeShort && j + len < nslots && bp_vid[j + len] == v) ++len;
        if (len > kEdgeShort) {
          if (c4 == 0) long_at[atomicAdd(&n_long, 1)] = j;
        } else {
          const int D = d4 * 4;
          double s0 = 0., s1 = 0., s2 = 0., s3 = 0.;
          for (int k = 0; k < len; ++k) {
            const double4 x = *reinterpret_cast<const double4*>(&bp[(int64_t)(j + k) * D + 4 * c4]);
            s0 += x.x; s1 += x.y; s2 += x.z; s3 += x.w;
          }
          update_one_row(op, v, c4, make_float4((float)s0, (float)s1, (float)s2, (float)s3), slot,
                         unique_ids, cw, cs, h, C, boff, d4);
        }
      }
    }
    __syncthreads();
    const int nl = n_long;
    for (int i = 0; i < nl; ++i) {
      int v;
      D4 s;
      const bool first = edge_run_sum(bp, bp_vid, nslots, d4, long_at[i], v, s);
      if (first && (int)threadIdx.x < d4)
        update_one_row(op, v, (int)threadIdx.x, d4_round(s), slot, unique_ids, cw, cs, h, C, boff, d4);
      __syncthreads();
    }
    return;
  }
  const int U = ctr->U;
  const int blk = (int)blockIdx.x - nedge, nblk = (int)gridDim.x - nedge;
  if (stream_rows(U, d4, Op::kParts * d4))
    update_rows<Op, true, kOneHot>(op, common, slot, unique_ids, cw, cs, h, C, boff, d4, U, cold_pay, grad, blk, nblk);
  else
    update_rows<Op, false, kOneHot>(op, common, slot, unique_ids, cw, cs, h, C, boff, d4, U, cold_pay, grad, blk, nblk);
}

// Four wavefronts per SIMD: with the registers of five or six the kernel is slower (31.1 and 36.4 us
// against 29.1 at the target configuration: fewer loads in flight per wavefront, and more
// wavefronts evicting each other's lines).
template <bool kOneHot>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4)))
void k_adagrad_rows(
    const float4* __restrict__ common, const int* __restrict__ slot,
    const int64_t* __restrict__ unique_ids, float4* __restrict__ cw, float4* __restrict__ ca,
    HostRows h, int C, int boff, float lr, float eps, int d4, const Ctr* ctr,
    const int2* __restrict__ cold_pay, const float4* __restrict__ grad,
    const double* __restrict__ bp, const int* __restrict__ bp_vid, int nslots, int nedge) {
  AdagradOp op;
  op.lr = lr; op.eps = eps;
  update_kernel<AdagradOp, kOneHot>(op, common, slot, unique_ids, cw, ca, h, C, boff, d4, ctr, cold_pay,
                                    grad, bp, bp_vid, nslots, nedge);
}

template <bool kOneHot>
__global__ __launch_bounds__(256) void k_adam_rows(
    const float4* __restrict__ common, const int* __restrict__ slot,
    const int64_t* __restrict__ unique_ids, float4* __restrict__ cw, float4* __restrict__ cs,
    HostRows h, int C, int boff, AdamArgs k, int d4, const Ctr* ctr,
    const int2* __restrict__ cold_pay, const float4* __restrict__ grad,
    const double* __restrict__ bp, const int* __restrict__ bp_vid, int nslots, int nedge) {
  AdamOp op;
  op.k = k;
  update_kernel<AdamOp, kOneHot>(op, common, slot, unique_ids, cw, cs, h, C, boff, d4, ctr, cold_pay,
                                 grad, bp, bp_vid, nslots, nedge);
}

// ---------------------------------------------------------------------------------------------
// Row-wise Adagrad: one accumulator per row (first float of a one-chunk state),
//   acc += mean_j(g_j^2) ; w_j -= lr * g_j / (sqrt(acc) + eps).
// One thread per 16-byte chunk of a row as above; the d4 lanes of a row add their squares with
// shuffles when d4 is a power of two (a row then never straddles a wavefront).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_rowwise_adagrad_rows(const float4* __restrict__ common,
                                                               const int* __restrict__ slot,
                                                               const int64_t* __restrict__ unique_ids,
                                                               float4* __restrict__ cw,
                                                               float4* __restrict__ cs, HostRows h,
                                                               int C, int boff, float lr, float eps,
                                                               int d4, int pow2, const Ctr* ctr) {
  const int64_t total = (int64_t)ctr->U * d4;
  const int64_t stride = (int64_t)gridDim.x * 256;
  const float inv_d = 1.0f / (float)(4 * d4);
  if (!pow2) {
    // any other width: one thread per row (the lanes of a row could straddle two wavefronts, and
    // the accumulator must be read by all of them before one writes it)
    for (int64_t vrow = (int64_t)blockIdx.x * 256 + threadIdx.x; vrow < ctr->U; vrow += stride) {
      const int sl = slot[vrow];
      if (sl < 0) continue;
      float ss = 0.f;
      for (int j = 0; j < d4; ++j) {
        const float4 q = common[vrow * d4 + j];
        ss += q.x * q.x + q.y * q.y + q.z * q.z + q.w * q.w;
      }
      const int64_t row = sl >= C ? sl + boff : sl;
      float4 st = cs[row];
      st.x = st.x + ss * inv_d;
      const float den = sqrtf(st.x) + eps;
      const int64_t id = unique_ids[vrow];
      for (int j = 0; j < d4; ++j) {
        const float4 g = common[vrow * d4 + j];
        float4 w = cw[row * d4 + j];
        w.x = w.x - lr * g.x / den; w.y = w.y - lr * g.y / den;
        w.z = w.z - lr * g.z / den; w.w = w.w - lr * g.w / den;
        cw[row * d4 + j] = w;
        if (sl >= C) h.w[id * h.hs4 + j] = w;
      }
      cs[row] = st;
      if (sl >= C) h.a[id * h.has4] = st;
    }
    return;
  }
  // every lane of a wavefront runs the same number of iterations: the shuffles stay convergent.
  // Four rows per thread in flight at each level (slot + gradient, then state + weights).
  const int64_t rounds = (total + 4 * stride - 1) / (4 * stride);
  int64_t i0 = (int64_t)blockIdx.x * 256 + threadIdx.x;
  for (int64_t it = 0; it < rounds; ++it, i0 += 4 * stride) {
    int vrow[4], c[4], sl[4];
    float4 g[4], st[4], w[4];
    float ss[4];
    int64_t row[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t i = i0 + u * stride;
      const bool live = i < total;
      vrow[u] = live ? (int)(i / d4) : 0;
      c[u] = live ? (int)(i % d4) : 0;
      sl[u] = live ? slot[vrow[u]] : -1;
      g[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (live) g[u] = common[i];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      ss[u] = g[u].x * g[u].x + g[u].y * g[u].y + g[u].z * g[u].z + g[u].w * g[u].w;
      for (int d = 1; d < d4; d <<= 1) ss[u] += __shfl_xor(ss[u], d, kWave);
      row[u] = sl[u] >= C ? sl[u] + boff : sl[u];
      if (sl[u] >= 0) { st[u] = cs[row[u]]; w[u] = cw[row[u] * d4 + c[u]]; }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (sl[u] < 0) continue;
      const float acc = st[u].x + ss[u] * inv_d;
      const float den = sqrtf(acc) + eps;
      w[u].x = w[u].x - lr * g[u].x / den; w[u].y = w[u].y - lr * g[u].y / den;
      w[u].z = w[u].z - lr * g[u].z / den; w[u].w = w[u].w - lr * g[u].w / den;
      cw[row[u] * d4 + c[u]] = w[u];
      st[u].x = acc;
      if (c[u] == 0) cs[row[u]] = st[u];
      if (sl[u] >= C) {
        const int64_t id = unique_ids[vrow[u]];
        h.w[id * h.hs4 + c[u]] = w[u];
        if (c[u] == 0) h.a[id * h.has4] = st[u];
      }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void k_fill(T* p, int64_t n, T v) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = v;
}

}  // namespace sfc
