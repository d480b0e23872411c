// Device-side building blocks shared by the kernels of the sparse-embedding step:
// hashing, wavefront/block scans and reductions for 64-wide wavefronts, 16-byte row chunks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sfc {

constexpr int kWave = 64;
constexpr int64_t kEmpty = -1;      // never-used entry of a hash table
constexpr int64_t kNullKey = -2;    // batch-unique table: the collapsed out-of-range id
constexpr int64_t kTomb = -2;       // cache index: deleted entry (ids in the index are >= 0)
constexpr int kMissMark = -2;       // d_slot value between resolve and assignment
constexpr int kIntMax = 0x7fffffff;

// Grouped positions (perm64): one 64-bit entry per position, (virtual id << 32) | gradient row,
// groups in virtual-id order.  Virtual ids stay below 2^30, so bit 62 is free: it marks the
// entries of a *cold* group, one of at most kColdMax positions whose virtual id lies outside the
// range the grouping passes treat in LDS.  Nine rows in ten of a power-law batch are such rows.
// Their gradients are summed by the optimizer kernel itself, straight from the gradient rows;
// the segment-sum stream passes over them, and their rows of the common-gradient matrix are
// neither written nor read.
constexpr int kHotBins = 8192;      // lowest virtual ids: counted and grouped through LDS histograms
constexpr int kColdMax = 2;
constexpr int64_t kColdBit = (int64_t)1 << 62;
// cold_pay[v] holds the (at most two) gradient rows of a cold group, (-1, -1) for any other group.
// A third value of its first word marks a group that the segment-sum stream left as block-edge
// partials: the optimizer kernel chains those itself and updates the row there.
constexpr int kEdgeMark = -2;
__device__ __forceinline__ int entry_vid(int64_t e) { return (int)(e >> 32) & 0x3fffffff; }
__device__ __forceinline__ bool entry_cold(int64_t e) { return (e & kColdBit) != 0; }
// per virtual id: (positions << 32) | start of its group in perm64
__device__ __forceinline__ bool group_cold(int v, int64_t grp) {
  return v >= kHotBins && (int)(grp >> 32) <= kColdMax;
}

// Status block in pinned, device-mapped Host memory: kernels write it, the host reads it without
// waiting for any stream (sfc_check, sfc_peek_stats and the first lines of every step call).
// The published counters are guarded by a sequence word: odd while a kernel is writing them.
struct HostStatus {
  int err;               // first device-side consistency check that fired (0 = none); never cleared
  int err_step;          // step of that check
  int bad_offsets_step;  // most recent step whose bag offsets were malformed (0 = none)
  int pad;
  int seq;               // 2 * step once that step's counters below are complete
  int U, n_hit, M, K, n_bypass, n_invalid, n_bad_offsets;
};

// Device counters of one cache.  Written by kernels only; the host reads a copy in get_stats.
struct Ctr {
  int U;          // unique ids of the batch
  int M;          // misses
  int K;          // victims
  int n_bypass;
  int n_hit;
  int n_invalid;
  int f;          // slots [0, f) are occupied, [f, C) have never been used
  int f_old;      // f before this step's inserts
  int need;       // misses that found no free slot
  int T;          // stamp threshold: stamp < T is evicted, stamp == T partly
  int r;          // how many slots with stamp == T are evicted (lowest slots first)
  int oldest;     // no occupied slot has a stamp below this
  int tomb;       // deleted entries in the cache index
  int rebuild;    // set when the index must be rebuilt before the next resolve
  int err;        // nonzero: a probe loop ran off its bound
  int fetch_on_main;  // pipelined mode: this step's Host copies ran behind the older steps' updates
  int U_prev;     // unique ids of the previous step (its per-tile tallies are still to be read)
  int dense;      // the id -> slot index is a dense map (no hashed entries, no tombstones, no rebuild)
  int t;          // number of the step these counters belong to
  int bad_offsets;    // violations found in the step's bag offsets (multi-hot input)
  HostStatus* hstat;  // device view of the cache's status block
};

// A device-side consistency check fired: remembered in the step's counters (every later step
// inherits it) and in the Host status block (plain stores over the link: if several checks fire
// together any one of their codes is kept, which is all the host needs to know).
__device__ __forceinline__ void flag_err(Ctr* ctr, int code) {
  ctr->err = code;
  volatile HostStatus* h = ctr->hstat;
  if (h) { h->err_step = ctr->t; h->err = code; }
}

// Entry of the per-step batch table: key and the smallest position that carries it, one 16-byte
// access for both.
struct __attribute__((aligned(16))) UEntry {
  int64_t key;    // id, kEmpty or kNullKey
  int32_t minpos; // kIntMax when unset
  int32_t pad;
};

struct __attribute__((aligned(16))) IdxEntry {
  int64_t key;    // id, kEmpty or kTomb
  int32_t slot;
  int32_t pad;
};

// murmur3 64-bit finaliser
__device__ __forceinline__ uint64_t mix64(uint64_t x) {
  x ^= x >> 33; x *= 0xff51afd7ed558ccdULL;
  x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ULL;
  x ^= x >> 33;
  return x;
}
// bucket in [0, n) without a power-of-two table: high half of a 32x32 product
__device__ __forceinline__ uint32_t bucket_of(int64_t key, uint32_t n) {
  return (uint32_t)(((mix64((uint64_t)key) >> 32) * (uint64_t)n) >> 32);
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

__device__ __forceinline__ int wave_incl_scan(int x) {
  const int lane = lane_id();
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    int y = __shfl_up(x, d, kWave);
    if (lane >= d) x += y;
  }
  return x;
}

__device__ __forceinline__ int wave_sum(int x) {
#pragma unroll
  for (int d = kWave / 2; d > 0; d >>= 1) x += __shfl_xor(x, d, kWave);
  return x;
}

// Exclusive scan of one int per thread over the block (blockDim.x multiple of 64, <= 1024).
// smem: at least 17 ints.  total = sum over the block.  Safe to call repeatedly.
__device__ __forceinline__ int block_excl_scan(int x, int& total, int* smem) {
  const int lane = lane_id(), w = (int)(threadIdx.x >> 6), nw = (int)(blockDim.x >> 6);
  int inc = wave_incl_scan(x);
  if (lane == kWave - 1) smem[w] = inc;
  __syncthreads();
  if (w == 0) {
    int s = lane < nw ? smem[lane] : 0;
    int si = wave_incl_scan(s);
    if (lane < nw) smem[lane] = si - s;   // exclusive prefix of the wave sums
    if (lane == nw - 1) smem[16] = si;
  }
  __syncthreads();
  int res = inc - x + smem[w];
  total = smem[16];
  __syncthreads();
  return res;
}

__device__ __forceinline__ int block_sum(int x, int* smem) {
  const int lane = lane_id(), w = (int)(threadIdx.x >> 6), nw = (int)(blockDim.x >> 6);
  x = wave_sum(x);
  if (lane == 0) smem[w] = x;
  __syncthreads();
  int s = 0;
  for (int i = 0; i < nw; ++i) s += smem[i];
  __syncthreads();
  return s;
}

}  // namespace sfc
