// Kernels of sfc_prepare: Virtual Sparse Id (batch unique with first-appearance order and the
// per-position inverse) and the MixCache manager (resolve against the index in HBM, victim
// selection by batch-granular LRU, slot assignment, index maintenance).
//
// Determinism: every output of sfc_prepare (unique ids, inverse, slots, miss and victim lists,
// cache state) is a function of the input sets and slot numbers only: their orders come from
// prefix scans over positions / virtual ids / slots, and atomics are used only where the result
// is order-free (min, counters, set insert).  The one thing that does follow the arrival order of
// atomics is internal: the order of a group's entries in perm64 (k_uniq_inverse ranks the
// positions of an id by the value its counting atomic returns).  It decides the order of an fp64
// sum, nothing else; see the segment-sum kernels for what that means for the results.
#pragma once
#include "sfc_device.h"

namespace sfc {

constexpr int kPosChunk = 2048;   // positions (or slots) per block in the scan passes
constexpr int kVidTile = 256;     // virtual ids per tile in resolve / assign
constexpr int kSortPer = 16;      // positions per thread in the count / group passes (8 and 32 measured slower)
constexpr int kSortChunk = 256 * kSortPer;

// ---------------------------------------------------------------------------------------------
// VSI pass 1: insert every position's id into the batch table (open addressing, linear probing,
// in HBM) and keep the smallest position per key; remember the table entry of each position.
//
// Same-address atomics serialise at the memory side (about 10 ns each on this chip), and the
// hottest id of a power-law batch owns a fifth of all positions.  So each block first
// deduplicates its kUniqChunk positions in an LDS table (key -> smallest position in the block) and
// only the distinct keys of the block go to HBM, up to four per thread in flight.  There a plain load
// comes first (the table entry of a key never changes once set, and a stale smallest-position
// word can only be too large), and an atomic is issued only when the load has not already seen
// the key / a small enough position.
// The kernel is launched twice: the first kHeadBlocks blocks, then the rest.  When all blocks
// start together they all find the table empty, and every block's copy of a frequent key goes
// through the claim / re-read / minimum atomics on one address (thousands in a row, about 10 ns
// each); after the head of the batch has been inserted the frequent keys are in the table with
// a smaller position than any later block holds, and the plain load settles them.
// hslot[p] = HBM table entry of position p; bit 31 marks the one position per (block, key) that
// can still be the key's first appearance, so the later passes test only those.
// ---------------------------------------------------------------------------------------------
constexpr int kUniqChunk = 512;    // positions per block (2048 with its 53 KB of LDS left 12 wavefronts per compute unit: 20 us slower)
constexpr int kUniqPer = kUniqChunk / 256;
constexpr int kLdsPer = 2 * kUniqChunk / 256;
constexpr int kHeadBlocks = 64;    // blocks of the first of the two launches
constexpr int kLdsTab = 2 * kUniqChunk;      // LDS table entries per block
constexpr unsigned kCandBit = 0x80000000u;

template <typename T>
__device__ __forceinline__ T coherent_load(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(256) void k_uniq_insert(const int64_t* __restrict__ ids, int n,
                                                      int64_t V, UEntry* utab, uint32_t hu,
                                                      int* __restrict__ hslot,
                                                      int* __restrict__ n_invalid, int block0) {
  __shared__ int64_t lkey[kLdsTab];
  __shared__ int lval[kLdsTab];               // smallest position of the key in this block; later its HBM entry
  __shared__ unsigned short lst[kUniqChunk];  // occupied LDS entries, compacted
  __shared__ unsigned cand[kUniqChunk / 32];  // bit per position of the block: block-local first of its key
  __shared__ int smem[20];
  for (int i = threadIdx.x; i < kLdsTab; i += 256) { lkey[i] = kEmpty; lval[i] = kIntMax; }
  if (threadIdx.x < kUniqChunk / 32) cand[threadIdx.x] = 0;
  __syncthreads();
  const int base = (block0 + (int)blockIdx.x) * kUniqChunk;
  int ls[kUniqPer];
  int64_t idv[kUniqPer];
#pragma unroll
  for (int j = 0; j < kUniqPer; ++j) {      // all loads in flight before the LDS work starts
    const int p = base + j * 256 + (int)threadIdx.x;
    idv[j] = p < n ? ids[p] : 0;
  }
#pragma unroll
  for (int j = 0; j < kUniqPer; ++j) {
    const int p = base + j * 256 + (int)threadIdx.x;
    bool invalid = false;
    ls[j] = 0;
    if (p < n) {
      int64_t key = idv[j];
      if (key < 0 || key >= V) { key = kNullKey; invalid = true; }
      uint32_t l = (uint32_t)mix64((uint64_t)key) & (kLdsTab - 1);
      for (int probes = 0; probes < kLdsTab; ++probes) {
        const int64_t k = lkey[l];
        if (k == key) break;
        if (k == kEmpty) {
          const int64_t old = (int64_t)atomicCAS((unsigned long long*)&lkey[l],
                                                 (unsigned long long)kEmpty, (unsigned long long)key);
          if (old == kEmpty || old == key) break;
        }
        l = (l + 1) & (kLdsTab - 1);
      }
      if (lval[l] > p) atomicMin(&lval[l], p);
      ls[j] = (int)l;
    }
    const uint64_t b = __ballot(invalid);
    if (b && lane_id() == 0) atomicAdd(n_invalid, __popcll(b));
  }
  __syncthreads();
  // compact the occupied entries (16 consecutive entries per thread)
  int nocc;
  {
    unsigned occ = 0;
#pragma unroll
    for (int k = 0; k < kLdsPer; ++k)
      if (lkey[threadIdx.x * kLdsPer + k] != kEmpty) occ |= 1u << k;
    int at = block_excl_scan(__popc(occ), nocc, smem);
#pragma unroll
    for (int k = 0; k < kLdsPer; ++k)
      if (occ & (1u << k)) lst[at++] = (unsigned short)(threadIdx.x * kLdsPer + k);
  }
  __syncthreads();
  // distinct keys of the block -> HBM table, four per thread in flight; one 16-byte load brings
  // the entry's key and its smallest position so far
  for (int i0 = threadIdx.x; i0 < nocc; i0 += 256 * 4) {
    int e[4], pm[4], m0[4];
    int64_t key[4], k0[4];
    uint32_t h[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * 256;
      e[u] = -1;
      if (i < nocc) {
        e[u] = lst[i];
        key[u] = lkey[e[u]];
        pm[u] = lval[e[u]];
        h[u] = bucket_of(key[u], hu);
        const int4 raw = *reinterpret_cast<const int4*>(&utab[h[u]]);
        k0[u] = ((int64_t)(uint32_t)raw.y << 32) | (uint32_t)raw.x;
        m0[u] = raw.z;
      }
    }
    // first probe: where the plain load saw an empty entry, try to claim it; all four in flight
    bool done[4], mine[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      mine[u] = false;
      done[u] = e[u] < 0 || k0[u] == key[u];
      if (!done[u] && k0[u] == kEmpty) {
        k0[u] = (int64_t)atomicCAS((unsigned long long*)&utab[h[u]].key, (unsigned long long)kEmpty,
                                   (unsigned long long)key[u]);
        m0[u] = kIntMax;          // whoever owns the entry now, its position word is re-read below
        mine[u] = k0[u] == kEmpty; // claimed by this thread: nothing to re-read, the atomic is due
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (done[u] || k0[u] == kEmpty || k0[u] == key[u]) continue;
      // the entry belongs to another key: walk on (rare at load factor <= 1/2)
      for (uint32_t probes = 0; probes < hu; ++probes) {
        h[u] = h[u] + 1 == hu ? 0 : h[u] + 1;
        int64_t k = coherent_load(&utab[h[u]].key);
        if (k == key[u]) break;
        if (k == kEmpty) {
          k = (int64_t)atomicCAS((unsigned long long*)&utab[h[u]].key, (unsigned long long)kEmpty,
                                 (unsigned long long)key[u]);
          if (k == kEmpty || k == key[u]) break;
        }
      }
      m0[u] = kIntMax;
    }
    // a plain load may be stale (too large), never too small: ask the memory side before the atomic
    int m1[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      m1[u] = mine[u] ? kIntMax
                      : ((e[u] >= 0 && m0[u] > pm[u]) ? coherent_load(&utab[h[u]].minpos) : 0);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (e[u] < 0) continue;
      if (m0[u] > pm[u] && m1[u] > pm[u]) atomicMin(&utab[h[u]].minpos, pm[u]);
      lval[e[u]] = (int)h[u];
      const int q = pm[u] - base;
      atomicOr(&cand[q >> 5], 1u << (q & 31));
    }
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kUniqPer; ++j) {
    const int q = j * 256 + (int)threadIdx.x;
    const int p = base + q;
    if (p < n) {
      const unsigned c = (cand[q >> 5] >> (q & 31)) & 1u;
      hslot[p] = (int)((unsigned)lval[ls[j]] | (c ? kCandBit : 0u));
    }
  }
}

// Rebuild of the cache index, second half (the first half empties it): every resident id goes
// back in.  Grid-stride over the occupied slots [0, f).
__device__ __forceinline__ void index_reinsert(IdxEntry* index, uint32_t hi,
                                               const int64_t* __restrict__ slot_id, int f) {
  for (int s = blockIdx.x * 256 + threadIdx.x; s < f; s += gridDim.x * 256) {
    const int64_t id = slot_id[s];
    if (id < 0) continue;
    uint32_t h = bucket_of(id, hi);
    for (uint32_t probes = 0; probes < hi; ++probes) {
      if (index[h].key == kEmpty &&
          (int64_t)atomicCAS((unsigned long long*)&index[h].key, (unsigned long long)kEmpty,
                             (unsigned long long)id) == kEmpty) {
        atomicExch(&index[h].slot, s);
        break;
      }
      h = h + 1 == hi ? 0 : h + 1;
    }
  }
}

// VSI pass 2: per chunk of positions, how many are the first appearance of their id.
__global__ __launch_bounds__(256) void k_uniq_count(const int* __restrict__ hslot,
                                                     const UEntry* __restrict__ utab, int n,
                                                     int* __restrict__ blk_cnt) {
  __shared__ int smem[20];
  const int base = blockIdx.x * kPosChunk + (int)threadIdx.x * 8;
  int c = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int p = base + j;
    if (p < n) {
      const unsigned hs = (unsigned)hslot[p];
      if ((hs & kCandBit) && utab[hs & ~kCandBit].minpos == p) ++c;
    }
  }
  const int tot = block_sum(c, smem);
  if (threadIdx.x == 0) blk_cnt[blockIdx.x] = tot;
}

// Starts the step's counters, once the previous step's prepare has run to its end: they inherit the
// cache-wide fields (watermark, oldest stamp, tombstones, rebuild flag, error) from the previous
// step's and start their own tallies at zero.  Steps in flight on the other streams keep reading
// their own copy.  n_invalid is the insert pass's tally of out-of-range positions, returned to
// zero here.
// The same launch empties the cache index when the previous step's plan asked for a rebuild (too
// many deleted entries); k_index_refill then puts every resident id back.  Both run between the
// last index update of one step and the resolve of the next.  They read the flag and the
// watermark from the previous step's counters, which no kernel changes any more (on the very
// first step prev == cur and both fields are zero before and after).
__device__ __forceinline__ void ctr_start(Ctr* cur, const Ctr* prev, const int* n_unique,
                                          int* n_invalid, int t) {
  Ctr c = *prev;
  c.U_prev = c.U;
  c.U = *n_unique;
  c.M = c.K = c.n_bypass = c.n_hit = 0;
  c.n_invalid = *n_invalid;
  *n_invalid = 0;
  c.f_old = c.f; c.need = 0; c.T = 0; c.r = 0; c.fetch_on_main = 0;
  c.t = t; c.bad_offsets = 0;
  *cur = c;
}

__global__ __launch_bounds__(256) void k_ctr_init(Ctr* cur, const Ctr* prev, const int* n_unique,
                                                  int* n_invalid, IdxEntry* index, uint32_t hi,
                                                  int t) {
  const bool rebuild = prev->rebuild != 0;
  if (blockIdx.x == 0 && threadIdx.x == 0) ctr_start(cur, prev, n_unique, n_invalid, t);
  if (!rebuild) return;
  IdxEntry e; e.key = kEmpty; e.slot = -1; e.pad = 0;
  for (uint32_t i = blockIdx.x * 256 + threadIdx.x; i < hi; i += gridDim.x * 256) index[i] = e;
}
__global__ __launch_bounds__(256) void k_index_refill(IdxEntry* index, uint32_t hi,
                                                       const int64_t* __restrict__ slot_id,
                                                       const Ctr* ctr) {
  if (ctr->rebuild) index_reinsert(index, hi, slot_id, ctr->f);
}

// VSI pass 3: the first appearances get their virtual ids (rank among all first appearances) and
// the tables keyed by them.  A chunk's first virtual id is the sum of the counts of the chunks
// before it, which every block adds up for itself (a few loads per thread from a list that sits in
// L2: cheaper than a scan kernel between the two passes).  The last chunk leaves the number of
// unique ids in *n_unique for k_ctr_init.
__global__ __launch_bounds__(256) void k_uniq_assign(const int* __restrict__ hslot,
                                                      const UEntry* __restrict__ utab, int n,
                                                      const int* __restrict__ blk_cnt,
                                                      int64_t* __restrict__ unique_ids,
                                                      int* __restrict__ uvid,
                                                      int* __restrict__ vid_hslot,
                                                      int* __restrict__ cnt, int* n_unique) {
  __shared__ int smem[20];
  int before = 0;
  for (int i = (int)threadIdx.x; i < (int)blockIdx.x; i += 256) before += blk_cnt[i];
  before = block_sum(before, smem);
  const int base = blockIdx.x * kPosChunk + (int)threadIdx.x * 8;
  int hs[8];
  unsigned flags = 0;
  int c = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int p = base + j;
    hs[j] = 0;
    if (p < n) {
      const unsigned raw = (unsigned)hslot[p];
      hs[j] = (int)(raw & ~kCandBit);
      if ((raw & kCandBit) && utab[hs[j]].minpos == p) { flags |= 1u << j; ++c; }
    }
  }
  int tot;
  int vid = block_excl_scan(c, tot, smem) + before;
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) *n_unique = before + tot;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    if (flags & (1u << j)) {
      const int64_t key = utab[hs[j]].key;
      unique_ids[vid] = key == kNullKey ? (int64_t)-1 : key;
      uvid[hs[j]] = vid;
      vid_hslot[vid] = hs[j];
      cnt[vid] = 0;
      ++vid;
    }
  }
}

// VSI pass 4: virtual id of every position, and cnt[v] = number of positions of virtual id v.
// For the ids outside the LDS range the atomic that counts a position also ranks it inside its
// group (rank[p]): the grouping pass then needs no atomic of its own for them.
// Virtual ids are handed out in order of first appearance, so the frequent ids of a power-law
// batch are (nearly all) among the lowest ones: those are counted in an LDS histogram per block
// and flushed with one coalesced atomic per bin; the rest go to HBM atomics on distinct words.
// Every block adds its tally of a frequent id to one counter: a thousand atomics in a row on one
// address (about 10 ns each).  The counters of the hot bins are therefore kept in kHotRep copies,
// block b using copy b mod kHotRep; resolve folds the copies into cnt, the miss assignment turns
// them into one group cursor per copy.
constexpr int kHotRep = 32;
constexpr int kFlushPer = 16;     // bins per thread and round when k_scatter flushes its LDS tallies

__global__ __launch_bounds__(256) void k_uniq_inverse(const int* __restrict__ hslot,
                                                       const int* __restrict__ uvid, int n,
                                                       int* __restrict__ inverse, int* cnt,
                                                       int* cnt_rep, int* __restrict__ rank) {
  __shared__ int lh[kHotBins];
  for (int i = threadIdx.x; i < kHotBins; i += 256) lh[i] = 0;
  __syncthreads();
  const int base = blockIdx.x * kSortChunk;
  int hv[kSortPer], vv[kSortPer];
#pragma unroll
  for (int j = 0; j < kSortPer; ++j) {          // kSortPer loads in flight per level of indirection
    const int p = base + j * 256 + (int)threadIdx.x;
    hv[j] = p < n ? (int)((unsigned)hslot[p] & ~kCandBit) : -1;
  }
#pragma unroll
  for (int j = 0; j < kSortPer; ++j) vv[j] = hv[j] >= 0 ? uvid[hv[j]] : -1;
#pragma unroll
  for (int j = 0; j < kSortPer; ++j) {
    const int p = base + j * 256 + (int)threadIdx.x;
    const int v = vv[j];
    if (v >= 0) {
      inverse[p] = v;
      if (v < kHotBins) atomicAdd(&lh[v], 1);
      else rank[p] = atomicAdd(&cnt[v], 1);      // arrival order inside the group, for k_scatter
    }
  }
  __syncthreads();
  int* mine = cnt_rep + (blockIdx.x & (kHotRep - 1)) * kHotBins;
  for (int b = threadIdx.x; b < kHotBins; b += 256) {
    const int c = lh[b];
    if (c) atomicAdd(&mine[b], c);
  }
}

// Multi-hot input: bag index of every position.  Also checks the bag structure (first offset 0,
// last offset n, none decreasing); violations are tallied in the step's counters and reported in
// the Host status block.  A malformed structure cannot make any kernel leave its buffers: ranges
// are clamped to [0, n] here and in the forward gather, and a position that no bag covers keeps a
// stale bag number, which the grouping pass clamps to the step's bags.
__global__ __launch_bounds__(256) void k_pos2bag(const int64_t* __restrict__ offsets, int n_bags,
                                                  int n, int* __restrict__ pos2bag, Ctr* ctr) {
  const int b = blockIdx.x * 256 + (int)threadIdx.x;
  bool bad = false;
  if (b < n_bags) {
    int64_t lo = offsets[b], hi = offsets[b + 1];
    bad = hi < lo || (b == 0 && lo != 0) || (b == n_bags - 1 && hi != n);
    if (lo < 0) lo = 0;
    if (hi > n) hi = n;
    for (int64_t q = lo; q < hi; ++q) pos2bag[q] = b;
  }
  const uint64_t m = __ballot(bad);
  if (m && lane_id() == 0) {
    atomicAdd(&ctr->bad_offsets, __popcll(m));
    volatile HostStatus* h = ctr->hstat;
    if (h) h->bad_offsets_step = ctr->t;
  }
}

// Grouping of positions by virtual id (counting sort): perm64[cursor[v]++] = (v << 32) | payload,
// payload = position (one-hot) or bag index (multi-hot).  cursor[v] starts at the exclusive scan
// of cnt.  Same LDS treatment of the low virtual ids as above; the others already carry their rank
// inside the group from the counting pass (rank_slot[p], the array this pass then overwrites with
// pos_slot[p]).  The order inside a group is the order in which the atomics land.
// Also writes pos_slot[p] = row of slot[inverse[p]] for the forward gather (a bypass slot C + j
// lives at row C + boff + j: each step in flight has its own bypass region).
__global__ __launch_bounds__(256) void k_scatter(const int* __restrict__ inverse,
                                                  const int* __restrict__ pos2bag, int n,
                                                  const int64_t* __restrict__ grp,
                                                  int* __restrict__ cold_pay,
                                                  int* cur_rep,
                                                  int64_t* __restrict__ perm64,
                                                  const int* __restrict__ slot,
                                                  int* rank_slot, int C, int boff, int n_bags) {
  __shared__ int lh[kHotBins];
  for (int i = threadIdx.x; i < kHotBins; i += 256) lh[i] = 0;
  __syncthreads();
  const int base = blockIdx.x * kSortChunk;
  int vv[kSortPer], rr[kSortPer], sv[kSortPer], cb[kSortPer], pay[kSortPer];
  unsigned coldm = 0;                       // bit j: position j of this thread belongs to a cold group
  // two levels of indirection, kSortPer loads in flight at each: position -> vid -> slot / group start
#pragma unroll
  for (int j = 0; j < kSortPer; ++j) {
    const int p = base + j * 256 + (int)threadIdx.x;
    vv[j] = p < n ? inverse[p] : -1;
    rr[j] = p < n ? rank_slot[p] : 0;           // meaningful for the ids outside the LDS range only
    pay[j] = (p < n && pos2bag) ? pos2bag[p] : p;
    // a position that malformed offsets left uncovered carries a stale bag number
    if (pos2bag && (unsigned)pay[j] >= (unsigned)n_bags) pay[j] = 0;
  }
#pragma unroll
  for (int j = 0; j < kSortPer; ++j) {
    sv[j] = vv[j] >= 0 ? slot[vv[j]] : -1;
    cb[j] = 0;
    if (vv[j] >= kHotBins) {
      const int64_t g = grp[vv[j]];
      cb[j] = (int)g;
      if (group_cold(vv[j], g)) coldm |= 1u << j;
    }
  }
  // the hot ids' ranks come from LDS; every group entry is written at the end
#pragma unroll
  for (int j = 0; j < kSortPer; ++j) {
    const int p = base + j * 256 + (int)threadIdx.x;
    if (vv[j] < 0) continue;
    rank_slot[p] = sv[j] >= C ? sv[j] + boff : sv[j];   // pos_slot: row index for the forward gather
    if (vv[j] < kHotBins) rr[j] = atomicAdd(&lh[vv[j]], 1);
    else {
      // a cold group's gradient rows also go where the optimizer kernel finds them without
      // walking the grouping: two words per virtual id, filled in the order of the ranks
      if ((coldm >> j) & 1u) cold_pay[2 * vv[j] + rr[j]] = pay[j];
      rr[j] += cb[j];
    }
  }
  __syncthreads();
  int* mine = cur_rep + (blockIdx.x & (kHotRep - 1)) * kHotBins;
  // the block's share of each non-empty bin's cursor: returning atomics, sixteen in flight per
  // thread (each round of them is a round trip to the memory side)
  static_assert(kHotBins % (256 * kFlushPer) == 0, "flush rounds cover the bins exactly");
  for (int b0 = threadIdx.x; b0 < kHotBins; b0 += 256 * kFlushPer) {
    int c[kFlushPer], r[kFlushPer];
#pragma unroll
    for (int u = 0; u < kFlushPer; ++u) c[u] = lh[b0 + u * 256];
#pragma unroll
    for (int u = 0; u < kFlushPer; ++u) r[u] = c[u] ? atomicAdd(&mine[b0 + u * 256], c[u]) : 0;
#pragma unroll
    for (int u = 0; u < kFlushPer; ++u) if (c[u]) lh[b0 + u * 256] = r[u];
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kSortPer; ++j)
    if (vv[j] >= 0) {
      const int at = vv[j] < kHotBins ? lh[vv[j]] + rr[j] : rr[j];
      perm64[at] = ((int64_t)vv[j] << 32) | (uint32_t)pay[j] | ((coldm >> j) & 1u ? kColdBit : (int64_t)0);
    }
}

// ---------------------------------------------------------------------------------------------
// The cache index (id -> slot) comes in two kinds.
//   dense: one int per Host row, dmap[id] = slot or -1.  With 288 GB of HBM a map of 4 bytes per
//     Host row (1.6 % of a dim-32 table with its accumulators) is affordable for every table that
//     fits a host, and it needs no probing, no atomics (the ids of a batch are distinct: one writer
//     per word), no tombstones and no rebuild.  The kernels below take it as `dmap`.
//   hashed (dmap == nullptr): open addressing, linear probing, tombstones, rebuilt on the device when
//     deleted entries pass an eighth of the table: for id ranges too large for a dense map, or on
//     request (sfc_config.index_kind).  The helpers that follow are its probe / insert.
// ---------------------------------------------------------------------------------------------
// A probe sequence is walked eight entries (128 bytes) at a time, all eight loads in flight
// together: the longest cluster among the tens of thousands of probes of a step sets the duration
// of the kernel, and a dependent load per entry made that tail tens of microseconds long.
constexpr int kProbeBatch = 8;

__device__ __forceinline__ int64_t idx_key(const int4& raw) {
  return ((int64_t)(uint32_t)raw.y << 32) | (uint32_t)raw.x;
}
__device__ __forceinline__ void idx_load_batch(const IdxEntry* index, uint32_t hi, uint32_t h,
                                               int4 (&raw)[kProbeBatch]) {
#pragma unroll
  for (int j = 0; j < kProbeBatch; ++j) {
    uint32_t hj = h + j;
    if (hj >= hi) hj -= hi;                  // hi >= 64: wraps at most once
    raw[j] = *reinterpret_cast<const int4*>(&index[hj]);
  }
}

__device__ __forceinline__ int index_find(const IdxEntry* __restrict__ index, uint32_t hi,
                                          int64_t id, uint32_t* where, Ctr* ctr) {
  uint32_t h = bucket_of(id, hi);
  for (uint32_t probes = 0; probes < hi; probes += kProbeBatch) {
    int4 raw[kProbeBatch];
    idx_load_batch(index, hi, h, raw);
#pragma unroll
    for (int j = 0; j < kProbeBatch; ++j) {
      const int64_t k = idx_key(raw[j]);
      if (k == id) {
        if (where) { uint32_t hj = h + j; *where = hj >= hi ? hj - hi : hj; }
        return raw[j].z;
      }
      if (k == kEmpty) return -1;
    }
    h += kProbeBatch;
    if (h >= hi) h -= hi;
  }
  flag_err(ctr, 1);
  return -1;
}

// id is known to be absent.  Takes the first empty or deleted entry of its probe sequence.
// Returns true if that was a deleted entry: the caller takes it off the tombstone count.
__device__ __forceinline__ bool index_insert(IdxEntry* index, uint32_t hi, int64_t id, int slot,
                                             Ctr* ctr) {
  uint32_t h = bucket_of(id, hi);
  for (uint32_t probes = 0; probes < hi; probes += kProbeBatch) {
    int4 raw[kProbeBatch];
    idx_load_batch(index, hi, h, raw);
#pragma unroll
    for (int j = 0; j < kProbeBatch; ++j) {
      const int64_t k = idx_key(raw[j]);
      if (k == kEmpty || k == kTomb) {
        uint32_t hj = h + j;
        if (hj >= hi) hj -= hi;
        // an entry seen free may have been taken by another insert since: then walk on
        const int64_t old = (int64_t)atomicCAS((unsigned long long*)&index[hj].key,
                                               (unsigned long long)k, (unsigned long long)id);
        if (old == k) {
          atomicExch(&index[hj].slot, slot);
          return k == kTomb;
        }
      }
    }
    h += kProbeBatch;
    if (h >= hi) h -= hi;
  }
  flag_err(ctr, 2);
  return false;
}

// ---------------------------------------------------------------------------------------------
// Resolve: each unique id against the index.  Hits get their slot and the current stamp.  The
// recency histogram hist[stamp] = #slots with that stamp must stay exact; stamps of hits cluster
// on the last few steps, i.e. on a few words of hist, so each block tallies its hits by age
// (t - old stamp) in LDS and adds its nonzero bins to age_hist, which the plan kernel applies
// to hist and returns to zero.  Only ages beyond the LDS range use an atomic on hist.  Bin 0
// counts the hits.  Also returns the batch-table entries of this step to the empty state, so that
// table never needs a per-step clear, and sums cnt per tile for the segment offsets.
// ---------------------------------------------------------------------------------------------
constexpr int kAgeBins = 1024;
constexpr int kResolveGrid = 256;

__global__ __launch_bounds__(256) void k_resolve(const int64_t* __restrict__ unique_ids,
                                                  const int* __restrict__ vid_hslot, UEntry* utab,
                                                  const IdxEntry* __restrict__ index, uint32_t hi,
                                                  const int* __restrict__ dmap,
                                                  int* stamp, int* hist, int t,
                                                  int* __restrict__ slot_out,
                                                  int* __restrict__ tile_miss,
                                                  int* __restrict__ cnt,
                                                  const int* __restrict__ cnt_rep,
                                                  int* __restrict__ tile_cnt,
                                                  int* __restrict__ age_hist, Ctr* ctr,
                                                  const Ctr* prev, const int* n_unique,
                                                  int* n_invalid) {
  __shared__ int smem[20];
  __shared__ int lage[kAgeBins];
  for (int i = threadIdx.x; i < kAgeBins; i += 256) lage[i] = 0;
  // Dense index (prev != nullptr): nothing has to happen between the previous step's prepare and
  // this kernel, so it starts the step's counters itself (k_ctr_init is not launched): the first
  // thread writes them for the kernels that follow, and every block takes the number of unique ids
  // from where the unique passes left it.  Nothing else of the counters is read in this kernel,
  // and the dense index has no probe that could flag an error into them meanwhile.
  const int U = prev ? *n_unique : ctr->U;
  __syncthreads();
  if (prev && blockIdx.x == 0 && threadIdx.x == 0) ctr_start(ctr, prev, n_unique, n_invalid, t);
  // four tiles per iteration, so that each level of the chain vid -> id -> index entry -> stamp
  // has four loads in flight per thread
  for (int tile0 = blockIdx.x * 4; tile0 * kVidTile < U; tile0 += gridDim.x * 4) {
    int hs[4], cc[4], sl[4], old[4];
    int64_t id[4];
    uint32_t hb[4];
    int4 ent[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int v = (tile0 + k) * kVidTile + (int)threadIdx.x;
      hs[k] = -1; cc[k] = 0; id[k] = -1;
      if (v < U) {
        hs[k] = vid_hslot[v]; id[k] = unique_ids[v];
        if (v < kHotBins) {                     // fold the copies of a hot bin
          int c = 0;
#pragma unroll
          for (int r = 0; r < kHotRep; ++r) c += cnt_rep[r * kHotBins + v];
          cnt[v] = c; cc[k] = c;
        } else {
          cc[k] = cnt[v];
        }
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (hs[k] >= 0) { UEntry z; z.key = kEmpty; z.minpos = kIntMax; z.pad = 0; utab[hs[k]] = z; }
      if (id[k] >= 0) {
        if (dmap) {
          ent[k].z = dmap[id[k]];
        } else {
          hb[k] = bucket_of(id[k], hi);
          ent[k] = *reinterpret_cast<const int4*>(&index[hb[k]]);
        }
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      sl[k] = -1;
      if (id[k] >= 0) {
        if (dmap) {
          sl[k] = ent[k].z;
        } else {
          const int64_t k0 = ((int64_t)(uint32_t)ent[k].y << 32) | (uint32_t)ent[k].x;
          if (k0 == id[k]) sl[k] = ent[k].z;
          else if (k0 != kEmpty) sl[k] = index_find(index, hi, id[k], nullptr, ctr);   // walk on
        }
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) old[k] = sl[k] >= 0 ? stamp[sl[k]] : 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int tile = tile0 + k;
      if (tile * kVidTile >= U) break;               // uniform over the block
      const int v = tile * kVidTile + (int)threadIdx.x;
      const bool hit = sl[k] >= 0, miss = id[k] >= 0 && sl[k] < 0;
      int age = 0;
      if (v < U) slot_out[v] = hit ? sl[k] : (miss ? kMissMark : -1);
      if (hit) {
        stamp[sl[k]] = t;
        age = t - old[k];
        if (age >= kAgeBins) atomicSub(&hist[old[k]], 1);
      }
      // most hits were last used one step ago: count those per wavefront, the rest one by one
      const uint64_t m1 = __ballot(hit && age == 1);
      if (m1 && lane_id() == 0) atomicAdd(&lage[1], __popcll(m1));
      if (hit && age > 1 && age < kAgeBins) atomicAdd(&lage[age], 1);
      const uint64_t mh = __ballot(hit);
      if (mh && lane_id() == 0) atomicAdd(&lage[0], __popcll(mh));
      const int nmiss = block_sum(miss ? 1 : 0, smem);
      const int csum = block_sum(cc[k], smem);
      if (threadIdx.x == 0) { tile_miss[tile] = nmiss; tile_cnt[tile] = csum; }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < kAgeBins; i += 256)
    if (lage[i]) atomicAdd(&age_hist[i], lage[i]);
}

// ---------------------------------------------------------------------------------------------
// Plan (one block): scan the per-tile miss counts, then decide the victims' stamp threshold from
// the recency histogram: need = M - free; T is the stamp at which the running count of
// evictable slots (stamp < limit, oldest first) passes need; r of the slots stamped T go too.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_plan(int* tile_miss, int* tile_cnt,
                                               int* __restrict__ age_hist,
                                               int* __restrict__ tile_reuse, int* hist, int t,
                                               int lookahead, int C, uint32_t hi, Ctr* ctr) {
  static_assert(kAgeBins == 1024, "one thread per age bin");
  __shared__ int smem[20];
  __shared__ int s_found;
  // every thread reads the counters here; thread 0 overwrites them only after the last barrier
  const int U = ctr->U;
  const int f = ctr->f;
  const int oldest = ctr->oldest;
  const int ntiles = (U + kVidTile - 1) / kVidTile;
  // deleted index entries that the previous step's miss assignment took back into use
  int reuse = 0;
  const int reuse_tiles = (ctr->U_prev + kVidTile - 1) / kVidTile;
  for (int i = (int)threadIdx.x; i < reuse_tiles; i += 1024) { reuse += tile_reuse[i]; tile_reuse[i] = 0; }
  reuse = block_sum(reuse, smem);
  // hits by age: thread a owns age a.  hist[t] gains the hits, hist[t - a] loses its share.
  {
    const int a = (int)threadIdx.x;
    const int sum = age_hist[a];
    age_hist[a] = 0;
    if (a == 0) { hist[t] += sum; ctr->n_hit = sum; }
    else if (sum) hist[t - a] -= sum;
  }
  __syncthreads();
  int carry = 0;
  for (int b = 0; b < ntiles; b += 1024) {
    const int i = b + (int)threadIdx.x;
    const int x = i < ntiles ? tile_miss[i] : 0;
    int tot;
    const int e = block_excl_scan(x, tot, smem);
    if (i < ntiles) tile_miss[i] = carry + e;
    carry += tot;
  }
  const int M = carry;
  carry = 0;
  for (int b = 0; b < ntiles; b += 1024) {
    const int i = b + (int)threadIdx.x;
    const int x = i < ntiles ? tile_cnt[i] : 0;
    int tot;
    const int e = block_excl_scan(x, tot, smem);
    if (i < ntiles) tile_cnt[i] = carry + e;
    carry += tot;
  }
  const int free_slots = C - f;
  const int need = M - free_slots;
  const int limit = t - lookahead;       // candidates have stamp < limit
  int T = limit, r = 0, K = 0;
  if (need > 0) {
    // running count of candidates from the oldest stamp upwards
    int cum = 0;           // slots with stamp in [oldest, b)
    bool done = false;
    for (int b = oldest; b < limit && !done; b += 1024) {
      if (threadIdx.x == 0) s_found = kIntMax;
      __syncthreads();
      const int s = b + (int)threadIdx.x;
      const int x = s < limit ? hist[s] : 0;
      int tot;
      const int e = block_excl_scan(x, tot, smem);
      // first stamp whose inclusive count exceeds need
      if (s < limit && cum + e + x > need) atomicMin(&s_found, s);
      __syncthreads();
      if (s_found != kIntMax) {
        T = s_found;
        if (s == T) smem[18] = cum + e;    // candidates strictly older than T
        __syncthreads();
        r = need - smem[18];
        K = need;
        done = true;
      } else {
        cum += tot;
      }
      __syncthreads();
    }
    if (!done) { T = limit; r = 0; K = cum; }   // everything evictable goes, the rest bypasses
    // the histogram after eviction: stamps below T vanish, r leave stamp T
    for (int s = oldest + (int)threadIdx.x; s < T; s += 1024) hist[s] = 0;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (need > 0 && r > 0) hist[T] -= r;
    int f_new = f + (M - K);
    if (f_new > C) f_new = C;
    const int n_bypass = M - K - (f_new - f);
    hist[t] += M - n_bypass;
    ctr->M = M; ctr->K = K; ctr->n_bypass = n_bypass;
    ctr->need = need; ctr->T = T; ctr->r = r;
    ctr->f_old = f; ctr->f = f_new;
    if (need > 0 && T > oldest) ctr->oldest = T;
    ctr->tomb -= reuse;
    // a rebuild asked for by the previous step has run ahead of this step's resolve
    if (ctr->rebuild) { ctr->rebuild = 0; ctr->tomb = 0; }
    // K deletions are about to add tombstones; ask for a rebuild before the next resolve when a
    // eighth of the index would be deleted entries
    if (!ctr->dense && (unsigned)(ctr->tomb + K) > hi / 8) ctr->rebuild = 1;
  }
}

// ---------------------------------------------------------------------------------------------
// Victim selection over the occupied slots, in slot order (two passes around a scan):
// victim  <=>  stamp < T, or stamp == T and fewer than r earlier slots carry stamp T.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_victim_count(const int* __restrict__ stamp,
                                                       int* __restrict__ tile_lt,
                                                       int* __restrict__ tile_eq, const Ctr* ctr) {
  __shared__ int smem[20];
  if (ctr->K == 0) return;
  const int f = ctr->f_old, T = ctr->T;
  for (int tile = blockIdx.x; tile * kPosChunk < f; tile += gridDim.x) {
    const int base = tile * kPosChunk + (int)threadIdx.x * 8;
    int lt = 0, eq = 0;
    if (base + 8 <= f) {
      const int4 a = *reinterpret_cast<const int4*>(stamp + base);
      const int4 b = *reinterpret_cast<const int4*>(stamp + base + 4);
      const int v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
      for (int j = 0; j < 8; ++j) { lt += v[j] < T; eq += v[j] == T; }
    } else {
      for (int j = 0; j < 8; ++j) {
        const int s = base + j;
        if (s < f) { const int st = stamp[s]; lt += st < T; eq += st == T; }
      }
    }
    // both counts in one block reduction: a tile has 2048 slots, so each fits in 16 bits
    const int both = block_sum((lt << 16) | eq, smem);
    if (threadIdx.x == 0) { tile_lt[tile] = both >> 16; tile_eq[tile] = both & 0xffff; }
  }
}

__global__ __launch_bounds__(256) void k_victim_write(const int* __restrict__ stamp,
                                                       const int64_t* __restrict__ slot_id,
                                                       const int* __restrict__ tile_lt,
                                                       const int* __restrict__ tile_eq,
                                                       int* __restrict__ victim_slot,
                                                       int64_t* __restrict__ victim_id, Ctr* ctr,
                                                       int* __restrict__ dmap) {
  __shared__ int smem[20];
  if (ctr->K == 0) return;
  const int f = ctr->f_old, T = ctr->T, r = ctr->r, K = ctr->K;
  // victims in the tiles before this block's current one: summed from the per-tile counts, and
  // carried on from tile to tile (each block reads every count at most once)
  int pre_lt = 0, pre_eq = 0, summed = 0;
  for (int tile = blockIdx.x; tile * kPosChunk < f; tile += gridDim.x) {
    {
      int a = 0, b = 0;
      for (int i = summed + (int)threadIdx.x; i < tile; i += 256) { a += tile_lt[i]; b += tile_eq[i]; }
      pre_lt += block_sum(a, smem);
      pre_eq += block_sum(b, smem);
      summed = tile;
    }
    const int base = tile * kPosChunk + (int)threadIdx.x * 8;
    unsigned mlt = 0, meq = 0;
    int lt = 0, eq = 0;
    int v[8];
    if (base + 8 <= f) {
      const int4 a = *reinterpret_cast<const int4*>(stamp + base);
      const int4 b = *reinterpret_cast<const int4*>(stamp + base + 4);
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = base + j < f ? stamp[base + j] : kIntMax;   // never a victim
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (v[j] < T) { mlt |= 1u << j; ++lt; }
      if (v[j] == T) { meq |= 1u << j; ++eq; }
    }
    // one scan for both counts: a tile has 2048 slots, so each prefix fits in 16 bits
    int tot;
    const int both = block_excl_scan((lt << 16) | eq, tot, smem);
    int lt_before = (both >> 16) + pre_lt;
    int eq_before = (both & 0xffff) + pre_eq;
    // list position of each victim among this thread's eight slots, then the resident ids with all
    // loads in flight (a thread rarely has more than one victim, but a dependent load per victim
    // inside this loop made the pass latency-bound)
    int idx[8];
    int64_t vid8[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool is_lt = mlt & (1u << j), is_eq = meq & (1u << j);
      idx[j] = -1;
      if (is_lt || (is_eq && eq_before < r)) {
        idx[j] = lt_before + (eq_before < r ? eq_before : r);
        if (idx[j] >= K) { idx[j] = -1; flag_err(ctr, 4); }     // never while hist mirrors the stamps
      }
      lt_before += is_lt;
      eq_before += is_eq;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) if (idx[j] >= 0) vid8[j] = slot_id[base + j];
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (idx[j] >= 0) {
        victim_slot[idx[j]] = base + j; victim_id[idx[j]] = vid8[j];
        if (dmap) dmap[vid8[j]] = -1;          // dense index: the victim leaves it here, one store
      }
  }
  // hashed index: the victims are deleted by the next pass (k_victim_unmap)
  if (!dmap && blockIdx.x == 0 && threadIdx.x == 0) atomicAdd(&ctr->tomb, ctr->K);
}

// The victims leave the index: one thread per victim.  A kernel of its own, before the inserts:
// with deletions and inserts in one kernel a resident id went missing from the index about once in
// a hundred steps at the target size (plain stores and memory-side atomics on neighbouring
// entries of one line from different XCDs); separated, and with every write to the index of a
// kernel that also uses atomics on it made an atomic itself, it has not been seen again.
__global__ __launch_bounds__(256) void k_victim_unmap(const int64_t* __restrict__ victim_id,
                                                       IdxEntry* index, uint32_t hi, Ctr* ctr) {
  const int K = ctr->K;
  for (int k = blockIdx.x * 256 + (int)threadIdx.x; k < K; k += gridDim.x * 256) {
    uint32_t where;
    if (index_find(index, hi, victim_id[k], &where, ctr) >= 0)
      atomicExch((unsigned long long*)&index[where].key, (unsigned long long)kTomb);
    else
      flag_err(ctr, 3);
  }
}

// ---------------------------------------------------------------------------------------------
// Assignment: the i-th miss in virtual-id order takes the i-th slot of (victims u free) in
// ascending slot order: victims (all below the watermark) first, then never-used slots from the
// watermark up, then transient bypass rows C + j.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_assign_misses(const int64_t* __restrict__ unique_ids,
                                                        const int* __restrict__ cnt,
                                                        int* __restrict__ cnt_rep,
                                                        int* __restrict__ cur_rep,
                                                        const int* __restrict__ tile_coff,
                                                        int64_t* __restrict__ grp,
                                                        int2* __restrict__ cold_pay,
                                                        const int* __restrict__ tile_moff,
                                                        const int* __restrict__ victim_slot,
                                                        int* __restrict__ slot_out,
                                                        int* __restrict__ miss_vids,
                                                        int* __restrict__ miss_row,
                                                        int64_t* __restrict__ miss_id, int boff,
                                                        int64_t* __restrict__ slot_id, int* stamp,
                                                        IdxEntry* index, uint32_t hi,
                                                        int* __restrict__ dmap, int t, int C,
                                                        int* __restrict__ tile_reuse, Ctr* ctr) {
  __shared__ int smem[20];
  const int U = ctr->U, K = ctr->K, f = ctr->f_old;
  const int free_slots = C - f;
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
    // The step's counters have been final since the plan: publish them to the Host status block
    // (sequence word odd while they are being written).  Here, in one thread of a wide kernel,
    // the two fences cost nothing that anyone waits for; in the single-block plan kernel they
    // lengthened the prepare by 6 us.
    volatile HostStatus* h = ctr->hstat;
    if (h) {
      h->seq = 2 * t - 1;
      __threadfence_system();
      h->U = U; h->n_hit = ctr->n_hit; h->M = ctr->M; h->K = K; h->n_bypass = ctr->n_bypass;
      h->n_invalid = ctr->n_invalid; h->n_bad_offsets = ctr->bad_offsets;
      __threadfence_system();
      h->seq = 2 * t;
    }
  }
  for (int tile = blockIdx.x; tile * kVidTile < U; tile += gridDim.x) {
    const int v = tile * kVidTile + (int)threadIdx.x;
    const bool miss = v < U && slot_out[v] == kMissMark;
    int tot;
    // start of the group of virtual id v in perm64 = exclusive scan of cnt
    const int nv = v < U ? cnt[v] : 0;
    const int off = block_excl_scan(nv, tot, smem) + tile_coff[tile];
    if (v < U) {
      grp[v] = ((int64_t)nv << 32) | (uint32_t)off;
      cold_pay[v] = make_int2(-1, -1);          // the grouping pass fills in the cold groups' rows
    }
    if (v < U && v < kHotBins) {                // one cursor per copy of a hot bin; copies back to zero
      int at = off;
#pragma unroll
      for (int r = 0; r < kHotRep; ++r) {
        const int c = cnt_rep[r * kHotBins + v];
        cur_rep[r * kHotBins + v] = at;
        at += c;
        cnt_rep[r * kHotBins + v] = 0;
      }
    }
    const int i = block_excl_scan(miss ? 1 : 0, tot, smem) + tile_moff[tile];
    bool reused = false;
    if (miss) {
      miss_vids[i] = v;
      int s;
      if (i < K) s = victim_slot[i];
      else if (i - K < free_slots) s = f + (i - K);
      else s = C + (i - K - free_slots);
      slot_out[v] = s;
      const int64_t id = unique_ids[v];
      miss_row[i] = s >= C ? s + boff : s;      // for the Host copies: cache row and Host row per miss
      miss_id[i] = id;
      if (s < C) {
        slot_id[s] = id;
        stamp[s] = t;
        if (dmap) dmap[id] = s;
        else reused = index_insert(index, hi, id, s, ctr);
      }
    }
    // deleted entries taken back into use: tallied per tile for the next plan pass (thousands of
    // atomics on one counter would serialise at the memory side, about 10 ns each)
    const int nre = block_sum(reused ? 1 : 0, smem);
    if (threadIdx.x == 0) tile_reuse[tile] = nre;
  }
}

// ---------------------------------------------------------------------------------------------
// Test aid (sfc_verify): recount of the manager state after a complete prepare.
//   bad[0]  occupied slots (below the watermark) whose id the index does not map to that slot
//   bad[1]  live index entries that do not point at a slot holding their id
//   bad[2]  words of the recency histogram that differ from the recount of the slots' stamps
//   bad[3]  live index entries (the host compares them with the number of occupied slots)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void tally(unsigned long long* word, int mine) {
  const int w = wave_sum(mine);
  if (w && lane_id() == 0) atomicAdd(word, (unsigned long long)w);
}

__global__ __launch_bounds__(256) void k_verify_slots(const int64_t* __restrict__ slot_id,
                                                       const int* __restrict__ stamp,
                                                       const IdxEntry* __restrict__ index,
                                                       uint32_t hi, const int* __restrict__ dmap,
                                                       int* recount, int hist_len,
                                                       unsigned long long* bad, Ctr* ctr) {
  const int f = ctr->f;
  const int rounds = (f + (int)gridDim.x * 256 - 1) / ((int)gridDim.x * 256);
  int s = blockIdx.x * 256 + (int)threadIdx.x;
  for (int it = 0; it < rounds; ++it, s += gridDim.x * 256) {   // every lane stays for the wave sums
    int lost = 0, off = 0;
    if (s < f) {
      const int64_t id = slot_id[s];
      if (id < 0 || (dmap ? dmap[id] : index_find(index, hi, id, nullptr, ctr)) != s) lost = 1;
      const int st = stamp[s];
      if (st >= 0 && st < hist_len) atomicAdd(&recount[st], 1); else off = 1;
    }
    tally(&bad[0], lost);
    tally(&bad[2], off);
  }
}

__global__ __launch_bounds__(256) void k_verify_entries(const IdxEntry* __restrict__ index,
                                                         uint32_t hi,
                                                         const int64_t* __restrict__ slot_id, int C,
                                                         unsigned long long* bad) {
  const uint32_t stride = gridDim.x * 256;
  const uint32_t rounds = (hi + stride - 1) / stride;
  uint32_t i = blockIdx.x * 256 + threadIdx.x;
  int live = 0, stray = 0;
  for (uint32_t it = 0; it < rounds; ++it, i += stride) {
    if (i < hi) {
      const int4 raw = *reinterpret_cast<const int4*>(&index[i]);
      const int64_t key = idx_key(raw);
      if (key >= 0) {
        ++live;
        if (raw.z < 0 || raw.z >= C || slot_id[raw.z] != key) ++stray;
      }
    }
  }
  tally(&bad[3], live);
  tally(&bad[1], stray);
}

// the same for the dense index: every entry >= 0 is live and must point at a slot holding its id
__global__ __launch_bounds__(256) void k_verify_dense(const int* __restrict__ dmap, int64_t V,
                                                       const int64_t* __restrict__ slot_id, int C,
                                                       unsigned long long* bad) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  const int64_t rounds = (V + stride - 1) / stride;
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  int live = 0, stray = 0;
  for (int64_t it = 0; it < rounds; ++it, i += stride) {
    if (i < V) {
      const int s = dmap[i];
      if (s >= 0) {
        ++live;
        if (s >= C || slot_id[s] != i) ++stray;
      }
    }
  }
  tally(&bad[3], live);
  tally(&bad[1], stray);
}

__global__ __launch_bounds__(256) void k_verify_hist(const int* __restrict__ hist,
                                                      const int* __restrict__ recount, int hist_len,
                                                      unsigned long long* bad) {
  const int stride = (int)gridDim.x * 256;
  const int rounds = (hist_len + stride - 1) / stride;
  int i = blockIdx.x * 256 + (int)threadIdx.x, off = 0;
  for (int it = 0; it < rounds; ++it, i += stride)
    if (i < hist_len && hist[i] != recount[i]) ++off;
  tally(&bad[2], off);
}

}  // namespace sfc
