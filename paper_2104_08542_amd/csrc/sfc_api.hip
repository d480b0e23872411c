// Host side of the C ABI declared in include/sfc.h: owns the device memory of one cache and
// enqueues the kernels of each step call on the caller's streams.  No call after
// sfc_cache_create allocates device memory or waits for the device, except the ones the header
// documents as synchronising.
//
// A step in flight is a StepCtx: the caller's buffers, the step's device counters, its grouping
// of positions, its victim list and its bypass region.  lookahead = L has L + 1 contexts.
// L = 0 runs the prepare on the main stream.  L >= 1 gives the prepare two streams of its own (one
// for the unique passes, one for the cache manager's kernels) and the Host copies run on the side
// stream, so that the prepare of step t+L, the copies of the step before it and lookup / update of
// step t overlap (the paper's pipeline of Data-Loader, Host-Manager and GPU-Worker stages); a
// larger L means more contexts, i.e. a prepare need not wait for the most recent update.  The
// Prefetch comparison strategy keeps its prepare on the side stream, ahead of its copies.
// Streams are ordered by events only; the host never waits.
#include "../../include/sfc.h"

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "sfc_prepare_kernels.h"
#include "sfc_row_kernels.h"

using namespace sfc;

namespace {

thread_local std::string g_err;
std::mutex g_host_mu;
std::map<void*, int64_t> g_host_allocs;     // pieces handed out by sfc_host_alloc and still alive

int fail(int code, const char* what, hipError_t e = hipSuccess) {
  char buf[512];
  if (e != hipSuccess) snprintf(buf, sizeof buf, "%s: %s", what, hipGetErrorString(e));
  else snprintf(buf, sizeof buf, "%s", what);
  g_err = buf;
  return code;
}

#define HIPCHK(call)                                            \
  do {                                                          \
    hipError_t e_ = (call);                                     \
    if (e_ != hipSuccess) return fail(SFC_EHIP, #call, e_);     \
  } while (0)

// Scratch of sfc_segment_sum_static: lives in the code object, one copy per GPU that loads the
// library, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the address that kernels and copies use is scratch_ptr[device].
static __device__ __align__(256) unsigned char scratch[SFC_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
void* scratch_ptr[kMaxDevices] = {};
std::mutex scratch_mu;

// The device address of `scratch` on the current device (looked up once per device).
int static_scratch(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) return fail(SFC_EINVAL, "device number out of range");
  std::lock_guard<std::mutex> lk(scratch_mu);
  if (!scratch_ptr[device]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(SFC_EHIP, "hipGetSymbolAddress(scratch)", e);
    scratch_ptr[device] = p;
  }
  *out = scratch_ptr[device];
  return SFC_OK;
}

// life of a step context
enum State { FREE = 0, PREPARED = 1, FETCHED = 2 };
enum { P_PREPARE = 0, P_FETCH = 1, P_LOOKUP = 2, P_BACKWARD = 3, P_SEG_STREAM = 4, P_SEG_FINISH = 5,
       P_ADAGRAD = 6, P_N = 7 };

struct EventPair {
  hipEvent_t a, b;
  bool extra = false;   // adds to the time of its call but is not a call of its own
};

struct StepCtx {
  int state = FREE;
  int t = 0;                          // step number
  int64_t n_ids = 0, n_bags = 0;
  const int64_t* d_offsets = nullptr; // caller's buffers of this step
  int64_t* d_unique = nullptr;
  int32_t *d_inverse = nullptr, *d_slot = nullptr, *d_miss = nullptr;
  Ctr* ctr = nullptr;                 // device counters of this step
  int64_t* perm64 = nullptr;          // [max_ids] positions grouped by virtual id
  int2* cold_pay = nullptr;           // [max_ids] per virtual id: the gradient rows of a cold group (-1 = none)
  int* pos_slot = nullptr;            // [max_ids] cache row of each position
  int* victim_slot = nullptr;         // [max_ids]
  int64_t* victim_id = nullptr;       // [max_ids]
  int* miss_row = nullptr;            // [max_ids] cache row of each miss (bypass rows already offset)
  int64_t* miss_id = nullptr;         // [max_ids] id of each miss
  int boff = 0;                       // bypass slot C + j lives at row C + boff + j
  hipEvent_t ev_prepared = nullptr;   // the step's prepare kernels have run
  hipEvent_t ev_fetched = nullptr;    // the side-stream launch of the step's Host copies has run
  bool updated = false;               // backward_update has been enqueued for this step
  bool discarded = false;             // freed by sfc_discard: the step's copies may still be running
  // pipelined mode: the second launch of the Host copies, due on the main stream behind the
  // update of step main_after (see k_swap_rows); older1 .. older3 = counters of the older steps
  // that were still in flight when the fetch was issued
  bool main_pending = false;
  int main_after = 0;
  const Ctr *older1 = nullptr, *older2 = nullptr, *older3 = nullptr;
  int chain = 0;
};

constexpr int kMaxCtx = 4;

}  // namespace

struct sfc_cache {
  sfc_config cfg{};
  int64_t C = 0, V = 0, max_ids = 0, max_bags = 0;
  int D = 0, d4 = 0, nctx = 1;
  hipStream_t st = nullptr, side = nullptr;     // main stream; stream of the Host copies
  hipStream_t prep = nullptr;                   // stream of the prepare kernels
  bool own_prep = false;                        // prep was created here (lookahead >= 1)
  // lookahead >= 1: the unique passes of a step (insert, count, scan, assign, inverse) run on a
  // stream of their own as soon as the previous step's resolve has emptied the batch table,
  // beside the rest of that step's prepare
  hipStream_t ins = nullptr;
  hipEvent_t ev_resolved = nullptr, ev_inserted = nullptr;
  bool resolved_once = false;                   // ev_resolved has been recorded
  hipEvent_t ev_tmp = nullptr;                  // cross-stream ordering inside one call
  // device memory
  float *cw = nullptr, *ca = nullptr;           // rows [(C + nctx * max_ids), D] and their optimizer state [.., S]
  int S = 0, s4 = 0;                            // floats / 16-byte chunks of optimizer state per row
  int64_t* slot_id = nullptr;                   // [C]
  int* stamp = nullptr;                         // [C]
  IdxEntry* index = nullptr; uint32_t hi = 0;   // cache index, hashed kind
  int* dmap = nullptr;                          // cache index, dense kind: [V] slot per id or -1 (else nullptr)
  int* hist = nullptr; int hist_len = 0;        // [max_steps + 2]
  UEntry* utab = nullptr; int* uvid = nullptr;  // batch table [2*max_ids]: key + first position; vid
  int* hslot = nullptr;                         // [max_ids]
  int* vid_hslot = nullptr;                     // [max_ids]
  int* blk_cnt = nullptr;                       // [max_ids / kPosChunk + 1]
  int *tile_lt = nullptr, *tile_eq = nullptr;   // [C / kPosChunk + 1]
  int* tile_miss = nullptr;                     // [max_ids / kVidTile + 1]
  // positions per virtual id [max_ids] and its copies for the lowest virtual ids [kHotRep, kHotBins]:
  // two sets, used by steps of even / odd number, so that the unique passes of a step can run
  // beside the previous step's miss assignment and grouping, which still read that step's counts
  int* cnt2[2] = {nullptr, nullptr};
  int* cnt_rep2[2] = {nullptr, nullptr};
  int64_t* grp = nullptr;                       // [max_ids] per virtual id: (positions << 32) | start of its group
  int* cur_rep = nullptr;                       // [kHotRep, kHotBins] group cursors of the lowest virtual ids, one per copy
  int* n_unique = nullptr;                      // unique ids of the step whose unique passes ran last
  int* pos2bag = nullptr;                       // [max_ids] multi-hot: bag of each position
  int* tile_cnt = nullptr;                      // [max_ids / kVidTile + 1]
  int* tile_reuse = nullptr;                    // [max_ids / kVidTile + 1] deleted index entries reused per tile
  int* n_invalid = nullptr;                     // out-of-range positions of the step being prepared
  int* age_hist = nullptr;                      // [kAgeBins] hits of the step by age, zero between steps
  double* bp = nullptr; int* bp_vid = nullptr;  // [2 * blocks, D] edge partial sums of k_seg_stream
  float* gsum = nullptr;                        // [max_ids, D] common gradients of the step
  float* warm_sink = nullptr;                   // one float that k_warm_rows never writes
  HostRows host{};                              // device view of the Host table
  HostStatus* hstat = nullptr;                  // pinned status block (host view); d_hstat its device view
  HostStatus* d_hstat = nullptr;
  int reported_bad_step = 0;                    // last malformed-offsets step that sfc_check has returned
  int device = 0;                               // the GPU this cache lives on
  std::vector<void*> allocs;
  // steps
  StepCtx ctx[kMaxCtx];
  int t = 0;                                    // steps prepared so far
  int last_prepared = -1;                       // context of the most recent sfc_prepare
  // profiling
  int prof = 0;                                 // 0 off, 1 step calls, 2 also the kernels inside them
  std::vector<EventPair> pending[P_N], spare;
  double ms_sum[P_N] = {};
  int64_t calls[P_N] = {};
};

namespace {

template <typename T>
int dalloc(sfc_cache* c, T** p, int64_t n) {
  if (n < 1) n = 1;
  void* q = nullptr;
  hipError_t e = hipMalloc(&q, (size_t)n * sizeof(T));
  if (e != hipSuccess) return fail(SFC_ENOMEM, "hipMalloc", e);
  c->allocs.push_back(q);
  *p = (T*)q;
  return SFC_OK;
}

template <typename T>
void fill(hipStream_t s, T* p, int64_t n, T v) {
  if (n <= 0) return;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(k_fill<T>, dim3((unsigned)blocks), dim3(256), 0, s, p, n, v);
}

int grid_for(int64_t items, int per_block, int cap) {
  int64_t b = (items + per_block - 1) / per_block;
  if (b < 1) b = 1;
  if (b > cap) b = cap;
  return (int)b;
}

bool prof_on(const sfc_cache* c, int which) { return c->prof >= (which > P_BACKWARD ? 2 : 1); }

int prof_begin(sfc_cache* c, int which, hipStream_t s, EventPair* ep) {
  if (!prof_on(c, which)) return SFC_OK;
  if (!c->spare.empty()) { *ep = c->spare.back(); c->spare.pop_back(); }
  else { HIPCHK(hipEventCreate(&ep->a)); HIPCHK(hipEventCreate(&ep->b)); }
  ep->extra = false;
  HIPCHK(hipEventRecord(ep->a, s));
  return SFC_OK;
}
// a pair of events for a timed launch (see LAUNCH_TIMED)
int prof_events(sfc_cache* c, EventPair* ep) {
  if (!c->spare.empty()) { *ep = c->spare.back(); c->spare.pop_back(); }
  else { HIPCHK(hipEventCreate(&ep->a)); HIPCHK(hipEventCreate(&ep->b)); }
  ep->extra = false;
  return SFC_OK;
}

// Launches a kernel; when profile entry `which` is on (and `timed`), the dispatch itself records
// the kernel's start and end in a pair of events, so the time read back is the kernel's own
// duration, as a profiler's kernel trace reports it, without the launch latency that a bracket
// of hipEventRecord calls around the launch would include.
#define LAUNCH_TIMED(c, which, timed, kernel, grid, block, s, ...) \
  LAUNCH_TIMED_X(c, which, timed, false, kernel, grid, block, s, __VA_ARGS__)
// extra: the kernel's time is added to the entry, but it is not a call of its own
#define LAUNCH_TIMED_X(c, which, timed, extra_, kernel, grid, block, s, ...)                     \
  do {                                                                                           \
    if ((timed) && prof_on(c, which)) {                                                          \
      EventPair ep_{};                                                                           \
      if (int rc_ = prof_events(c, &ep_)) return rc_;                                            \
      ep_.extra = (extra_);                                                                      \
      hipExtLaunchKernelGGL(kernel, grid, block, 0, s, ep_.a, ep_.b, 0, __VA_ARGS__);            \
      c->pending[which].push_back(ep_);                                                          \
    } else {                                                                                     \
      hipLaunchKernelGGL(kernel, grid, block, 0, s, __VA_ARGS__);                                \
    }                                                                                            \
  } while (0)

int prof_end(sfc_cache* c, int which, hipStream_t s, EventPair* ep) {
  if (!prof_on(c, which)) return SFC_OK;
  HIPCHK(hipEventRecord(ep->b, s));
  c->pending[which].push_back(*ep);
  return SFC_OK;
}
int prof_collect(sfc_cache* c) {
  for (int w = 0; w < P_N; ++w) {
    for (EventPair& ep : c->pending[w]) {
      float ms = 0.f;
      HIPCHK(hipEventSynchronize(ep.b));
      HIPCHK(hipEventElapsedTime(&ms, ep.a, ep.b));
      c->ms_sum[w] += ms;
      if (!ep.extra) c->calls[w] += 1;
      c->spare.push_back(ep);
    }
    c->pending[w].clear();
  }
  return SFC_OK;
}

// One read of pinned memory, no waiting: has a device-side consistency check fired?
int healthy(sfc_cache* c) {
  const volatile HostStatus* h = c->hstat;
  if (h && h->err) {
    // 1: a lookup walked the whole index, 2: so did an insert, 3: a victim was not in the index,
    // 4: more victims than the recency histogram promised
    char msg[128];
    snprintf(msg, sizeof msg, "cache manager state is inconsistent (device check %d at step %d)",
             h->err, h->err_step);
    return fail(SFC_ECORRUPT, msg);
  }
  return SFC_OK;
}

constexpr int kGridCap = 2048;   // blocks of the grid-stride kernels whose size lives on the device
constexpr int kRebuildGrid = 2048; // blocks of the two launches that only work when the index is rebuilt

// The step that lookup / segment_sum / backward_update act on: the oldest one whose rows are (or
// are about to be) in place and that has not been updated yet.
StepCtx* training_ctx(sfc_cache* c) {
  StepCtx* best = nullptr;
  for (int k = 0; k < c->nctx; ++k) {
    StepCtx* x = &c->ctx[k];
    if (x->state == FETCHED && !x->updated && (!best || x->t < best->t))
      best = x;
  }
  return best;
}

// The copies are bound by the host link: 32 blocks x 256 lanes x 16 bytes in flight saturate it
// (measured), and a wider grid only slows the kernels that run beside it on the other streams.
constexpr int kSwapBlocks = 32;
// A step that moves hundreds of megabytes over the link (a miss-dominated workload) is bound by
// the link whatever else runs: there a wider grid is worth its disturbance of the other streams
// (128 blocks: 16.3 against 18.6 ms per step with 4e6 misses of 128 bytes per step).  The host
// cannot know a step's misses without waiting, so it goes by the latest count the device has
// published in the status block, which is a step or two old.
constexpr int kSwapBlocksWide = 128;
constexpr int64_t kSwapWideBytes = (int64_t)256 << 20;

// One launch of the Host<->cache copies of a step on stream s (see k_swap_rows for the two
// launches of pipelined mode).
int launch_swap(sfc_cache* c, StepCtx* x, hipStream_t s, int main_variant) {
  EventPair ep{};
  int rc;
  // the copies read the step's counters, miss list and victim list: its prepare comes first
  if (s != c->prep) HIPCHK(hipStreamWaitEvent(s, x->ev_prepared, 0));
  if ((rc = prof_begin(c, P_FETCH, s, &ep))) return rc;
  ep.extra = main_variant != 0;          // the second launch of a step: same call
  const int64_t recent_bytes = (int64_t)((const volatile HostStatus*)c->hstat)->M * (c->d4 + c->s4) * 16;
  const int swap_blocks = recent_bytes > kSwapWideBytes ? kSwapBlocksWide : kSwapBlocks;
  hipLaunchKernelGGL(k_swap_rows, dim3(grid_for(x->n_ids * (c->d4 + c->s4), 256, swap_blocks)),
                     dim3(256), 0, s,
                     x->miss_row, x->miss_id, x->victim_id, (float4*)c->cw, (float4*)c->ca, c->host,
                     c->d4, c->s4, x->ctr, x->older1, x->older2, x->older3, x->chain, main_variant);
  HIPCHK(hipGetLastError());
  if ((rc = prof_end(c, P_FETCH, s, &ep))) return rc;
  if (main_variant) x->main_pending = false;
  else HIPCHK(hipEventRecord(x->ev_fetched, s));
  return SFC_OK;
}

// Before main-stream work that reads the step's rows: both launches of its copies come first.
int rows_ready(sfc_cache* c, StepCtx* x) {
  int rc;
  if (x->main_pending && (rc = launch_swap(c, x, c->st, 1))) return rc;
  if (c->side != c->st) HIPCHK(hipStreamWaitEvent(c->st, x->ev_fetched, 0));
  return SFC_OK;
}

// common[v] = segment sum of d_grad over the step's grouping: the stream, then the block-edge partials.
// bp / bp_vid: the block-edge partial sums and their virtual ids, 2 per block of the stream; timed:
// bracket the kernels with profiling events (which may have to be created).
// fused (sfc_backward_update with the Adagrad kernel): the stream passes over the cold groups and
// marks the groups it leaves as block-edge partials, and no finish kernel runs: the optimizer
// kernel chains the *n_slots partials itself.
int seg_launch(sfc_cache* c, StepCtx* x, const float* d_grad, float* d_common, double* bp,
               int* bp_vid, bool timed, bool fused, int* n_slots) {
  const int n = (int)x->n_ids;
  if (n_slots) *n_slots = 0;
  if (n <= 0) return SFC_OK;
  const SegGeom g = seg_geom(c->D, n);
  const int nblk = (g.waves + 3) / 4;
  auto kern = x->d_offsets ? (fused ? k_seg_stream<false, true> : k_seg_stream<false, false>)
                           : (fused ? k_seg_stream<true, true> : k_seg_stream<true, false>);
  LAUNCH_TIMED(c, P_SEG_STREAM, timed, kern, dim3(nblk), dim3(256), c->st, (const float4*)d_grad,
               (const int64_t*)x->perm64, n, c->d4, g.G, g.L, (float4*)d_common, bp, bp_vid,
               fused ? (int*)x->cold_pay : (int*)nullptr);
  if (n_slots) *n_slots = 2 * nblk;
  if (fused) return SFC_OK;
  LAUNCH_TIMED(c, P_SEG_FINISH, timed, k_seg_finish, dim3((unsigned)(2 * nblk)), dim3(256), c->st,
               (const double*)bp, (const int*)bp_vid, 2 * nblk, c->d4, (float4*)d_common);
  return SFC_OK;
}

int sync_all(sfc_cache* c) {
  HIPCHK(hipStreamSynchronize(c->st));
  if (c->side != c->st) HIPCHK(hipStreamSynchronize(c->side));
  if (c->prep != c->st && c->prep != c->side) HIPCHK(hipStreamSynchronize(c->prep));
  if (c->ins) HIPCHK(hipStreamSynchronize(c->ins));
  return SFC_OK;
}

}  // namespace

extern "C" {

const char* sfc_strerror(int code) {
  switch (code) {
    case SFC_OK: return "ok";
    case SFC_EINVAL: return "invalid argument";
    case SFC_ESTATE: return "call out of order";
    case SFC_EHIP: return "HIP runtime error";
    case SFC_ENOMEM: return "out of memory";
    case SFC_ELIMIT: return "step limit reached";
    case SFC_ECORRUPT: return "cache manager state inconsistent";
    default: return "unknown error";
  }
}
const char* sfc_last_error(void) { return g_err.c_str(); }

void* sfc_host_alloc(int64_t bytes) {
  void* p = nullptr;
  if (bytes <= 0) return nullptr;
  {
    // several large pinned pieces at once have crashed the runtime at the next kernel launch
    // (see the header): refuse that layout instead of handing it out
    std::lock_guard<std::mutex> lk(g_host_mu);
    int64_t total = bytes;
    bool other_large = false;
    for (auto& kv : g_host_allocs) { total += kv.second; other_large |= kv.second >= SFC_HOST_ALLOC_LARGE_BYTES; }
    if (other_large && bytes >= SFC_HOST_ALLOC_LARGE_BYTES && total > SFC_HOST_ALLOC_MAX_BYTES) {
      fail(SFC_ENOMEM, "sfc_host_alloc: a second large pinned piece would take the total beyond "
                       "SFC_HOST_ALLOC_MAX_BYTES; allocate the table as one interleaved piece");
      return nullptr;
    }
  }
  if (hipHostMalloc(&p, (size_t)bytes, hipHostMallocMapped | hipHostMallocPortable) != hipSuccess) {
    (void)hipGetLastError();
    fail(SFC_ENOMEM, "hipHostMalloc failed");
    return nullptr;
  }
  std::lock_guard<std::mutex> lk(g_host_mu);
  g_host_allocs[p] = bytes;
  return p;
}
void sfc_host_free(void* p) {
  if (!p) return;
  { std::lock_guard<std::mutex> lk(g_host_mu); g_host_allocs.erase(p); }
  (void)hipHostFree(p);
}

void sfc_cache_destroy(sfc_cache* c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->st);
  if (c->side != c->st) (void)hipStreamSynchronize(c->side);
  if (c->own_prep && c->prep) (void)hipStreamSynchronize(c->prep);
  if (c->ins) (void)hipStreamSynchronize(c->ins);
  for (int w = 0; w < P_N; ++w)
    for (EventPair& ep : c->pending[w]) { (void)hipEventDestroy(ep.a); (void)hipEventDestroy(ep.b); }
  for (EventPair& ep : c->spare) { (void)hipEventDestroy(ep.a); (void)hipEventDestroy(ep.b); }
  if (c->ev_tmp) (void)hipEventDestroy(c->ev_tmp);
  for (int k = 0; k < kMaxCtx; ++k) {
    if (c->ctx[k].ev_prepared) (void)hipEventDestroy(c->ctx[k].ev_prepared);
    if (c->ctx[k].ev_fetched) (void)hipEventDestroy(c->ctx[k].ev_fetched);
  }
  if (c->own_prep && c->prep) (void)hipStreamDestroy(c->prep);
  if (c->ins) (void)hipStreamDestroy(c->ins);
  if (c->ev_resolved) (void)hipEventDestroy(c->ev_resolved);
  if (c->ev_inserted) (void)hipEventDestroy(c->ev_inserted);
  for (void* p : c->allocs) (void)hipFree(p);
  if (c->hstat) (void)hipHostFree(c->hstat);
  delete c;
}

int sfc_cache_create(const sfc_config* cfg, sfc_cache** out) {
  if (!cfg || !out) return fail(SFC_EINVAL, "null config or output pointer");
  *out = nullptr;
  if (cfg->capacity_rows < 0 || cfg->dim <= 0 || cfg->dim % 4 || cfg->dim > 256)
    return fail(SFC_EINVAL, "capacity_rows must be >= 0 and dim a multiple of 4 in [4, 256]");
  if (cfg->policy != SFC_POLICY_LRU_BATCH && cfg->policy != SFC_POLICY_PREFETCH)
    return fail(SFC_EINVAL, "unknown policy");
  if (cfg->policy == SFC_POLICY_PREFETCH && (cfg->capacity_rows != 0 || cfg->lookahead != 1))
    return fail(SFC_EINVAL, "the Prefetch strategy needs capacity_rows = 0 and lookahead = 1");
  if (cfg->max_ids_per_batch < 1 || cfg->max_bags_per_batch < 1 || cfg->host_rows < 1)
    return fail(SFC_EINVAL, "max_ids_per_batch, max_bags_per_batch and host_rows must be >= 1");
  if (cfg->lookahead < 0 || cfg->lookahead > 3) return fail(SFC_EINVAL, "lookahead must be 0, 1, 2 or 3");
  if (cfg->lookahead > 0 && (!cfg->side_stream || cfg->side_stream == cfg->stream))
    return fail(SFC_EINVAL, "lookahead > 0 needs a side_stream different from stream");
  const int64_t nctx = cfg->lookahead + 1;
  if (cfg->capacity_rows + nctx * cfg->max_ids_per_batch >= (int64_t)1 << 31 ||
      cfg->max_ids_per_batch >= (int64_t)1 << 30 || cfg->max_bags_per_batch >= (int64_t)1 << 31)
    return fail(SFC_EINVAL, "capacity_rows + (lookahead + 1) * max_ids_per_batch must stay below 2^31");
  if (!cfg->h_weights || !cfg->h_acc) return fail(SFC_EINVAL, "null host table");
  if (((uintptr_t)cfg->h_weights | (uintptr_t)cfg->h_acc) & 15)
    return fail(SFC_EINVAL, "host table must be 16-byte aligned");
  if (cfg->host_row_stride && (cfg->host_row_stride < cfg->dim || cfg->host_row_stride % 4))
    return fail(SFC_EINVAL, "host_row_stride must be 0 or a multiple of 4 that is >= dim");
  if (cfg->max_steps < 0) return fail(SFC_EINVAL, "max_steps must be >= 0");
  if (cfg->optimizer < SFC_OPT_ADAGRAD || cfg->optimizer > SFC_OPT_ROWWISE_ADAGRAD)
    return fail(SFC_EINVAL, "unknown optimizer");
  if (cfg->index_kind < SFC_INDEX_AUTO || cfg->index_kind > SFC_INDEX_DENSE)
    return fail(SFC_EINVAL, "unknown index_kind");
  const int S = cfg->optimizer == SFC_OPT_ADAM ? 2 * cfg->dim
              : cfg->optimizer == SFC_OPT_ROWWISE_ADAGRAD ? 4 : cfg->dim;
  if (cfg->host_state_stride && (cfg->host_state_stride < S || cfg->host_state_stride % 4))
    return fail(SFC_EINVAL, "host_state_stride must be 0 or a multiple of 4 that is >= the state size");
  if (cfg->optimizer == SFC_OPT_ADAM &&
      !(cfg->beta1 >= 0.0 && cfg->beta1 < 1.0 && cfg->beta2 >= 0.0 && cfg->beta2 < 1.0))
    return fail(SFC_EINVAL, "Adam needs 0 <= beta1, beta2 < 1");

  sfc_cache* c = new (std::nothrow) sfc_cache;
  if (!c) return fail(SFC_ENOMEM, "host allocation failed");
  c->cfg = *cfg;
  c->C = cfg->capacity_rows; c->V = cfg->host_rows; c->D = cfg->dim; c->d4 = cfg->dim / 4;
  c->S = S; c->s4 = S / 4;
  c->max_ids = cfg->max_ids_per_batch; c->max_bags = cfg->max_bags_per_batch;
  c->nctx = (int)nctx;
  c->st = (hipStream_t)cfg->stream;
  c->side = cfg->side_stream ? (hipStream_t)cfg->side_stream : c->st;
  c->hist_len = (cfg->max_steps ? cfg->max_steps : (1 << 20)) + 2;
  (void)hipGetDevice(&c->device);
  const bool dense = cfg->index_kind == SFC_INDEX_DENSE ||
                     (cfg->index_kind == SFC_INDEX_AUTO &&
                      cfg->host_rows * (int64_t)sizeof(int) <= SFC_DENSE_INDEX_MAX_BYTES);
  if (!dense) {
    // four entries per possible resident id keep probe sequences short (HBM is plentiful); two
    // where four would not fit a 32-bit entry number
    int64_t h = 4 * (c->C + c->max_ids);
    if (h > (int64_t)0xF0000000LL) h = 2 * (c->C + c->max_ids);
    c->hi = (uint32_t)h;
  }
  if (c->hi < 64) c->hi = 64;

  int rc = SFC_OK;
  hipError_t e;
  void* dp = nullptr;
  if ((e = hipHostGetDevicePointer(&dp, cfg->h_weights, 0)) != hipSuccess) {
    rc = fail(SFC_EINVAL, "h_weights is not pinned device-mapped host memory", e); goto bad;
  }
  c->host.w = (float4*)dp;
  if ((e = hipHostGetDevicePointer(&dp, cfg->h_acc, 0)) != hipSuccess) {
    rc = fail(SFC_EINVAL, "h_acc is not pinned device-mapped host memory", e); goto bad;
  }
  c->host.a = (float4*)dp;
  c->host.hs4 = (cfg->host_row_stride ? cfg->host_row_stride : cfg->dim) / 4;
  c->host.has4 = (cfg->host_state_stride ? cfg->host_state_stride : S) / 4;
  // lookahead 0: prepare on the main stream; otherwise on two streams of its own, beside the Host
  // copies of the step before (the Prefetch strategy: on the side stream, ahead of its copies)
  c->prep = cfg->lookahead == 0 ? c->st : c->side;
  if (cfg->lookahead >= 1 && cfg->policy != SFC_POLICY_PREFETCH) {
    if ((e = hipStreamCreateWithFlags(&c->prep, hipStreamNonBlocking)) != hipSuccess) {
      c->prep = nullptr;
      rc = fail(SFC_EHIP, "hipStreamCreate", e); goto bad;
    }
    c->own_prep = true;
    if ((e = hipStreamCreateWithFlags(&c->ins, hipStreamNonBlocking)) != hipSuccess) {
      c->ins = nullptr;
      rc = fail(SFC_EHIP, "hipStreamCreate", e); goto bad;
    }
    if ((e = hipEventCreateWithFlags(&c->ev_resolved, hipEventDisableTiming)) != hipSuccess ||
        (e = hipEventCreateWithFlags(&c->ev_inserted, hipEventDisableTiming)) != hipSuccess) {
      rc = fail(SFC_EHIP, "hipEventCreate", e); goto bad;
    }
  }

  {
    void* hp = nullptr;
    if ((e = hipHostMalloc(&hp, sizeof(HostStatus), hipHostMallocMapped | hipHostMallocPortable)) != hipSuccess) {
      rc = fail(SFC_ENOMEM, "hipHostMalloc (status block)", e); goto bad;
    }
    c->hstat = (HostStatus*)hp;
    memset(c->hstat, 0, sizeof(HostStatus));
    if ((e = hipHostGetDevicePointer(&dp, hp, 0)) != hipSuccess) {
      rc = fail(SFC_EHIP, "hipHostGetDevicePointer (status block)", e); goto bad;
    }
    c->d_hstat = (HostStatus*)dp;
  }
  {
    const int64_t rows = c->C + nctx * c->max_ids;
    // the batch table of a step has max(2 * n_ids, 64) entries (see sfc_prepare)
    const int64_t hu = 2 * c->max_ids < 64 ? 64 : 2 * c->max_ids;
    if ((rc = dalloc(c, &c->cw, rows * c->D))) goto bad;
    if ((rc = dalloc(c, &c->ca, rows * c->S))) goto bad;
    if ((rc = dalloc(c, &c->slot_id, c->C))) goto bad;
    if ((rc = dalloc(c, &c->stamp, c->C))) goto bad;
    if ((rc = dalloc(c, &c->index, (int64_t)c->hi))) goto bad;
    if (dense && (rc = dalloc(c, &c->dmap, c->V))) goto bad;
    if ((rc = dalloc(c, &c->hist, (int64_t)c->hist_len))) goto bad;
    if ((rc = dalloc(c, &c->utab, hu))) goto bad;
    if ((rc = dalloc(c, &c->uvid, hu))) goto bad;
    if ((rc = dalloc(c, &c->hslot, c->max_ids))) goto bad;
    if ((rc = dalloc(c, &c->vid_hslot, c->max_ids))) goto bad;
    if ((rc = dalloc(c, &c->blk_cnt, c->max_ids / kPosChunk + 2))) goto bad;
    if ((rc = dalloc(c, &c->tile_lt, c->C / kPosChunk + 2))) goto bad;
    if ((rc = dalloc(c, &c->tile_eq, c->C / kPosChunk + 2))) goto bad;
    if ((rc = dalloc(c, &c->tile_miss, c->max_ids / kVidTile + 2))) goto bad;
    if ((rc = dalloc(c, &c->cnt2[0], c->max_ids))) goto bad;
    if ((rc = dalloc(c, &c->cnt2[1], c->max_ids))) goto bad;
    if ((rc = dalloc(c, &c->n_unique, 1))) goto bad;
    if ((rc = dalloc(c, &c->grp, c->max_ids))) goto bad;
    if ((rc = dalloc(c, &c->pos2bag, c->max_ids))) goto bad;
    if ((rc = dalloc(c, &c->tile_cnt, c->max_ids / kVidTile + 2))) goto bad;
    if ((rc = dalloc(c, &c->tile_reuse, c->max_ids / kVidTile + 2))) goto bad;
    if ((rc = dalloc(c, &c->age_hist, (int64_t)kAgeBins))) goto bad;
    if ((rc = dalloc(c, &c->n_invalid, 1))) goto bad;
    if ((rc = dalloc(c, &c->cnt_rep2[0], (int64_t)kHotRep * kHotBins))) goto bad;
    if ((rc = dalloc(c, &c->cnt_rep2[1], (int64_t)kHotRep * kHotBins))) goto bad;
    if ((rc = dalloc(c, &c->cur_rep, (int64_t)kHotRep * kHotBins))) goto bad;
    {
      const int64_t nw = seg_geom(c->D, c->max_ids).waves + 8;
      const int64_t nwmax = nw > kSegTargetWaves + 8 ? nw : kSegTargetWaves + 8;
      if ((rc = dalloc(c, &c->bp, 2 * nwmax * c->D))) goto bad;
      if ((rc = dalloc(c, &c->bp_vid, 2 * nwmax))) goto bad;
    }
    if ((rc = dalloc(c, &c->gsum, c->max_ids * c->D))) goto bad;
    if ((rc = dalloc(c, &c->warm_sink, 1))) goto bad;
    for (int k = 0; k < c->nctx; ++k) {
      StepCtx* x = &c->ctx[k];
      if ((rc = dalloc(c, &x->ctr, 1))) goto bad;
      if ((rc = dalloc(c, &x->perm64, c->max_ids))) goto bad;
      if ((rc = dalloc(c, &x->cold_pay, c->max_ids))) goto bad;
      if ((rc = dalloc(c, &x->pos_slot, c->max_ids))) goto bad;
      if ((rc = dalloc(c, &x->victim_slot, c->max_ids))) goto bad;
      if ((rc = dalloc(c, &x->victim_id, c->max_ids))) goto bad;
      if ((rc = dalloc(c, &x->miss_row, c->max_ids))) goto bad;
      if ((rc = dalloc(c, &x->miss_id, c->max_ids))) goto bad;
      x->boff = (int)(k * c->max_ids);
      if ((e = hipEventCreateWithFlags(&x->ev_prepared, hipEventDisableTiming)) != hipSuccess ||
          (e = hipEventCreateWithFlags(&x->ev_fetched, hipEventDisableTiming)) != hipSuccess) {
        rc = fail(SFC_EHIP, "hipEventCreate", e); goto bad;
      }
    }

    hipStream_t s = c->st;
    fill<int64_t>(s, c->slot_id, c->C, (int64_t)-1);
    fill<int>(s, c->stamp, c->C, 0);
    IdxEntry empty; empty.key = kEmpty; empty.slot = -1; empty.pad = 0;
    fill<IdxEntry>(s, c->index, (int64_t)c->hi, empty);
    if (dense) fill<int>(s, c->dmap, c->V, -1);
    fill<int>(s, c->hist, (int64_t)c->hist_len, 0);
    fill<int>(s, c->age_hist, (int64_t)kAgeBins, 0);
    fill<int>(s, c->n_invalid, 1, 0);
    fill<int>(s, c->cnt_rep2[0], (int64_t)kHotRep * kHotBins, 0);
    fill<int>(s, c->cnt_rep2[1], (int64_t)kHotRep * kHotBins, 0);
    fill<int>(s, c->n_unique, 1, 0);
    fill<int>(s, c->tile_reuse, c->max_ids / kVidTile + 2, 0);
    UEntry uempty; uempty.key = kEmpty; uempty.minpos = kIntMax; uempty.pad = 0;
    fill<UEntry>(s, c->utab, hu, uempty);
    Ctr z; memset(&z, 0, sizeof z); z.oldest = 1; z.hstat = c->d_hstat; z.dense = dense ? 1 : 0;
    for (int k = 0; k < c->nctx; ++k)
      if ((e = hipMemcpyAsync(c->ctx[k].ctr, &z, sizeof z, hipMemcpyHostToDevice, s)) != hipSuccess) {
        rc = fail(SFC_EHIP, "cache initialisation", e); goto bad;
      }
    if ((e = hipEventCreateWithFlags(&c->ev_tmp, hipEventDisableTiming)) != hipSuccess ||
        (e = hipStreamSynchronize(s)) != hipSuccess || (e = hipGetLastError()) != hipSuccess) {
      rc = fail(SFC_EHIP, "cache initialisation", e); goto bad;
    }
  }
  *out = c;
  return SFC_OK;
bad:
  sfc_cache_destroy(c);
  return rc;
}

int sfc_prepare(sfc_cache* c, const int64_t* d_ids, int64_t n_ids, const int64_t* d_offsets,
                int64_t n_bags, int64_t* d_unique_ids, int32_t* d_inverse, int32_t* d_slot,
                int32_t* d_miss_vids) {
  if (!c) return fail(SFC_EINVAL, "null cache");
  if (int hrc = healthy(c)) return hrc;
  if (n_ids < 0 || n_bags < 0 || n_ids > c->max_ids || n_bags > c->max_bags)
    return fail(SFC_EINVAL, "n_ids / n_bags out of range");
  if (!d_offsets && n_bags != n_ids) return fail(SFC_EINVAL, "one-hot input needs n_bags == n_ids");
  if (d_offsets && n_bags == 0 && n_ids > 0) return fail(SFC_EINVAL, "multi-hot input with ids but no bags");
  if ((n_ids > 0 && !d_ids) || !d_unique_ids || !d_inverse || !d_slot || !d_miss_vids)
    return fail(SFC_EINVAL, "null buffer");
  if (c->last_prepared >= 0 && c->ctx[c->last_prepared].state == PREPARED)
    return fail(SFC_ESTATE, "sfc_prepare twice without sfc_fetch_misses: missed rows would never arrive");
  if (c->t + 1 >= c->hist_len - 1) return fail(SFC_ELIMIT, "max_steps reached");

  StepCtx* x = nullptr;
  for (int k = 0; k < c->nctx; ++k)
    if (c->ctx[k].state == FREE) { x = &c->ctx[k]; break; }
  if (!x)
    return fail(SFC_ESTATE, "every step context holds a step that has not been updated: call "
                            "sfc_backward_update (or sfc_discard) first");
  StepCtx* prev = c->last_prepared >= 0 ? &c->ctx[c->last_prepared] : x;
  hipStream_t s = c->prep;
  if (s != c->st) {
    // the prepare stream must not overtake what the main stream has been given so far: the
    // producer of d_ids and the last update that read this context's buffers
    HIPCHK(hipEventRecord(c->ev_tmp, c->st));
    HIPCHK(hipStreamWaitEvent(s, c->ev_tmp, 0));
    // a context freed by sfc_discard: its copies may still be reading its lists
    if (x->discarded && s != c->side) HIPCHK(hipStreamWaitEvent(s, x->ev_fetched, 0));
    if (c->ins) {
      // The unique passes touch the batch table, the per-position table slots, the tally of
      // invalid ids, this step's set of counts, its context's position array and the caller's
      // buffers of this step: the previous step's prepare has finished with the shared ones once
      // its resolve has run, so they need not wait for that step's victim, assignment and
      // grouping passes (small grids that leave most of the GPU idle).
      HIPCHK(hipStreamWaitEvent(c->ins, c->ev_tmp, 0));
      if (x->discarded) HIPCHK(hipStreamWaitEvent(c->ins, x->ev_fetched, 0));
      if (c->resolved_once) HIPCHK(hipStreamWaitEvent(c->ins, c->ev_resolved, 0));
    }
  }
  hipStream_t su = c->ins ? c->ins : s;          // stream of the unique passes
  c->t += 1;
  x->t = c->t; x->state = PREPARED; x->updated = false; x->main_pending = false; x->discarded = false;
  x->n_ids = n_ids; x->n_bags = n_bags; x->d_offsets = d_offsets;
  x->d_unique = d_unique_ids; x->d_inverse = d_inverse; x->d_slot = d_slot; x->d_miss = d_miss_vids;
  c->last_prepared = (int)(x - c->ctx);
  int* const cnt = c->cnt2[x->t & 1];
  int* const cnt_rep = c->cnt_rep2[x->t & 1];

  EventPair ep{};
  int rc;
  if ((rc = prof_begin(c, P_PREPARE, s, &ep))) return rc;
  const int n = (int)n_ids;
  uint32_t hu = (uint32_t)(2 * n_ids);
  if (hu < 64) hu = 64;                       // the batch table is empty between steps: any size works
  const int nchunk = (n + kPosChunk - 1) / kPosChunk;
  if (n > 0) {
    const int nub = (n + kUniqChunk - 1) / kUniqChunk, head = nub < kHeadBlocks ? nub : kHeadBlocks;
    hipLaunchKernelGGL(k_uniq_insert, dim3(head), dim3(256), 0, su, d_ids, n, c->V, c->utab, hu,
                       c->hslot, c->n_invalid, 0);
    if (nub > head)
      hipLaunchKernelGGL(k_uniq_insert, dim3(nub - head), dim3(256), 0, su, d_ids, n, c->V, c->utab,
                         hu, c->hslot, c->n_invalid, head);
    hipLaunchKernelGGL(k_uniq_count, dim3(nchunk), dim3(256), 0, su, c->hslot, c->utab, n, c->blk_cnt);
    hipLaunchKernelGGL(k_uniq_assign, dim3(nchunk), dim3(256), 0, su, c->hslot, c->utab, n,
                       c->blk_cnt, d_unique_ids, c->uvid, c->vid_hslot, cnt, c->n_unique);
    hipLaunchKernelGGL(k_uniq_inverse, dim3((n + kSortChunk - 1) / kSortChunk), dim3(256), 0, su,
                       c->hslot, c->uvid, n, d_inverse, cnt, cnt_rep, x->pos_slot);
  } else {
    fill<int>(su, c->n_unique, 1, 0);
  }
  if (su != s) {
    HIPCHK(hipEventRecord(c->ev_inserted, su));
    HIPCHK(hipStreamWaitEvent(s, c->ev_inserted, 0));
  }
  // from here on behind the whole prepare of the previous step: the step's counters start from
  // that step's, the index is rebuilt if its plan asked for it
  // (a dense index is never rebuilt: k_resolve starts the counters itself, neither is launched)
  if (!c->dmap) {
    hipLaunchKernelGGL(k_ctr_init, dim3(kRebuildGrid), dim3(256), 0, s, x->ctr, prev->ctr,
                       c->n_unique, c->n_invalid, c->index, c->hi, x->t);
    hipLaunchKernelGGL(k_index_refill, dim3(kRebuildGrid), dim3(256), 0, s, c->index, c->hi, c->slot_id, x->ctr);
  }
  const int gr = grid_for(n, 4 * kVidTile, kResolveGrid);
  hipLaunchKernelGGL(k_resolve, dim3(gr), dim3(256), 0, s, d_unique_ids, c->vid_hslot, c->utab,
                     c->index, c->hi, c->dmap, c->stamp, c->hist, x->t, d_slot, c->tile_miss, cnt, cnt_rep,
                     c->tile_cnt, c->age_hist, x->ctr, c->dmap ? (const Ctr*)prev->ctr : (const Ctr*)nullptr,
                     (const int*)c->n_unique, c->n_invalid);
  if (c->ins) { HIPCHK(hipEventRecord(c->ev_resolved, s)); c->resolved_once = true; }
  // (after the resolve: it tallies into the step's counters, which that kernel may have started)
  if (n > 0 && d_offsets)
    hipLaunchKernelGGL(k_pos2bag, dim3((unsigned)((n_bags + 255) / 256)), dim3(256), 0, s,
                       d_offsets, (int)n_bags, n, c->pos2bag, x->ctr);
  hipLaunchKernelGGL(k_plan, dim3(1), dim3(1024), 0, s, c->tile_miss, c->tile_cnt, c->age_hist,
                     c->tile_reuse,
                     c->hist, x->t, c->cfg.lookahead, (int)c->C, c->hi, x->ctr);
  const int gs = grid_for(c->C, kPosChunk, kGridCap);
  hipLaunchKernelGGL(k_victim_count, dim3(gs), dim3(256), 0, s, c->stamp, c->tile_lt, c->tile_eq,
                     x->ctr);
  hipLaunchKernelGGL(k_victim_write, dim3(gs), dim3(256), 0, s, c->stamp, c->slot_id, c->tile_lt,
                     c->tile_eq, x->victim_slot, x->victim_id, x->ctr, c->dmap);
  const int gv = grid_for(n, kVidTile, kGridCap);
  if (!c->dmap)
    hipLaunchKernelGGL(k_victim_unmap, dim3(gv), dim3(256), 0, s, x->victim_id, c->index, c->hi,
                       x->ctr);
  hipLaunchKernelGGL(k_assign_misses, dim3(gv), dim3(256), 0, s, d_unique_ids, cnt, cnt_rep,
                     c->cur_rep, c->tile_cnt,
                     c->grp, x->cold_pay, c->tile_miss, x->victim_slot, d_slot, d_miss_vids, x->miss_row,
                     x->miss_id, x->boff, c->slot_id,
                     c->stamp, c->index, c->hi, c->dmap, x->t, (int)c->C, c->tile_reuse, x->ctr);
  if (n > 0)
    hipLaunchKernelGGL(k_scatter, dim3((n + kSortChunk - 1) / kSortChunk), dim3(256), 0, s, d_inverse,
                       d_offsets ? c->pos2bag : (const int*)nullptr, n, c->grp, (int*)x->cold_pay, c->cur_rep,
                       x->perm64, d_slot, x->pos_slot, (int)c->C, x->boff, (int)n_bags);
  HIPCHK(hipGetLastError());
  if ((rc = prof_end(c, P_PREPARE, s, &ep))) return rc;
  HIPCHK(hipEventRecord(x->ev_prepared, s));
  return SFC_OK;
}

int sfc_fetch_misses(sfc_cache* c) {
  if (!c) return fail(SFC_EINVAL, "null cache");
  if (int hrc = healthy(c)) return hrc;
  StepCtx* x = c->last_prepared >= 0 ? &c->ctx[c->last_prepared] : nullptr;
  if (!x || x->state != PREPARED) return fail(SFC_ESTATE, "sfc_fetch_misses needs a preceding sfc_prepare");
  // older steps whose update has not been enqueued yet: their bypass rows are not in the Host
  // table yet (k_swap_rows decides on the device which of its two launches does the work)
  x->older1 = x->older2 = x->older3 = nullptr;
  x->chain = 0; x->main_pending = false; x->main_after = 0;
  for (int k = 0; k < c->nctx && c->cfg.policy != SFC_POLICY_PREFETCH; ++k) {
    StepCtx* o = &c->ctx[k];
    if (o == x || o->state != FETCHED || o->updated) continue;
    if (o->t == x->t - 1) { x->older1 = o->ctr; x->chain = o->main_pending ? 1 : 0; }
    else if (o->t == x->t - 2) x->older2 = o->ctr;
    else if (o->t == x->t - 3) x->older3 = o->ctr;
    if (o->t > x->main_after) x->main_after = o->t;
  }
  if (c->side != c->st) {
    // everything the main stream has been given so far comes first: this step's prepare
    // (lookahead 0), older updates and their second launches
    HIPCHK(hipEventRecord(c->ev_tmp, c->st));
    HIPCHK(hipStreamWaitEvent(c->side, c->ev_tmp, 0));
  }
  int rc = launch_swap(c, x, c->side, 0);
  if (rc) return rc;
  x->main_pending = x->older1 || x->older2 || x->older3;
  x->state = FETCHED;
  return SFC_OK;
}

int sfc_lookup(sfc_cache* c, float* d_out) {
  if (!c) return fail(SFC_EINVAL, "null cache");
  if (int hrc = healthy(c)) return hrc;
  StepCtx* x = training_ctx(c);
  if (!x) return fail(SFC_ESTATE, "sfc_lookup needs sfc_prepare and sfc_fetch_misses first");
  if (x->n_bags > 0 && !d_out) return fail(SFC_EINVAL, "null output");
  if ((uintptr_t)d_out & 15) return fail(SFC_EINVAL, "output must be 16-byte aligned");
  int rc;
  if ((rc = rows_ready(c, x))) return rc;
  hipStream_t s = c->st;
  const int64_t total = x->n_bags * c->d4;
  if (total > 0) {
    // the rows of the batch into the memory-side cache first (returns at once when they are too many)
    LAUNCH_TIMED_X(c, P_LOOKUP, true, true, k_warm_rows, dim3(grid_for(x->n_ids * c->d4, 2048, kWarmGrid)),
                   dim3(256), s, (const int*)x->d_slot, (const float4*)c->cw, c->d4, (int)c->C, x->boff,
                   (const Ctr*)x->ctr, c->warm_sink, (const int4*)x->pos_slot, (int)(x->n_ids / 4));
    if (!x->d_offsets) {
      const int d4 = c->d4, sh = (d4 & (d4 - 1)) == 0 ? __builtin_ctz(d4) : -1;
      const int bpb = lookup_rows_per_block(d4);
      LAUNCH_TIMED(c, P_LOOKUP, true, k_lookup_onehot,
                   dim3((unsigned)((x->n_bags + bpb - 1) / bpb)), dim3(256), s,
                   (const int*)x->pos_slot, (const float4*)c->cw, (float4*)d_out, (int)x->n_bags, d4, sh, bpb);
    } else {
      const int G = 64 / c->d4 > 0 ? 64 / c->d4 : 1;          // bags per wavefront
      const int64_t per_block = 4 * (int64_t)G;
      LAUNCH_TIMED(c, P_LOOKUP, true, k_lookup_bags,
                   dim3((unsigned)((x->n_bags + per_block - 1) / per_block)), dim3(256), s,
                   x->d_offsets, (const int*)x->pos_slot, (const float4*)c->cw, (float4*)d_out,
                   (int)x->n_bags, c->d4, G, x->n_ids);
    }
  }
  HIPCHK(hipGetLastError());
  return SFC_OK;
}

int sfc_segment_sum(sfc_cache* c, const float* d_grad, float* d_common_grad) {
  if (!c) return fail(SFC_EINVAL, "null cache");
  if (int hrc = healthy(c)) return hrc;
  StepCtx* x = training_ctx(c);
  if (!x) return fail(SFC_ESTATE, "sfc_segment_sum needs sfc_prepare and sfc_fetch_misses first");
  if ((x->n_bags > 0 && !d_grad) || !d_common_grad) return fail(SFC_EINVAL, "null buffer");
  if (((uintptr_t)d_grad | (uintptr_t)d_common_grad) & 15) return fail(SFC_EINVAL, "buffers must be 16-byte aligned");
  int rc;
  if ((rc = rows_ready(c, x))) return rc;
  if ((rc = seg_launch(c, x, d_grad, d_common_grad, c->bp, c->bp_vid, true, false, nullptr))) return rc;
  HIPCHK(hipGetLastError());
  return SFC_OK;
}

int sfc_segment_sum_static(sfc_cache* c, const float* d_grad, float* d_common_grad) {
  if (!c) return fail(SFC_EINVAL, "null cache");
  if (int hrc = healthy(c)) return hrc;
  StepCtx* x = training_ctx(c);
  if (!x) return fail(SFC_ESTATE, "sfc_segment_sum_static needs sfc_prepare and sfc_fetch_misses first");
  if ((x->n_bags > 0 && !d_grad) || !d_common_grad) return fail(SFC_EINVAL, "null buffer");
  if (((uintptr_t)d_grad | (uintptr_t)d_common_grad) & 15) return fail(SFC_EINVAL, "buffers must be 16-byte aligned");
  int dev = -1;
  HIPCHK(hipGetDevice(&dev));
  if (dev != c->device) return fail(SFC_EINVAL, "the cache lives on another device than the current one");
  // the scratch the step needs: per block of the stream two fp64 rows and two virtual ids
  const SegGeom g = seg_geom(c->D, x->n_ids > 0 ? x->n_ids : 1);
  const int64_t nblk = (g.waves + 3) / 4;
  const int64_t sums = 2 * nblk * c->D * (int64_t)sizeof(double);
  const int64_t need = sums + 2 * nblk * (int64_t)sizeof(int);
  if (need > (int64_t)SFC_STATIC_SCRATCH_BYTES) {
    char msg[160];
    snprintf(msg, sizeof msg, "sfc_segment_sum_static: this step needs %lld bytes of scratch, the "
             "fixed array holds %d", (long long)need, (int)SFC_STATIC_SCRATCH_BYTES);
    return fail(SFC_ELIMIT, msg);
  }
  void* base = nullptr;
  int rc;
  if ((rc = static_scratch(dev, &base))) return rc;
  // both launches of the step's copies must have been issued already: issuing the second one here
  // could create profiling events
  if (x->main_pending)
    return fail(SFC_ESTATE, "the step's rows are still due on the main stream: call sfc_lookup first");
  if (c->side != c->st) HIPCHK(hipStreamWaitEvent(c->st, x->ev_fetched, 0));
  // every slot that k_seg_finish reads is written by k_seg_stream in the same call: nothing to clear
  double* bp = (double*)base;
  int* bp_vid = (int*)((unsigned char*)base + sums);
  if ((rc = seg_launch(c, x, d_grad, d_common_grad, bp, bp_vid, false, false, nullptr))) return rc;
  HIPCHK(hipGetLastError());
  return SFC_OK;
}

int sfc_backward_update(sfc_cache* c, const float* d_grad) {
  if (!c) return fail(SFC_EINVAL, "null cache");
  if (int hrc = healthy(c)) return hrc;
  StepCtx* x = training_ctx(c);
  if (!x) return fail(SFC_ESTATE, "sfc_backward_update needs sfc_prepare and sfc_fetch_misses first");
  if (x->n_bags > 0 && !d_grad) return fail(SFC_EINVAL, "null gradient");
  if ((uintptr_t)d_grad & 15) return fail(SFC_EINVAL, "gradient must be 16-byte aligned");
  int rc;
  if ((rc = rows_ready(c, x))) return rc;
  hipStream_t s = c->st;
  EventPair ep{};
  if ((rc = prof_begin(c, P_BACKWARD, s, &ep))) return rc;
  int n_slots = 0;
  // Adagrad and Adam: the update kernel sums the cold groups and chains the block-edge partials itself
  const bool fused = c->cfg.optimizer == SFC_OPT_ADAGRAD || c->cfg.optimizer == SFC_OPT_ADAM;
  if ((rc = seg_launch(c, x, d_grad, c->gsum, c->bp, c->bp_vid, true, fused, &n_slots))) return rc;
  if (c->cfg.policy == SFC_POLICY_PREFETCH) {
    // the copies of a newer step issued so far read the Host table before this update writes it
    for (int k = 0; k < c->nctx; ++k) {
      StepCtx* y = &c->ctx[k];
      if (y != x && y->state == FETCHED && !y->updated && y->t > x->t)
        HIPCHK(hipStreamWaitEvent(s, y->ev_fetched, 0));
    }
  }
  const dim3 ug(grid_for(x->n_ids * c->d4, 1024, kGridCap));
  // the stream above passed over the cold groups and left the block-edge partials unchained:
  // the fused kernels sum both themselves (their first blocks chain the partials, a lane group per slot)
  const int n_edge = edge_blocks(n_slots, c->d4);
  if (c->cfg.optimizer == SFC_OPT_ADAGRAD) {
    auto kern = x->d_offsets ? k_adagrad_rows<false> : k_adagrad_rows<true>;
    LAUNCH_TIMED(c, P_ADAGRAD, true, kern, dim3(ug.x + (unsigned)n_edge), dim3(256), s, (const float4*)c->gsum,
                 (const int*)x->d_slot, (const int64_t*)x->d_unique, (float4*)c->cw, (float4*)c->ca,
                 c->host, (int)c->C, x->boff, c->cfg.lr, c->cfg.eps, c->d4, (const Ctr*)x->ctr,
                 (const int2*)x->cold_pay, (const float4*)d_grad, (const double*)c->bp,
                 (const int*)c->bp_vid, n_slots, n_edge);
  } else if (c->cfg.optimizer == SFC_OPT_ADAM) {
    // every constant derived from the decay rates is computed in double and rounded to fp32 once
    AdamArgs k;
    k.b1 = (float)c->cfg.beta1; k.c1 = (float)(1.0 - c->cfg.beta1);
    k.b2 = (float)c->cfg.beta2; k.c2 = (float)(1.0 - c->cfg.beta2);
    k.bc1 = (float)(1.0 - pow(c->cfg.beta1, (double)x->t));
    k.bc2 = (float)(1.0 - pow(c->cfg.beta2, (double)x->t));
    k.lr = c->cfg.lr; k.eps = c->cfg.eps;
    auto kern = x->d_offsets ? k_adam_rows<false> : k_adam_rows<true>;
    LAUNCH_TIMED(c, P_ADAGRAD, true, kern, dim3(ug.x + (unsigned)n_edge), dim3(256), s, (const float4*)c->gsum,
                 (const int*)x->d_slot, (const int64_t*)x->d_unique, (float4*)c->cw, (float4*)c->ca,
                 c->host, (int)c->C, x->boff, k, c->d4, (const Ctr*)x->ctr,
                 (const int2*)x->cold_pay, (const float4*)d_grad, (const double*)c->bp,
                 (const int*)c->bp_vid, n_slots, n_edge);
  } else {
    const int pow2 = (c->d4 & (c->d4 - 1)) == 0;
    LAUNCH_TIMED(c, P_ADAGRAD, true, k_rowwise_adagrad_rows, ug, dim3(256), s,
                 (const float4*)c->gsum, (const int*)x->d_slot, (const int64_t*)x->d_unique,
                 (float4*)c->cw, (float4*)c->ca, c->host, (int)c->C, x->boff, c->cfg.lr, c->cfg.eps,
                 c->d4, pow2, (const Ctr*)x->ctr);
  }
  HIPCHK(hipGetLastError());
  if ((rc = prof_end(c, P_BACKWARD, s, &ep))) return rc;
  x->updated = true;
  x->state = FREE;
  // second launches of the copies of newer steps that had to stay behind this update, oldest first
  for (int pass = 0; pass < c->nctx; ++pass) {
    StepCtx* y = nullptr;
    for (int k = 0; k < c->nctx; ++k) {
      StepCtx* z = &c->ctx[k];
      if (z->state == FETCHED && z->main_pending && z->main_after <= x->t && (!y || z->t < y->t)) y = z;
    }
    if (!y) break;
    if ((rc = launch_swap(c, y, s, 1))) return rc;
  }
  return SFC_OK;
}

int sfc_flush(sfc_cache* c) {
  if (!c) return fail(SFC_EINVAL, "null cache");
  for (int k = 0; k < c->nctx; ++k)
    if (c->ctx[k].state == PREPARED || (c->ctx[k].state == FETCHED && c->ctx[k].main_pending))
      return fail(SFC_ESTATE, "sfc_flush while a prepared step still waits for its rows");
  int rc = sync_all(c);
  if (rc) return rc;
  if (c->last_prepared < 0) return SFC_OK;
  hipLaunchKernelGGL(k_flush, dim3(grid_for(c->C * 2 * c->d4, 256, kGridCap)), dim3(256), 0, c->st,
                     c->slot_id, (const float4*)c->cw, (const float4*)c->ca, c->host, c->d4, c->s4,
                     c->ctx[c->last_prepared].ctr);
  HIPCHK(hipGetLastError());
  return sync_all(c);
}

int sfc_get_stats(sfc_cache* c, sfc_stats* h_out) {
  if (!c || !h_out) return fail(SFC_EINVAL, "null argument");
  int rc = sync_all(c);
  if (rc) return rc;
  memset(h_out, 0, sizeof *h_out);
  if (c->last_prepared < 0) return SFC_OK;
  Ctr h;
  HIPCHK(hipMemcpy(&h, c->ctx[c->last_prepared].ctr, sizeof h, hipMemcpyDeviceToHost));
  if (h.err) {
    char msg[96];
    snprintf(msg, sizeof msg, "cache manager state is inconsistent (device check %d)", h.err);
    return fail(SFC_ECORRUPT, msg);
  }
  const int64_t rowbytes = (int64_t)sizeof(float) * (c->D + c->S);
  h_out->n_unique = h.U; h_out->n_hit = h.n_hit; h_out->n_miss = h.M; h_out->n_evict = h.K;
  h_out->n_bypass = h.n_bypass; h_out->n_invalid = h.n_invalid;
  h_out->h2d_bytes = h.M * rowbytes;
  h_out->d2h_bytes = ((int64_t)h.K + h.n_bypass) * rowbytes;
  h_out->n_bad_offsets = h.bad_offsets;
  return SFC_OK;
}

int sfc_check(sfc_cache* c) {
  if (!c) return fail(SFC_EINVAL, "null cache");
  if (int hrc = healthy(c)) return hrc;
  const int bad = ((const volatile HostStatus*)c->hstat)->bad_offsets_step;
  if (bad > c->reported_bad_step) {
    c->reported_bad_step = bad;
    char msg[96];
    snprintf(msg, sizeof msg, "malformed bag offsets in step %d (most recent such step)", bad);
    return fail(SFC_EINVAL, msg);
  }
  return SFC_OK;
}

int sfc_peek_stats(sfc_cache* c, sfc_stats* h_out, int64_t* h_step) {
  if (!c || !h_out || !h_step) return fail(SFC_EINVAL, "null argument");
  const volatile HostStatus* h = c->hstat;
  memset(h_out, 0, sizeof *h_out);
  *h_step = 0;
  // the kernel that publishes makes the sequence word odd, writes, makes it even: take a copy
  // that has the same even sequence word before and after
  for (int tries = 0; tries < 1000; ++tries) {
    const int s1 = h->seq;
    if (s1 & 1) continue;
    std::atomic_thread_fence(std::memory_order_acquire);
    const int U = h->U, nh = h->n_hit, M = h->M, K = h->K, nb = h->n_bypass, ni = h->n_invalid,
              bo = h->n_bad_offsets;
    std::atomic_thread_fence(std::memory_order_acquire);
    if (h->seq != s1) continue;
    const int64_t rowbytes = (int64_t)sizeof(float) * (c->D + c->S);
    h_out->n_unique = U; h_out->n_hit = nh; h_out->n_miss = M; h_out->n_evict = K;
    h_out->n_bypass = nb; h_out->n_invalid = ni; h_out->n_bad_offsets = bo;
    h_out->h2d_bytes = M * rowbytes;
    h_out->d2h_bytes = ((int64_t)K + nb) * rowbytes;
    *h_step = s1 / 2;
    return SFC_OK;
  }
  return fail(SFC_EHIP, "status block kept changing");
}

int sfc_discard(sfc_cache* c) {
  if (!c) return fail(SFC_EINVAL, "null cache");
  StepCtx* x = training_ctx(c);
  if (!x) return fail(SFC_ESTATE, "no fetched step to give up");
  if (x->main_pending)
    return fail(SFC_ESTATE, "the step's copies wait for an older update: it cannot be given up yet");
  x->state = FREE;
  x->discarded = true;
  return SFC_OK;
}

int sfc_verify(sfc_cache* c, int64_t* h_bad) {
  if (!c || !h_bad) return fail(SFC_EINVAL, "null argument");
  for (int k = 0; k < c->nctx; ++k)
    if (c->ctx[k].state == PREPARED)
      return fail(SFC_ESTATE, "sfc_verify while a prepared step still waits for its rows");
  int rc = sync_all(c);
  if (rc) return rc;
  for (int k = 0; k < 4; ++k) h_bad[k] = 0;
  if (c->last_prepared < 0) return SFC_OK;
  int* recount = nullptr;
  unsigned long long* d_bad = nullptr;
  HIPCHK(hipMalloc((void**)&recount, (size_t)c->hist_len * sizeof(int)));
  if (hipMalloc((void**)&d_bad, 4 * sizeof(unsigned long long)) != hipSuccess) {
    (void)hipFree(recount);
    return fail(SFC_ENOMEM, "hipMalloc");
  }
  hipStream_t s = c->st;
  fill<int>(s, recount, (int64_t)c->hist_len, 0);
  fill<unsigned long long>(s, d_bad, 4, 0ull);
  Ctr* ctr = c->ctx[c->last_prepared].ctr;
  hipLaunchKernelGGL(k_verify_slots, dim3(grid_for(c->C, 256, kGridCap)), dim3(256), 0, s,
                     c->slot_id, c->stamp, c->index, c->hi, c->dmap, recount, c->hist_len, d_bad, ctr);
  if (c->dmap)
    hipLaunchKernelGGL(k_verify_dense, dim3(grid_for(c->V, 256, kGridCap)), dim3(256), 0, s,
                       c->dmap, c->V, c->slot_id, (int)c->C, d_bad);
  else
    hipLaunchKernelGGL(k_verify_entries, dim3(grid_for((int64_t)c->hi, 256, kGridCap)), dim3(256), 0, s,
                       c->index, c->hi, c->slot_id, (int)c->C, d_bad);
  hipLaunchKernelGGL(k_verify_hist, dim3(grid_for((int64_t)c->hist_len, 256, kGridCap)), dim3(256), 0, s,
                     c->hist, recount, c->hist_len, d_bad);
  unsigned long long hb[4] = {0, 0, 0, 0};
  hipError_t e = hipMemcpyAsync(hb, d_bad, sizeof hb, hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  (void)hipFree(recount);
  (void)hipFree(d_bad);
  if (e != hipSuccess) return fail(SFC_EHIP, "sfc_verify", e);
  Ctr h;
  HIPCHK(hipMemcpy(&h, ctr, sizeof h, hipMemcpyDeviceToHost));
  h_bad[0] = (int64_t)hb[0]; h_bad[1] = (int64_t)hb[1]; h_bad[2] = (int64_t)hb[2];
  h_bad[3] = (int64_t)hb[3] - (int64_t)h.f;          // live entries against occupied slots
  if (h_bad[0] || h_bad[1] || h_bad[2] || h_bad[3]) {
    char msg[160];
    snprintf(msg, sizeof msg, "sfc_verify: %lld slots not findable, %lld stray entries, %lld histogram "
             "words off, %lld live entries beyond the occupied slots",
             (long long)h_bad[0], (long long)h_bad[1], (long long)h_bad[2], (long long)h_bad[3]);
    return fail(SFC_ECORRUPT, msg);
  }
  return SFC_OK;
}

int sfc_cache_state(sfc_cache* c, int64_t* h_slot_id, int32_t* h_stamp, float* h_rows, float* h_acc) {
  if (!c) return fail(SFC_EINVAL, "null cache");
  int rc = sync_all(c);
  if (rc) return rc;
  if (c->C == 0) return SFC_OK;
  const size_t rows = (size_t)c->C * c->D * sizeof(float);
  if (h_slot_id) HIPCHK(hipMemcpy(h_slot_id, c->slot_id, (size_t)c->C * sizeof(int64_t), hipMemcpyDeviceToHost));
  if (h_stamp) HIPCHK(hipMemcpy(h_stamp, c->stamp, (size_t)c->C * sizeof(int32_t), hipMemcpyDeviceToHost));
  if (h_rows) HIPCHK(hipMemcpy(h_rows, c->cw, rows, hipMemcpyDeviceToHost));
  if (h_acc) HIPCHK(hipMemcpy(h_acc, c->ca, (size_t)c->C * c->S * sizeof(float), hipMemcpyDeviceToHost));
  return SFC_OK;
}

int sfc_profile_enable(sfc_cache* c, int32_t level) {
  if (!c) return fail(SFC_EINVAL, "null cache");
  c->prof = level < 0 ? 0 : (level > 2 ? 2 : level);
  return SFC_OK;
}

int sfc_profile_read(sfc_cache* c, int32_t which, double* h_ms_sum, int64_t* h_calls) {
  if (!c || which < 0 || which >= P_N || !h_ms_sum || !h_calls) return fail(SFC_EINVAL, "bad argument");
  int rc = sync_all(c);
  if (rc) return rc;
  if ((rc = prof_collect(c))) return rc;
  *h_ms_sum = c->ms_sum[which];
  *h_calls = c->calls[which];
  c->ms_sum[which] = 0;
  c->calls[which] = 0;
  return SFC_OK;
}

}  // extern "C"
