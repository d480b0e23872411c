/*
 * sfc.h - C ABI of the one-GPU sparse-embedding hot path of ScaleFreeCTR
 * (Virtual Sparse Id + MixCache + gather + gradient segment-sum + sparse
 * optimizer update), implemented with HIP kernels for gfx950 (MI355X).
 *
 * One training step is four calls, in this order (with lookahead = L > 0 the first two of step t+L may
 * precede the last of step t; sfc_lookup, sfc_segment_sum and sfc_backward_update always act on
 * the oldest step that has been fetched and not yet updated) (Algorithm 1, lines 3-14,
 * with the multi-GPU lines 7, 10 and 13 and the dense model of line 12 left to
 * the caller):
 *
 *     sfc_prepare          lines 3-4   ids -> global_id / virtual_id, hit / miss / victims, slots
 *     sfc_fetch_misses     lines 5-6   victims cache->Host, missed rows Host->cache (side stream)
 *     sfc_lookup           lines 9,11  [bags, dim] model input from the cached rows
 *     sfc_backward_update  line 14     segment-sum of the gradients per virtual id + optimizer update
 *
 * Conventions
 *   - Every function returns 0 (SFC_OK) or a negative SFC_E* code; nothing throws or aborts.
 *     sfc_last_error() gives a text for the most recent failure on the calling thread.
 *   - Pointers named d_* are DEVICE memory owned by the caller; pointers named h_* are HOST
 *     memory owned by the caller.  The library owns the cache rows, their optimizer state, the
 *     cache index and all scratch.  Buffers handed to sfc_prepare are used by the later calls
 *     of the same step and must stay alive and unmodified until sfc_backward_update (or the
 *     next sfc_prepare) has completed on the stream.
 *   - All work is enqueued on the streams given at creation and is asynchronous to the host,
 *     except sfc_cache_create, sfc_flush, sfc_get_stats, sfc_cache_state, sfc_verify and
 *     sfc_cache_destroy, which synchronise.  No call allocates device memory after
 *     sfc_cache_create (sfc_verify, a test aid, excepted).
 *   - Errors that only the device can see (a consistency check of the cache manager that fired,
 *     malformed bag offsets) are written by the kernels into a pinned status block.  Every step
 *     call looks at it first, without waiting, and refuses to go on (SFC_ECORRUPT) once the manager
 *     state is inconsistent; sfc_check reads the same block on demand.
 *   - One sfc_cache must be driven by one host thread at a time.
 *   - Rows are fp32, row-major, dim floats each; dim must be a multiple of 4 and all row
 *     buffers 16-byte aligned.
 */
#ifndef SFC_H
#define SFC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SFC_OK 0
#define SFC_EINVAL (-1)  /* bad argument: null pointer, size out of range, dim not a multiple of 4 */
#define SFC_ESTATE (-2)  /* call out of order */
#define SFC_EHIP (-3)    /* a HIP runtime call failed; see sfc_last_error() */
#define SFC_ENOMEM (-4)  /* device or host allocation failed */
#define SFC_ELIMIT (-5)  /* more steps than max_steps */
#define SFC_ECORRUPT (-6) /* a device-side consistency check of the cache manager has fired */

#define SFC_POLICY_LRU_BATCH 0
/* The "Prefetch" strategy of the paper's MixCache ablation (RQ3), for comparison runs: nothing is
 * kept resident (capacity_rows must be 0, lookahead must be 1) and the rows of step t+1 are copied
 * from Host while step t is looked up, without waiting for step t's update: a row of both batches
 * is trained from its stale value and step t's update of it is overwritten.  Made deterministic:
 * sfc_backward_update of step t waits for the copies of step t+1 when they were issued before it,
 * so step t+1 misses exactly the update of step t.  (The ablation's "Host" strategy is
 * SFC_POLICY_LRU_BATCH with capacity_rows = 0.) */
#define SFC_POLICY_PREFETCH 1

/* Optimizers and the floats of state S that travel with every row (cache <-> Host):
 *   ADAGRAD          S = D    element-wise accumulator
 *   ADAM             S = 2D   first moments [D], then second moments [D] (Experiment settings: the
 *                             paper's optimizer; its state makes the training parameters three
 *                             times the embedding size)
 *   ROWWISE_ADAGRAD  S = 4    one accumulator per row in the first float; the other three floats
 *                             pad the state to one 16-byte chunk and are carried unchanged */
#define SFC_OPT_ADAGRAD 0
#define SFC_OPT_ADAM 1
#define SFC_OPT_ROWWISE_ADAGRAD 2

/* The manager's id -> slot index in HBM.  DENSE: one int per Host row (4 * host_rows bytes): no
 * probing, no deleted entries, no rebuild.  HASHED: open addressing with 16-byte entries, four per
 * possible resident id, rebuilt on the device when deleted entries pass an eighth of it: for id
 * ranges whose dense map would not fit.  AUTO takes DENSE up to SFC_DENSE_INDEX_MAX_BYTES. */
#define SFC_INDEX_AUTO 0
#define SFC_INDEX_HASHED 1
#define SFC_INDEX_DENSE 2
#define SFC_DENSE_INDEX_MAX_BYTES ((int64_t)32 << 30)

typedef struct sfc_cache sfc_cache; /* opaque */

typedef struct {
  int64_t capacity_rows;      /* C >= 0: row slots of the cache buffer (0 = every row bypasses) */
  int32_t dim;                /* D: floats per row, multiple of 4, <= 256 */
  int32_t policy;             /* SFC_POLICY_LRU_BATCH or SFC_POLICY_PREFETCH */
  int64_t max_ids_per_batch;  /* upper bound on n_ids of any step; sizes scratch and bypass rows */
  int64_t max_bags_per_batch; /* upper bound on n_bags of any step */
  int64_t host_rows;          /* V: rows of the Host table; valid ids are [0, V) */
  float* h_weights;           /* [V, D] Host table, pinned and device-mapped (see sfc_host_alloc) */
  float* h_acc;               /* [V, S] optimizer state of every row, same kind of memory */
  int64_t host_row_stride;    /* floats between consecutive rows of h_weights; 0 = D.
                                 With h_acc = h_weights + D and both strides D + S each row's
                                 weights and state are one contiguous block, the layout the host
                                 link moves fastest. */
  float lr;                   /* learning rate */
  float eps;                  /* epsilon, added outside the square root */
  int32_t lookahead;          /* L = 0 .. 3: how many steps may be prepared ahead of the one being
                                 trained.  Rows used by the batch being prepared and by the L
                                 batches before it are protected from eviction.
                                 0: calls of a step go prepare, fetch_misses, lookup,
                                 backward_update, all in order.
                                 L > 0 (needs side_stream != stream): sfc_prepare /
                                 sfc_fetch_misses of step t+L may be called before
                                 sfc_backward_update of step t; they run on other streams while the
                                 main stream works on step t (the paper's pipeline of Data-Loader,
                                 Host-Manager and GPU-Worker stages): the prepare on two streams
                                 the library creates, the Host copies on side_stream.  Each
                                 further step of lookahead adds a step context, so that a prepare
                                 waits for an older update.  The caller rotates L + 1 sets of
                                 prepare buffers. */
  int32_t max_steps;          /* steps this cache may run (sizes the recency histogram); 0 = 1<<20 */
  void* stream;               /* hipStream_t for prepare / lookup / backward_update */
  void* side_stream;          /* hipStream_t for the Host<->cache copies; may equal stream */
  int32_t optimizer;          /* SFC_OPT_* */
  int32_t index_kind;         /* SFC_INDEX_AUTO (0), SFC_INDEX_HASHED or SFC_INDEX_DENSE */
  int64_t host_state_stride;  /* floats between consecutive rows of h_acc; 0 = S */
  double beta1, beta2;        /* Adam's decay rates (ignored otherwise) */
} sfc_config;

typedef struct {
  int64_t n_unique;   /* U: distinct ids of the batch (a null entry for out-of-range ids included) */
  int64_t n_hit;      /* unique ids already resident */
  int64_t n_miss;     /* unique ids fetched from Host (bypass rows included) */
  int64_t n_evict;    /* resident rows written back to Host to make room */
  int64_t n_bypass;   /* misses that found no slot and live in a transient row for this step */
  int64_t n_invalid;  /* positions whose id was outside [0, V) */
  int64_t h2d_bytes;  /* Host->cache bytes of this step (rows + optimizer state) */
  int64_t d2h_bytes;  /* cache->Host bytes of this step (victims + bypass rows) */
  int64_t n_bad_offsets; /* violations found in d_offsets (0 for well-formed input) */
} sfc_stats;

/* Pinned, device-mapped Host memory suitable for h_weights / h_acc.  Returns NULL on failure.
 * One table should be ONE allocation (weights and state interleaved, see host_row_stride): the
 * runtime has been seen to refuse a single piece beyond about 50 GB and to crash at the next
 * kernel launch after two pieces of 35 GB each, so this call refuses (NULL) a request that would
 * take the total handed out by it in this process beyond SFC_HOST_ALLOC_MAX_BYTES while another
 * piece of at least SFC_HOST_ALLOC_LARGE_BYTES is alive. */
#define SFC_HOST_ALLOC_MAX_BYTES ((int64_t)56 << 30)
#define SFC_HOST_ALLOC_LARGE_BYTES ((int64_t)8 << 30)
void* sfc_host_alloc(int64_t bytes);
void sfc_host_free(void* p);

/*
 * Create an empty cache: the per-GPU cache buffer of MixCache (Host-Manager section), a fixed
 * number of row slots in HBM holding the working rows and their optimizer state.  The manager
 * state (id -> slot index, per-slot recency stamp) lives in HBM too.  Allocates all device
 * memory the later calls use.
 */
int sfc_cache_create(const sfc_config* cfg, sfc_cache** out);
void sfc_cache_destroy(sfc_cache* c);

/*
 * Step 1 (Algorithm 1 lines 3-4; Data-Loader section, Host-Manager section).
 *  d_ids       [n_ids] int64 raw feature ids, row-major [batch, fields] or the concatenated bags.
 *              Produced on `stream` before this call (or already complete): with lookahead > 0 the
 *              prepare runs on other streams (streams the library creates; side_stream for
 *              SFC_POLICY_PREFETCH), which first wait for what `stream` has been given so far.
 *  d_offsets   NULL for one-hot input (then n_bags must equal n_ids), else [n_bags+1] int64 CSR
 *              offsets with d_offsets[0] = 0 and d_offsets[n_bags] = n_ids, non-decreasing.
 *  outputs (each sized for n_ids entries by the caller):
 *  d_unique_ids  global_id: the distinct ids in order of first appearance; ids outside [0, V)
 *                all collapse into one null entry with value -1.
 *  d_inverse     virtual_id per position: d_unique_ids[d_inverse[p]] == d_ids[p] (or -1).
 *  d_slot        per virtual id: cache slot in [0, C), or C + j for the j-th bypass row of this
 *                step, or -1 for the null entry.  Slots of misses hold valid data only after
 *                sfc_fetch_misses.
 *  d_miss_vids   virtual ids that must be fetched from Host, ascending; n_miss entries.
 * Hit / miss / victim counts stay on the device (sfc_get_stats reads them).
 * Victims are chosen by batch-granular LRU: among resident rows not used by this batch (nor by
 * the `lookahead` batches before it), those whose last use is oldest, ties by lower slot; the
 * i-th miss takes the i-th slot of (free + victim slots) in ascending slot order.
 * Errors: SFC_EINVAL (null pointers, n_ids > max_ids_per_batch, n_bags > max_bags_per_batch,
 * one-hot with n_bags != n_ids, multi-hot with ids but no bags), SFC_ESTATE (the previous step has
 * not been fetched yet, or all lookahead + 1 step contexts hold steps that have not been updated:
 * finish one with sfc_backward_update or give it up with sfc_discard), SFC_ELIMIT, SFC_EHIP,
 * SFC_ECORRUPT.
 * Malformed offsets live in device memory, so the host cannot refuse them here: the prepare
 * kernels check them (first 0, last n_ids, none decreasing), count the violations in
 * sfc_stats.n_bad_offsets and report the step through sfc_check.  Such a step reads and writes
 * inside its buffers only, and the cache manager state stays consistent (it depends on the ids
 * alone), but its lookup output and its update are meaningless.
 */
int sfc_prepare(sfc_cache* c, const int64_t* d_ids, int64_t n_ids, const int64_t* d_offsets,
                int64_t n_bags, int64_t* d_unique_ids, int32_t* d_inverse, int32_t* d_slot,
                int32_t* d_miss_vids);

/*
 * Step 2 (Algorithm 1 lines 5-6): on the side stream, after the prepare of this step, write every
 * victim row and its optimizer state back to the Host table and copy every missed row and its
 * state from the Host table into its slot (a victim's row is read before its slot is
 * overwritten).  The main stream is made to wait for it before it touches the step's rows.
 * With lookahead > 0 the copies run behind the updates of older steps still in flight whenever
 * one of those had bypass rows (their rows reach the Host table only with the update).
 */
int sfc_fetch_misses(sfc_cache* c);

/*
 * Step 3 (Algorithm 1 lines 9 and 11; GPU-Worker / Forward): d_out[b, :] = sum over the
 * positions q of bag b of the cached row of d_ids[q]  (one row for one-hot input).  Rows of the
 * null entry count as zeros.  d_out is [n_bags, D] fp32.  May be called more than once.
 */
int sfc_lookup(sfc_cache* c, float* d_out);

/*
 * GPU-Worker / Backward, first half: d_common_grad[v, :] = sum over positions q with
 * d_inverse[q] == v of d_grad[bag(q), :] (the unsorted segment sum that turns Local Gradients
 * into Local Common Gradients), accumulated in fp64 and rounded to fp32 once.
 * d_grad is [n_bags, D]; d_common_grad is [n_unique, D], caller-sized for n_ids rows.
 * Optional: a multi-GPU caller exchanges this matrix; sfc_backward_update does not need it.
 */
int sfc_segment_sum(sfc_cache* c, const float* d_grad, float* d_common_grad);

/*
 * sfc_segment_sum for callers that must not allocate or depend on allocations made for them: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs,
 * outputs and result (bit for bit), but the kernels' scratch (the partial sums of runs that cross
 * a thread block's edge) lives in a fixed array inside the library's code object instead of the
 * buffer sfc_cache_create allocated: SFC_STATIC_SCRATCH_BYTES per GPU, held until the process
 * ends.  Returns SFC_ELIMIT when the step needs more (2 * blocks * (8 * dim + 4) bytes, blocks =
 * wavefronts of the stream / 4; the target configuration takes 1.6 MB).  Calls no allocating
 * routine and creates no events.  Every call on one GPU shares the array: calls that overlap on
 * one GPU (two caches on two streams) race; nothing needs clearing between calls.
 */
#define SFC_STATIC_SCRATCH_BYTES (8 << 20)
int sfc_segment_sum_static(sfc_cache* c, const float* d_grad, float* d_common_grad);

/*
 * Step 4 (GPU-Worker / Backward; Algorithm 1 line 14): segment-sum d_grad [n_bags, D] per
 * virtual id as above and apply one optimizer update per unique row in the cache (fp32):
 *   ADAGRAD          acc += g*g ;  w -= lr * g / (sqrt(acc) + eps)             (element-wise)
 *   ADAM             m = b1*m + (1-b1)*g ;  v = b2*v + (1-b2)*g*g ;
 *                    w -= lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps)
 *                    with t = the number of this step's batch (the first sfc_prepare is 1); rows
 *                    outside the batch and their moments are left as they are
 *   ROWWISE_ADAGRAD  acc += mean_j(g_j^2) ;  w_j -= lr * g_j / (sqrt(acc) + eps)
 * Bypass rows are written back to the Host table by the same pass.  Ends the step.
 */
int sfc_backward_update(sfc_cache* c, const float* d_grad);

/*
 * Gives up the oldest step that has been fetched and not updated (a batch that was only looked
 * up, e.g. for inference): its step context becomes free, its rows stay in the cache unchanged.
 * SFC_ESTATE if there is no such step or its rows are still on their way.
 */
int sfc_discard(sfc_cache* c);

/* Write every resident row and accumulator to the Host table and wait; the cache stays warm. */
int sfc_flush(sfc_cache* c);

/* Counters of the most recent sfc_prepare; waits for the streams. */
int sfc_get_stats(sfc_cache* c, sfc_stats* h_out);

/*
 * What the device has reported so far, without waiting for any stream (one read of pinned
 * memory).  sfc_check returns SFC_ECORRUPT once a consistency check of the cache manager has
 * fired on the device (the cache must not be used any further; sfc_last_error names the check and
 * its step), SFC_EINVAL if a step since the last sfc_check had malformed bag offsets (reported
 * once; sfc_last_error names the step), else SFC_OK.
 * sfc_peek_stats returns the counters of the most recent step whose cache-manager plan has run on
 * the device and that step's number in *h_step (0: none yet); the byte counts are derived from
 * them.  A training loop can poll both every step at no cost.
 */
int sfc_check(sfc_cache* c);
int sfc_peek_stats(sfc_cache* c, sfc_stats* h_out, int64_t* h_step);

/*
 * Test aid: waits for the streams, then recounts the manager state on the device.  h_bad[0]:
 * occupied slots whose id the index does not map to that slot; h_bad[1]: live index entries that
 * do not point at a slot holding their id (stale or duplicate entries); h_bad[2]: words of the
 * recency histogram that differ from a recount of the slots' stamps; h_bad[3]: live entries minus
 * occupied slots.  Returns SFC_ECORRUPT if any is nonzero.  Needs every step context free or
 * fetched (no prepare without its fetch).  Allocates and frees a scratch histogram.
 */
int sfc_verify(sfc_cache* c, int64_t* h_bad /* [4] */);

/*
 * Snapshot of the cache for inspection; waits for the streams.  Any pointer may be NULL.
 *  h_slot_id [C] int64  resident id per slot, -1 = free
 *  h_stamp   [C] int32  step number of the last batch that used the slot, 0 = never
 *  h_rows    [C, D]     cached weights        h_acc [C, S] cached optimizer state
 */
int sfc_cache_state(sfc_cache* c, int64_t* h_slot_id, int32_t* h_stamp, float* h_rows, float* h_acc);

/*
 * Device timing.  level 1: the step calls.  sfc_prepare, sfc_fetch_misses and sfc_backward_update
 * (several kernels each) are bracketed by hipEvents on the stream they run on, so their times
 * include the launch latencies between the events (with lookahead >= 1 the prepare runs on two
 * library streams; its events sit on the one of the cache manager's kernels and include its wait
 * for the unique passes on the other).  sfc_lookup is two kernels (the batch's rows are read into
 * the memory-side cache, then gathered): the start and end of each are recorded by the dispatch
 * itself, i.e. the time is the sum of the two kernels' own durations as a profiler's kernel trace
 * shows them.  level 2: also, the same way, each of the kernels inside sfc_backward_update.
 * level 0: off.  sfc_profile_read waits for the streams and returns, for which = 0..6 (prepare,
 * fetch_misses, lookup, backward_update, segment-sum stream kernel, segment-sum finish kernel,
 * optimizer kernel), the summed milliseconds and the number of launches since the last read of
 * that entry.  With Adagrad or Adam sfc_backward_update launches no finish kernel (the
 * optimizer kernel chains the stream's block-edge partials itself): entry 5 then counts the
 * launches of sfc_segment_sum only.
 */
int sfc_profile_enable(sfc_cache* c, int32_t level);
int sfc_profile_read(sfc_cache* c, int32_t which, double* h_ms_sum, int64_t* h_calls);

const char* sfc_strerror(int code);
const char* sfc_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SFC_H */
