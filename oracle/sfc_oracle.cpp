// CPU oracle for the one-GPU sparse-embedding step of ScaleFreeCTR.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded, obviously
// correct statement of what one training step does to the embedding table.  It
// shares no code with the HIP library and must never be linked, imported or
// called by the product path; only tests, the smoke check and the benchmark's
// CPU-baseline leg use it.
//
// What it follows, by passage of the paper:
//   * Virtual Sparse Id (Data-Loader section, worked example): the batch's
//     distinct ids in order of first appearance (global_id) and, per position,
//     the index into that list (virtual_id).
//   * MixCache (Host-Manager section + worked example; Algorithm 1 lines 4-7):
//     which of the batch's rows are already in the cache buffer, which must be
//     pushed Host->cache ("working"), which resident rows are pulled back to
//     Host to make room ("noworking").  A row may only leave if it is not used
//     by the batch being prepared (nor, with lookahead, by the batch still in
//     flight).  The paper leaves the choice among evictable rows open; the
//     benchmark definition fixes least-recently-used.  The reading used here,
//     policy P1 "batch-granular LRU":
//       - every slot remembers the number t of the last step whose batch
//         contained its id (stamp);
//       - free slots F, need = #misses - |F|; if need > 0 the candidates are
//         occupied slots with stamp < t - lookahead, ordered by (stamp, slot),
//         and the first min(need, #candidates) are the victims;
//       - available = F u victims in ascending slot order; the i-th miss in
//         virtual-id order takes the i-th available slot (this reproduces the
//         paper's example: 7 replaces 1 in slot 0, 8 goes to the free slot);
//       - misses left over get a transient "bypass" row C+j that lives for
//         this step only and is written back to Host after the update.
//   * Forward (GPU-Worker / Forward, Algorithm 1 lines 9 and 11): the common
//     embedding is the cached row per virtual id, and the batch input is that
//     matrix indexed by virtual_id; a multi-hot bag is the sum of its rows.
//   * Backward (GPU-Worker / Backward): common gradient = unsorted segment sum
//     of the per-position gradients by virtual_id; then each cached row is
//     updated once per step from its summed gradient (Algorithm 1 line 14).
//     The optimizer is element-wise Adagrad as the benchmark definition fixes
//     it: acc += g*g ; w -= lr*g/(sqrt(acc)+eps), in fp32, with the summed
//     gradient accumulated in double and rounded to fp32 once.
//   * Other optimizers (Experiment settings: the paper trains with Adam, whose
//     two moment rows travel with each parameter row, so that the training
//     state is three times the embedding size).  S floats of optimizer state
//     follow every row through cache and Host:
//       - Adam (S = 2D, first moments then second moments), the textbook
//         update with the step number t of the batch in the bias correction:
//           m = b1*m + (1-b1)*g ; v = b2*v + (1-b2)*g*g
//           w -= lr * (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps)
//         The paper does not say what happens to rows outside the batch; the
//         reading here is the lazy one: they and their moments stay untouched.
//       - row-wise Adagrad (S = 1; not in the paper, the cheap variant of the
//         benchmark's Adagrad): one accumulator per row,
//           acc += mean_j(g_j^2) ; w_j -= lr*g_j/(sqrt(acc)+eps).
//   * The "Prefetch" strategy of the MixCache ablation (RQ3): no cache; the
//     rows of the next batch are copied from Host before the current batch is
//     trained, with no guarantee of consistency.  Made definite here as "stale
//     by exactly one step": the copy for batch t sees the Host table with the
//     write-backs of batches <= t-2; the rows trained by batch t-1 reach Host
//     only after that copy.  A row in two consecutive batches is therefore
//     trained from its old value and the earlier update is overwritten.  (The
//     "Host" strategy is capacity 0 without this: every copy sees every
//     earlier write-back.)
//   * Ids outside [0, V) (paper silent): all of them collapse to one null
//     entry with id -1; it owns no row, reads as zeros and drops its gradient.
//
// Parity pins for every function here live in tests/test_oracle_*.py.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <unordered_map>
#include <utility>
#include <vector>

namespace {

struct Stats {
  int64_t n_unique, n_hit, n_miss, n_evict, n_bypass, n_invalid, h2d_bytes, d2h_bytes;
};

struct Oracle {
  int64_t C = 0, V = 0;
  int D = 0;
  float lr = 0, eps = 0;
  double beta1 = 0, beta2 = 0;   // Adam's decay rates; every constant derived from them is rounded to fp32 once
  int lookahead = 0;
  int strategy = 0;           // 0 MixCache (capacity 0 = Host strategy), 1 Prefetch (stale by one step)
  std::vector<int64_t> pend_ids;       // Prefetch: rows trained by the last batch, not yet in Host
  std::vector<float> pend_w, pend_a;
  int opt = 0;                // 0 Adagrad, 1 Adam, 2 row-wise Adagrad
  int S = 0;                  // floats of optimizer state per row: D, 2D, 1
  float* host_w = nullptr;    // [V, D] caller-owned, updated in place
  float* host_acc = nullptr;  // [V, S]
  std::vector<float> cw, ca;  // [(C + bypass), D] cache rows and [(C + bypass), S] optimizer state
  std::vector<int64_t> slot_id;  // [C] resident id or -1
  std::vector<int32_t> stamp;    // [C] last step that used the slot, 0 = never
  std::unordered_map<int64_t, int32_t> where;  // id -> slot
  int64_t t = 0;
  // state of the step in progress
  std::vector<int64_t> uniq;
  std::vector<int32_t> inv, slot_of_vid, miss;
  std::vector<int64_t> ev_ids;
  std::vector<int32_t> ev_slots;
  std::vector<int64_t> offsets;  // empty = one-hot
  int64_t n_ids = 0, n_bags = 0, n_bypass = 0;
  Stats st{};
};

// Prefetch: the rows of the previous batch reach Host.
void apply_pending(Oracle* o) {
  const int D = o->D, S = o->S;
  for (size_t i = 0; i < o->pend_ids.size(); ++i) {
    int64_t id = o->pend_ids[i];
    std::memcpy(o->host_w + id * D, &o->pend_w[i * D], sizeof(float) * D);
    std::memcpy(o->host_acc + id * S, &o->pend_a[i * S], sizeof(float) * S);
  }
  o->pend_ids.clear(); o->pend_w.clear(); o->pend_a.clear();
}

void ensure_rows(Oracle* o, int64_t rows) {
  if (o->cw.size() < (size_t)rows * o->D) {
    o->cw.resize((size_t)rows * o->D, 0.f);
    o->ca.resize((size_t)rows * o->S, 0.f);
  }
}

}  // namespace

extern "C" {

void* orc_create(int64_t C, int32_t D, int64_t V, float* host_w, float* host_acc, float lr,
                 float eps, int32_t lookahead, int32_t optimizer, double beta1, double beta2,
                 int32_t strategy) {
  if (optimizer < 0 || optimizer > 2 || strategy < 0 || strategy > 1) return nullptr;
  if (strategy == 1 && C != 0) return nullptr;       // Prefetch keeps nothing resident
  Oracle* o = new Oracle;
  o->C = C; o->D = D; o->V = V; o->lr = lr; o->eps = eps; o->lookahead = lookahead;
  o->opt = optimizer; o->beta1 = beta1; o->beta2 = beta2; o->strategy = strategy;
  o->S = optimizer == 1 ? 2 * D : optimizer == 2 ? 1 : D;
  o->host_w = host_w; o->host_acc = host_acc;
  o->slot_id.assign((size_t)C, -1);
  o->stamp.assign((size_t)C, 0);
  ensure_rows(o, C);
  return o;
}

void orc_destroy(void* p) { delete (Oracle*)p; }

// Virtual Sparse Id + cache resolution + victim choice + slot assignment.
// Output arrays are sized by the caller for the worst case (n_ids entries).
// Returns 0, or -1 on a malformed bag structure.
int orc_prepare(void* p, const int64_t* ids, int64_t n_ids, const int64_t* offsets, int64_t n_bags,
                int64_t* unique_ids, int32_t* inverse, int32_t* slot, int32_t* miss_vids,
                int64_t* evict_ids, int32_t* evict_slots, Stats* stats) {
  Oracle* o = (Oracle*)p;
  if (offsets) {
    if (offsets[0] != 0 || offsets[n_bags] != n_ids) return -1;
    for (int64_t b = 0; b < n_bags; ++b) if (offsets[b + 1] < offsets[b]) return -1;
    o->offsets.assign(offsets, offsets + n_bags + 1);
  } else {
    if (n_bags != n_ids) return -1;
    o->offsets.clear();
  }
  o->t += 1;
  const int64_t t = o->t;
  o->n_ids = n_ids; o->n_bags = n_bags;
  o->st = Stats{};

  // 1. VSI: first-appearance unique and per-position virtual id.
  o->uniq.clear(); o->inv.assign((size_t)n_ids, 0);
  std::unordered_map<int64_t, int32_t> vid_of;
  for (int64_t q = 0; q < n_ids; ++q) {
    int64_t id = ids[q];
    if (id < 0 || id >= o->V) { id = -1; o->st.n_invalid++; }
    auto it = vid_of.find(id);
    if (it == vid_of.end()) {
      it = vid_of.emplace(id, (int32_t)o->uniq.size()).first;
      o->uniq.push_back(id);
    }
    o->inv[q] = it->second;
  }
  const int64_t U = (int64_t)o->uniq.size();
  o->st.n_unique = U;

  // 2. Resolve: hits refresh their stamp, misses are listed in vid order.
  o->slot_of_vid.assign((size_t)U, -1);
  o->miss.clear();
  for (int64_t v = 0; v < U; ++v) {
    int64_t id = o->uniq[v];
    if (id < 0) continue;                       // null entry owns no row
    auto it = o->where.find(id);
    if (it != o->where.end()) {
      o->slot_of_vid[v] = it->second;
      o->stamp[it->second] = (int32_t)t;
      o->st.n_hit++;
    } else {
      o->miss.push_back((int32_t)v);
    }
  }
  const int64_t M = (int64_t)o->miss.size();
  o->st.n_miss = M;

  // 3. Victims under policy P1.
  std::vector<int32_t> freeslots;
  for (int64_t s = 0; s < o->C; ++s) if (o->slot_id[s] < 0) freeslots.push_back((int32_t)s);
  int64_t need = M - (int64_t)freeslots.size();
  std::vector<int32_t> victims;
  if (need > 0) {
    std::vector<std::pair<int32_t, int32_t>> cand;  // (stamp, slot)
    for (int64_t s = 0; s < o->C; ++s)
      if (o->slot_id[s] >= 0 && (int64_t)o->stamp[s] < t - o->lookahead)
        cand.emplace_back(o->stamp[s], (int32_t)s);
    std::sort(cand.begin(), cand.end());
    int64_t k = std::min<int64_t>(need, (int64_t)cand.size());
    for (int64_t i = 0; i < k; ++i) victims.push_back(cand[i].second);
  }

  // 4. Assignment: ascending slots of (free u victims), then bypass rows.
  std::vector<int32_t> avail(freeslots);
  avail.insert(avail.end(), victims.begin(), victims.end());
  std::sort(avail.begin(), avail.end());
  std::sort(victims.begin(), victims.end());   // reported in ascending slot order
  o->ev_ids.clear(); o->ev_slots.clear();
  for (int32_t s : victims) { o->ev_slots.push_back(s); o->ev_ids.push_back(o->slot_id[s]); }
  o->st.n_evict = (int64_t)victims.size();
  int64_t nb = 0;
  for (int64_t i = 0; i < M; ++i) {
    int32_t v = o->miss[i];
    if (i < (int64_t)avail.size()) o->slot_of_vid[v] = avail[i];
    else o->slot_of_vid[v] = (int32_t)(o->C + nb++);
  }
  o->n_bypass = nb;
  o->st.n_bypass = nb;
  ensure_rows(o, o->C + nb);
  const int64_t rowbytes = (int64_t)sizeof(float) * (o->D + o->S);   // weights + optimizer state
  o->st.h2d_bytes = M * rowbytes;
  o->st.d2h_bytes = (o->st.n_evict + nb) * rowbytes;

  std::copy(o->uniq.begin(), o->uniq.end(), unique_ids);
  std::copy(o->inv.begin(), o->inv.end(), inverse);
  std::copy(o->slot_of_vid.begin(), o->slot_of_vid.end(), slot);
  std::copy(o->miss.begin(), o->miss.end(), miss_vids);
  std::copy(o->ev_ids.begin(), o->ev_ids.end(), evict_ids);
  std::copy(o->ev_slots.begin(), o->ev_slots.end(), evict_slots);
  if (stats) *stats = o->st;
  return 0;
}

// 5. Pull victims to Host, then push missed rows into their slots.
void orc_fetch_misses(void* p) {
  Oracle* o = (Oracle*)p;
  const int D = o->D, S = o->S;
  for (size_t i = 0; i < o->ev_slots.size(); ++i) {
    int64_t id = o->ev_ids[i]; int32_t s = o->ev_slots[i];
    std::memcpy(o->host_w + id * D, &o->cw[(size_t)s * D], sizeof(float) * D);
    std::memcpy(o->host_acc + id * S, &o->ca[(size_t)s * S], sizeof(float) * S);
    o->where.erase(id);
    o->slot_id[s] = -1;
  }
  for (int32_t v : o->miss) {
    int64_t id = o->uniq[v]; int32_t s = o->slot_of_vid[v];
    std::memcpy(&o->cw[(size_t)s * D], o->host_w + id * D, sizeof(float) * D);
    std::memcpy(&o->ca[(size_t)s * S], o->host_acc + id * S, sizeof(float) * S);
    if (s < o->C) {
      o->where[id] = s;
      o->slot_id[s] = id;
      o->stamp[s] = (int32_t)o->t;
    }
  }
  if (o->strategy == 1) apply_pending(o);    // only now do the previous batch's rows reach Host
}

// 6. out[b,:] = sum over the bag's positions of the cached row of that position's id.
void orc_lookup(void* p, float* out) {
  Oracle* o = (Oracle*)p;
  const int D = o->D;
  std::vector<double> acc((size_t)D);
  for (int64_t b = 0; b < o->n_bags; ++b) {
    int64_t lo = o->offsets.empty() ? b : o->offsets[b];
    int64_t hi = o->offsets.empty() ? b + 1 : o->offsets[b + 1];
    std::fill(acc.begin(), acc.end(), 0.0);
    for (int64_t q = lo; q < hi; ++q) {
      int32_t s = o->slot_of_vid[o->inv[q]];
      if (s < 0) continue;
      const float* row = &o->cw[(size_t)s * D];
      for (int j = 0; j < D; ++j) acc[j] += (double)row[j];
    }
    for (int j = 0; j < D; ++j) out[b * D + j] = (float)acc[j];
  }
}

// 7.-9. segment-sum of grad by virtual id, one optimizer update on each unique row, bypass rows
// to Host.  common_grad (optional, [U, D]) receives the summed gradients.
void orc_backward_update(void* p, const float* grad, float* common_grad) {
  Oracle* o = (Oracle*)p;
  const int D = o->D, S = o->S;
  // Adam's bias corrections for this step's number
  const float b1 = (float)o->beta1, b2 = (float)o->beta2;
  const float c1 = (float)(1.0 - o->beta1), c2 = (float)(1.0 - o->beta2);
  const float bc1 = (float)(1.0 - std::pow(o->beta1, (double)o->t));
  const float bc2 = (float)(1.0 - std::pow(o->beta2, (double)o->t));
  const int64_t U = (int64_t)o->uniq.size();
  std::vector<double> G((size_t)U * D, 0.0);
  for (int64_t b = 0; b < o->n_bags; ++b) {
    int64_t lo = o->offsets.empty() ? b : o->offsets[b];
    int64_t hi = o->offsets.empty() ? b + 1 : o->offsets[b + 1];
    for (int64_t q = lo; q < hi; ++q) {
      double* g = &G[(size_t)o->inv[q] * D];
      for (int j = 0; j < D; ++j) g[j] += (double)grad[b * D + j];
    }
  }
  for (int64_t v = 0; v < U; ++v) {
    if (common_grad)
      for (int j = 0; j < D; ++j) common_grad[v * D + j] = (float)G[(size_t)v * D + j];
    int32_t s = o->slot_of_vid[v];
    if (s < 0) continue;
    float* w = &o->cw[(size_t)s * D];
    float* a = &o->ca[(size_t)s * S];
    if (o->opt == 0) {
      for (int j = 0; j < D; ++j) {
        float g = (float)G[(size_t)v * D + j];
        float acc = a[j] + g * g;
        a[j] = acc;
        w[j] = w[j] - o->lr * g / (std::sqrt(acc) + o->eps);
      }
    } else if (o->opt == 1) {
      float* m = a;
      float* sq = a + D;
      for (int j = 0; j < D; ++j) {
        float g = (float)G[(size_t)v * D + j];
        m[j] = b1 * m[j] + c1 * g;
        sq[j] = b2 * sq[j] + c2 * (g * g);
        float mhat = m[j] / bc1;
        float vhat = sq[j] / bc2;
        w[j] = w[j] - o->lr * mhat / (std::sqrt(vhat) + o->eps);
      }
    } else {
      double ss = 0.0;
      for (int j = 0; j < D; ++j) {
        float g = (float)G[(size_t)v * D + j];
        ss += (double)g * (double)g;
      }
      float acc = a[0] + (float)(ss / D);
      a[0] = acc;
      for (int j = 0; j < D; ++j) {
        float g = (float)G[(size_t)v * D + j];
        w[j] = w[j] - o->lr * g / (std::sqrt(acc) + o->eps);
      }
    }
  }
  for (int32_t v : o->miss) {
    int32_t s = o->slot_of_vid[v];
    if (s < o->C) continue;
    int64_t id = o->uniq[v];
    if (o->strategy == 1) {
      o->pend_ids.push_back(id);
      o->pend_w.insert(o->pend_w.end(), &o->cw[(size_t)s * D], &o->cw[(size_t)s * D] + D);
      o->pend_a.insert(o->pend_a.end(), &o->ca[(size_t)s * S], &o->ca[(size_t)s * S] + S);
      continue;
    }
    std::memcpy(o->host_w + id * D, &o->cw[(size_t)s * D], sizeof(float) * D);
    std::memcpy(o->host_acc + id * S, &o->ca[(size_t)s * S], sizeof(float) * S);
  }
}

// 10. Every resident row and accumulator to Host (the cache stays resident).
void orc_flush(void* p) {
  Oracle* o = (Oracle*)p;
  const int D = o->D, S = o->S;
  apply_pending(o);
  for (int64_t s = 0; s < o->C; ++s) {
    int64_t id = o->slot_id[s];
    if (id < 0) continue;
    std::memcpy(o->host_w + id * D, &o->cw[(size_t)s * D], sizeof(float) * D);
    std::memcpy(o->host_acc + id * S, &o->ca[(size_t)s * S], sizeof(float) * S);
  }
}

// Cache state for comparison: resident id and stamp per slot, rows and accumulators.
void orc_get_state(void* p, int64_t* slot_id, int32_t* stamp, float* rows, float* acc) {
  Oracle* o = (Oracle*)p;
  if (slot_id) std::copy(o->slot_id.begin(), o->slot_id.end(), slot_id);
  if (stamp) std::copy(o->stamp.begin(), o->stamp.end(), stamp);
  if (rows) std::copy(o->cw.begin(), o->cw.begin() + (size_t)o->C * o->D, rows);
  if (acc) std::copy(o->ca.begin(), o->ca.begin() + (size_t)o->C * o->S, acc);
}

}  // extern "C"
