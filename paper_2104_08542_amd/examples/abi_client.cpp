// A client of include/sfc.h that uses nothing but the HIP runtime: device buffers from hipMalloc,
// two plain streams, the Host table from sfc_host_alloc.  It runs a few training steps over a
// small table with a cache that evicts, flushes, and checks the table against a dense table
// trained on the host with the same rule (one Adagrad update per unique id per step from the
// summed gradient).  Exit status 0 = every check passed.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <vector>

#include "../../include/sfc.h"

#define HIP_OK(x)                                                                  \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } \
  } while (0)
#define SFC_OK_OR_DIE(x)                                                           \
  do {                                                                             \
    int r_ = (x);                                                                  \
    if (r_ != SFC_OK) { printf("sfc error %d (%s): %s at line %d\n", r_, sfc_strerror(r_), sfc_last_error(), __LINE__); return 3; } \
  } while (0)

int main() {
  const int64_t V = 5000, C = 700, N = 2048;
  const int D = 16;
  const float lr = 0.05f, eps = 1e-8f;
  // Host table, rows interleaved [weights | accumulator]
  float* tab = (float*)sfc_host_alloc(V * 2 * D * sizeof(float));
  if (!tab) { printf("sfc_host_alloc failed\n"); return 2; }
  std::vector<float> rw(V * D), ra(V * D, 0.1f);          // reference table on the host
  uint64_t s = 12345;
  auto rnd = [&]() { s = s * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(s >> 33); };
  for (int64_t i = 0; i < V; ++i)
    for (int j = 0; j < D; ++j) {
      const float w = ((int)(rnd() % 2001) - 1000) * 1e-5f;
      tab[i * 2 * D + j] = w; tab[i * 2 * D + D + j] = 0.1f; rw[i * D + j] = w;
    }

  hipStream_t st, side;
  HIP_OK(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
  HIP_OK(hipStreamCreateWithFlags(&side, hipStreamNonBlocking));
  sfc_config cfg = {};
  cfg.capacity_rows = C; cfg.dim = D; cfg.policy = SFC_POLICY_LRU_BATCH;
  cfg.max_ids_per_batch = N; cfg.max_bags_per_batch = N; cfg.host_rows = V;
  cfg.h_weights = tab; cfg.h_acc = tab + D; cfg.host_row_stride = 2 * D; cfg.host_state_stride = 2 * D;
  cfg.lr = lr; cfg.eps = eps; cfg.lookahead = 0; cfg.stream = st; cfg.side_stream = side;
  cfg.optimizer = SFC_OPT_ADAGRAD;
  sfc_cache* cache = nullptr;
  SFC_OK_OR_DIE(sfc_cache_create(&cfg, &cache));

  int64_t *d_ids, *d_uniq;
  int32_t *d_inv, *d_slot, *d_miss;
  float *d_out, *d_grad;
  HIP_OK(hipMalloc(&d_ids, N * 8)); HIP_OK(hipMalloc(&d_uniq, N * 8));
  HIP_OK(hipMalloc(&d_inv, N * 4)); HIP_OK(hipMalloc(&d_slot, N * 4)); HIP_OK(hipMalloc(&d_miss, N * 4));
  HIP_OK(hipMalloc(&d_out, N * D * 4)); HIP_OK(hipMalloc(&d_grad, N * D * 4));
  std::vector<int64_t> ids(N), uniq(N);
  std::vector<int32_t> inv(N);
  std::vector<float> out(N * D), grad(N * D);
  int bad = 0;
  int64_t evicted = 0;
  for (int step = 0; step < 6; ++step) {
    for (int64_t p = 0; p < N; ++p) {                      // skewed ids: squares concentrate on small values
      const double u = (rnd() % 100000) / 100000.0;
      ids[p] = (int64_t)(u * u * u * (V - 1));
    }
    for (auto& g : grad) g = ((int)(rnd() % 2001) - 1000) * 1e-3f;
    HIP_OK(hipMemcpyAsync(d_ids, ids.data(), N * 8, hipMemcpyHostToDevice, st));
    HIP_OK(hipMemcpyAsync(d_grad, grad.data(), N * D * 4, hipMemcpyHostToDevice, st));
    SFC_OK_OR_DIE(sfc_prepare(cache, d_ids, N, nullptr, N, d_uniq, d_inv, d_slot, d_miss));
    SFC_OK_OR_DIE(sfc_fetch_misses(cache));
    SFC_OK_OR_DIE(sfc_lookup(cache, d_out));
    SFC_OK_OR_DIE(sfc_backward_update(cache, d_grad));
    sfc_stats stt;
    SFC_OK_OR_DIE(sfc_get_stats(cache, &stt));             // waits for the streams
    evicted += stt.n_evict;
    HIP_OK(hipMemcpy(uniq.data(), d_uniq, N * 8, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(inv.data(), d_inv, N * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(out.data(), d_out, N * D * 4, hipMemcpyDeviceToHost));
    // virtual ids: dense, first-appearance order, inverse consistent; lookup = table rows
    std::map<int64_t, int> seen;
    for (int64_t p = 0; p < N; ++p) {
      auto it = seen.find(ids[p]);
      if (it == seen.end()) it = seen.emplace(ids[p], (int)seen.size()).first;
      if (inv[p] != it->second || uniq[inv[p]] != ids[p]) ++bad;
      for (int j = 0; j < D; ++j) {
        const double r = rw[ids[p] * D + j];
        if (std::fabs((double)out[p * D + j] - r) > 1e-6 + 1e-5 * std::fabs(r)) ++bad;
      }
    }
    if ((int64_t)seen.size() != stt.n_unique) ++bad;
    // reference update: gradient summed per id in double, one Adagrad step per id
    std::map<int64_t, std::vector<double>> G;
    for (int64_t p = 0; p < N; ++p) {
      auto& g = G[ids[p]];
      if (g.empty()) g.assign(D, 0.0);
      for (int j = 0; j < D; ++j) g[j] += (double)grad[p * D + j];
    }
    for (auto& kv : G)
      for (int j = 0; j < D; ++j) {
        const float g = (float)kv.second[j];
        float& a = ra[kv.first * D + j];
        float& w = rw[kv.first * D + j];
        a = a + g * g;
        w = w - lr * g / (std::sqrt(a) + eps);
      }
    printf("step %d: unique %lld hit %lld miss %lld evict %lld bypass %lld\n", step, (long long)stt.n_unique,
           (long long)stt.n_hit, (long long)stt.n_miss, (long long)stt.n_evict, (long long)stt.n_bypass);
  }
  SFC_OK_OR_DIE(sfc_flush(cache));
  double worst = 0;
  for (int64_t i = 0; i < V; ++i)
    for (int j = 0; j < D; ++j) {
      const double dw = std::fabs((double)tab[i * 2 * D + j] - rw[i * D + j]);
      const double da = std::fabs((double)tab[i * 2 * D + D + j] - ra[i * D + j]);
      if (dw > 1e-6 + 1e-5 * std::fabs(rw[i * D + j]) || da > 1e-6 + 1e-5 * std::fabs(ra[i * D + j])) ++bad;
      if (dw > worst) worst = dw;
    }
  if (evicted == 0) { printf("the cache never evicted: the run did not exercise the write-back\n"); ++bad; }
  sfc_cache_destroy(cache);
  sfc_host_free(tab);
  printf("%s: %d mismatches, worst weight difference %.3g, %lld rows evicted\n", bad ? "FAILED" : "OK", bad, worst,
         (long long)evicted);
  return bad ? 1 : 0;
}
