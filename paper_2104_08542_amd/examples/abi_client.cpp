// A client of include/sfc.h that uses nothing but the HIP runtime: device buffers from hipMalloc,
// two plain streams, the Host table from sfc_host_alloc.  It runs a few training steps over a
// small table with a cache that evicts (optionally pipelined: abi_client <lookahead>), flushes,
// and checks every lookup output and the final table against a dense table trained on the host
// with the same rule (one Adagrad update per unique id per step from the summed gradient).
// Exit status 0 = every check passed.
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

int main(int argc, char** argv) {
  const int L = argc > 1 ? atoi(argv[1]) : 0;            // lookahead 0 .. 3
  if (L < 0 || L > 3) { printf("usage: abi_client [lookahead 0|1|2|3]\n"); return 2; }
  const int64_t V = 5000, C = 700, N = 2048;
  const int D = 16, T = 8;
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
  // all batches up front: skewed ids (cubes concentrate on small values), gradients in [-1, 1]
  std::vector<std::vector<int64_t>> ids(T, std::vector<int64_t>(N));
  std::vector<std::vector<float>> grad(T, std::vector<float>(N * D)), out(T, std::vector<float>(N * D));
  for (int t = 0; t < T; ++t) {
    for (int64_t p = 0; p < N; ++p) {
      const double u = (rnd() % 100000) / 100000.0;
      ids[t][p] = (int64_t)(u * u * u * (V - 1));
    }
    for (auto& g : grad[t]) g = ((int)(rnd() % 2001) - 1000) * 1e-3f;
  }

  hipStream_t st, side;
  HIP_OK(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
  HIP_OK(hipStreamCreateWithFlags(&side, hipStreamNonBlocking));
  sfc_config cfg = {};
  cfg.capacity_rows = C; cfg.dim = D; cfg.policy = SFC_POLICY_LRU_BATCH;
  cfg.max_ids_per_batch = N; cfg.max_bags_per_batch = N; cfg.host_rows = V;
  cfg.h_weights = tab; cfg.h_acc = tab + D; cfg.host_row_stride = 2 * D; cfg.host_state_stride = 2 * D;
  cfg.lr = lr; cfg.eps = eps; cfg.lookahead = L; cfg.stream = st; cfg.side_stream = side;
  cfg.optimizer = SFC_OPT_ADAGRAD;
  sfc_cache* cache = nullptr;
  SFC_OK_OR_DIE(sfc_cache_create(&cfg, &cache));
  SFC_OK_OR_DIE(sfc_profile_enable(cache, 1));

  // one set of step buffers per step in flight; ids and gradients of every batch stay on the device
  const int nset = L + 1;
  std::vector<int64_t*> d_ids(T), d_uniq(nset);
  std::vector<int32_t*> d_inv(nset), d_slot(nset), d_miss(nset);
  std::vector<float*> d_grad(T), d_out(T);
  for (int k = 0; k < nset; ++k) {
    HIP_OK(hipMalloc(&d_uniq[k], N * 8)); HIP_OK(hipMalloc(&d_inv[k], N * 4));
    HIP_OK(hipMalloc(&d_slot[k], N * 4)); HIP_OK(hipMalloc(&d_miss[k], N * 4));
  }
  for (int t = 0; t < T; ++t) {
    HIP_OK(hipMalloc(&d_ids[t], N * 8)); HIP_OK(hipMalloc(&d_grad[t], N * D * 4)); HIP_OK(hipMalloc(&d_out[t], N * D * 4));
    HIP_OK(hipMemcpy(d_ids[t], ids[t].data(), N * 8, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_grad[t], grad[t].data(), N * D * 4, hipMemcpyHostToDevice));
  }
  std::vector<std::vector<int64_t>> uniq(T, std::vector<int64_t>(N));
  std::vector<std::vector<int32_t>> inv(T, std::vector<int32_t>(N));
  std::vector<sfc_stats> stt(T);
  int bad = 0;
  auto prepare = [&](int t) -> int {                       // prepare + copies of batch t
    const int k = t % nset;
    SFC_OK_OR_DIE(sfc_prepare(cache, d_ids[t], N, nullptr, N, d_uniq[k], d_inv[k], d_slot[k], d_miss[k]));
    SFC_OK_OR_DIE(sfc_fetch_misses(cache));
    return 0;
  };
  // lookahead L: batch t+L is prepared between the lookup and the update of batch t; nothing
  // waits on the device inside the loop
  for (int t = 0; t < L && t < T; ++t) if (int r = prepare(t)) return r;
  for (int t = 0; t < T; ++t) {
    if (L == 0) { if (int r = prepare(t)) return r; }
    SFC_OK_OR_DIE(sfc_lookup(cache, d_out[t]));
    if (L > 0 && t + L < T) { if (int r = prepare(t + L)) return r; }
    SFC_OK_OR_DIE(sfc_backward_update(cache, d_grad[t]));
    if (L == 0) {                                          // outputs of this step's prepare, while its buffers are current
      SFC_OK_OR_DIE(sfc_get_stats(cache, &stt[t]));
      HIP_OK(hipMemcpy(uniq[t].data(), d_uniq[0], N * 8, hipMemcpyDeviceToHost));
      HIP_OK(hipMemcpy(inv[t].data(), d_inv[0], N * 4, hipMemcpyDeviceToHost));
    }
  }
  SFC_OK_OR_DIE(sfc_flush(cache));
  double ms; int64_t calls;
  SFC_OK_OR_DIE(sfc_profile_read(cache, 0, &ms, &calls));
  if (calls != T) { printf("profile: %lld prepare calls timed, expected %d\n", (long long)calls, T); ++bad; }
  for (int t = 0; t < T; ++t) HIP_OK(hipMemcpy(out[t].data(), d_out[t], N * D * 4, hipMemcpyDeviceToHost));

  // the same training on the host: dense table, gradient summed per id in double, one Adagrad
  // step per id and batch
  int64_t evicted = 0;
  for (int t = 0; t < T; ++t) {
    std::map<int64_t, int> seen;
    for (int64_t p = 0; p < N; ++p) {
      auto it = seen.find(ids[t][p]);
      if (it == seen.end()) it = seen.emplace(ids[t][p], (int)seen.size()).first;
      if (L == 0 && (inv[t][p] != it->second || uniq[t][inv[t][p]] != ids[t][p])) ++bad;   // dense, first-appearance order
      for (int j = 0; j < D; ++j) {
        const double r = rw[ids[t][p] * D + j];
        if (std::fabs((double)out[t][p * D + j] - r) > 1e-6 + 1e-5 * std::fabs(r)) ++bad;
      }
    }
    if (L == 0) {
      if ((int64_t)seen.size() != stt[t].n_unique) ++bad;
      evicted += stt[t].n_evict;
      printf("step %d: unique %lld hit %lld miss %lld evict %lld bypass %lld\n", t, (long long)stt[t].n_unique,
             (long long)stt[t].n_hit, (long long)stt[t].n_miss, (long long)stt[t].n_evict, (long long)stt[t].n_bypass);
    }
    std::map<int64_t, std::vector<double>> G;
    for (int64_t p = 0; p < N; ++p) {
      auto& g = G[ids[t][p]];
      if (g.empty()) g.assign(D, 0.0);
      for (int j = 0; j < D; ++j) g[j] += (double)grad[t][p * D + j];
    }
    for (auto& kv : G)
      for (int j = 0; j < D; ++j) {
        const float g = (float)kv.second[j];
        float& a = ra[kv.first * D + j];
        float& w = rw[kv.first * D + j];
        a = a + g * g;
        w = w - lr * g / (std::sqrt(a) + eps);
      }
  }
  double worst = 0;
  for (int64_t i = 0; i < V; ++i)
    for (int j = 0; j < D; ++j) {
      const double dw = std::fabs((double)tab[i * 2 * D + j] - rw[i * D + j]);
      const double da = std::fabs((double)tab[i * 2 * D + D + j] - ra[i * D + j]);
      if (dw > 1e-6 + 1e-5 * std::fabs(rw[i * D + j]) || da > 1e-6 + 1e-5 * std::fabs(ra[i * D + j])) ++bad;
      if (dw > worst) worst = dw;
    }
  if (L == 0 && evicted == 0) { printf("the cache never evicted: the run did not exercise the write-back\n"); ++bad; }
  sfc_cache_destroy(cache);
  sfc_host_free(tab);
  printf("%s: lookahead %d, %d mismatches, worst weight difference %.3g\n", bad ? "FAILED" : "OK", L, bad, worst);
  return bad ? 1 : 0;
}
