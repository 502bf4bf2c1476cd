// Control-plane formulas of the paper, host code only: the corrective
// seasonal predictor (Sec. 3.1, Eq. 1-3), the prewarming scores (App. B.1) and
// the placement algorithm (Sec. 3.2 Alg. 1, App. B.2).  Double precision.
#include <algorithm>
#include <cmath>
#include <limits>
#include <vector>

#include "common.h"

namespace warmkv {
namespace {

inline double hist(const double* h, uint32_t n_windows, uint32_t day, uint32_t window) {
  return h[(size_t)day * n_windows + window];
}

// Eq. 1: mean of the same window over the D previous days.
double seasonal(const double* h, uint32_t n_windows, uint32_t day, uint32_t window, uint32_t D) {
  double sum = 0.0;
  for (uint32_t d = 1; d <= D; ++d) sum += hist(h, n_windows, day - d, window);
  return sum / (double)D;
}

struct Counts {
  uint32_t basic, burst;
};

Counts replica_counts(const ws_model& m) {
  const double need_avg = std::ceil(m.load_avg / (double)m.batch);
  const double need_peak = std::ceil(m.load_peak / (double)m.batch);
  const double basic = std::max(need_avg - (double)m.active, 0.0);
  const double burst = std::max(need_peak - basic - (double)m.active, 0.0);
  return {(uint32_t)basic, (uint32_t)burst};
}

double replica_score(const ws_model& m, const Counts& c, bool burst, uint32_t i) {
  const double total = (double)c.basic + (double)c.burst;
  if (!burst) return std::exp(-(double)i / total) * m.cold_latency;
  const double burstiness = m.load_avg == 0.0 ? std::numeric_limits<double>::infinity()
                                              : (m.load_peak - m.load_avg) / m.load_avg;
  return std::exp(-((double)c.basic + (double)i) / total) * m.cold_latency * burstiness;
}

bool model_ok(const ws_model& m) {
  return m.batch >= 1 && m.degree >= 1 && m.load_avg >= 0.0 && m.load_peak >= 0.0 && m.size_bytes >= 0.0 &&
         m.load_peak / (double)m.batch < 1e6;
}

}  // namespace
}  // namespace warmkv

using namespace warmkv;

extern "C" int ws_predict_load(const double* history, uint32_t n_days, uint32_t n_windows, uint32_t day,
                               uint32_t window, uint32_t D, uint32_t N, double* prediction) {
  if (history == nullptr || prediction == nullptr) return KV_E_NULL;
  if (D == 0 || day < D || day >= n_days || window >= n_windows || N > 62) return KV_E_RANGE;
  const double p = seasonal(history, n_windows, day, window, D);
  const uint32_t m = window < N ? window : N;
  double delta = 0.0;
  if (m != 0) {
    double acc = 0.0;
    for (uint32_t w = 1; w <= m; ++w)  // Eq. 2
      acc += (hist(history, n_windows, day, window - w) - seasonal(history, n_windows, day, window - w, D)) *
             (double)(1ull << (w - 1));
    delta = acc / (double)((1ull << m) - 1ull);
  }
  *prediction = p + delta;  // Eq. 3
  return KV_OK;
}

extern "C" int ws_replica_scores(const ws_model* model, uint32_t* n_basic, uint32_t* n_burst, double* scores,
                                 uint32_t capacity) {
  if (model == nullptr || n_basic == nullptr || n_burst == nullptr) return KV_E_NULL;
  if (!model_ok(*model)) return KV_E_RANGE;
  const Counts c = replica_counts(*model);
  *n_basic = c.basic;
  *n_burst = c.burst;
  if ((uint64_t)c.basic + c.burst > capacity) return KV_E_TOOBIG;
  if (c.basic + c.burst != 0 && scores == nullptr) return KV_E_NULL;
  for (uint32_t i = 0; i < c.basic; ++i) scores[i] = replica_score(*model, c, false, i);
  for (uint32_t i = 0; i < c.burst; ++i) scores[c.basic + i] = replica_score(*model, c, true, i);
  return KV_OK;
}

extern "C" int ws_place_replicas(const ws_model* models, uint32_t n_models, double* gpu_free_bytes,
                                 uint32_t n_gpus, uint32_t gpus_per_server, ws_placement* out, uint32_t capacity,
                                 uint32_t* n_out) {
  return guarded([&]() -> int {
    if (n_out == nullptr || (n_models != 0 && models == nullptr) || (n_gpus != 0 && gpu_free_bytes == nullptr))
      return KV_E_NULL;
    if (gpus_per_server == 0 || n_gpus % gpus_per_server != 0) return KV_E_RANGE;
    struct Replica {
      uint32_t model, index, burst;
      double score;
    };
    std::vector<Replica> replicas;
    for (uint32_t i = 0; i < n_models; ++i) {
      if (!model_ok(models[i]) || gpus_per_server % models[i].degree != 0) return KV_E_RANGE;
      const Counts c = replica_counts(models[i]);
      for (uint32_t r = 0; r < c.basic; ++r) replicas.push_back({i, r, 0u, replica_score(models[i], c, false, r)});
      for (uint32_t r = 0; r < c.burst; ++r) replicas.push_back({i, c.basic + r, 1u, replica_score(models[i], c, true, r)});
    }
    std::stable_sort(replicas.begin(), replicas.end(), [](const Replica& a, const Replica& b) {
      if (a.burst != b.burst) return a.burst < b.burst;  // basic replicas always come first
      if (a.score != b.score) return a.score > b.score;
      if (a.model != b.model) return a.model < b.model;
      return a.index < b.index;
    });
  
    std::vector<double> free_bytes(gpu_free_bytes, gpu_free_bytes + n_gpus);  // committed only on success
    std::vector<ws_placement> placed;
    const double inf = std::numeric_limits<double>::infinity();
    for (const Replica& r : replicas) {
      const ws_model& m = models[r.model];
      const double need = std::ceil(m.size_bytes / (double)m.degree);
      int64_t best = -1, best_isolated = -1;
      double best_sum = inf, best_isolated_sum = inf;
      for (uint32_t g = 0; g + m.degree <= n_gpus; g += m.degree) {
        bool fits = true;
        for (uint32_t j = g; j < g + m.degree; ++j) fits = fits && free_bytes[j] >= need;
        if (!fits) continue;
        // H and R over the replicas that share a GPU with this group (aligned groups nest, so such
        // a replica either covers the group or lies inside it)
        double high = -inf, sum = 0.0;
        for (const ws_placement& q : placed) {
          const uint32_t q_end = q.first_gpu + models[q.model].degree;
          if (q.first_gpu < g + m.degree && g < q_end) {
            high = std::max(high, q.score);
            sum += q.score;
          }
        }
        if (best < 0 || sum < best_sum) { best_sum = sum; best = g; }
        if (high < r.score && (best_isolated < 0 || sum < best_isolated_sum)) { best_isolated_sum = sum; best_isolated = g; }
      }
      if (best < 0) continue;  // no group has room: next replica
      const uint32_t g = (uint32_t)(best_isolated >= 0 ? best_isolated : best);
      for (uint32_t j = g; j < g + m.degree; ++j) free_bytes[j] -= need;
      placed.push_back({r.model, r.index, g, r.burst, r.score});
    }
    *n_out = (uint32_t)placed.size();
    if (placed.size() > capacity) return KV_E_TOOBIG;
    if (!placed.empty() && out == nullptr) return KV_E_NULL;
    std::copy(placed.begin(), placed.end(), out);
    std::copy(free_bytes.begin(), free_bytes.end(), gpu_free_bytes);
    return KV_OK;
  });
}
