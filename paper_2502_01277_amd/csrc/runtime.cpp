// Run-time rules of the serving loop, host only: what an executor decides around the scheduler's output.  The paper
// names these in prose (burstiness: Sec. III-B; portions: Sec. III-C; horizontal scaling: Sec. III-D; lazy dropping:
// Sec. IV-A); the readings are stated at the declarations in include/octo.h.
#include <algorithm>
#include <cmath>
#include <deque>
#include <new>
#include <numeric>
#include <vector>

#include "../../include/octo.h"

// Sliding window of the last `window` duty cycles of one pipeline.
struct octo_scaler {
  double capacity = 0.0;     // requests one instance serves per duty cycle
  int window = 0;
  double up = 1.0, down = 0.75;
  int max_instances = 2;
  std::deque<long long> arrived, backlog;

  void forget() { arrived.clear(); backlog.clear(); }
  bool window_full() const { return (int)arrived.size() >= window; }
  double mean_arrivals() const { return (double)std::accumulate(arrived.begin(), arrived.end(), 0LL) / (double)window; }
  long long least_backlog() const { return *std::min_element(backlog.begin(), backlog.end()); }
};

extern "C" {

octo_status octo_burstiness(const double* times, int32_t n, double* cv) {
  if (!cv || n < 0 || (n > 0 && !times)) return OCTO_EINVAL;
  *cv = 0.0;
  if (n < 3) return OCTO_OK;
  std::vector<double> t(times, times + n);
  std::sort(t.begin(), t.end());
  const int m = n - 1;                       // gaps
  double mean = 0.0;
  for (int i = 0; i < m; ++i) mean += t[i + 1] - t[i];
  mean /= m;
  if (!(mean > 0.0)) return OCTO_OK;
  double var = 0.0;
  for (int i = 0; i < m; ++i) { const double d = (t[i + 1] - t[i]) - mean; var += d * d; }
  *cv = std::sqrt(var / m) / mean;
  return OCTO_OK;
}

octo_status octo_batches_per_cycle(double rate_per_s, double duty_ms, int32_t bz, int32_t* k) {
  if (!k || bz < 1 || !(rate_per_s >= 0.0) || !(duty_ms > 0.0)) return OCTO_EINVAL;
  const double need = rate_per_s * duty_ms / 1000.0 / (double)bz;
  const long long c = (long long)std::ceil(need - 1e-9);
  *k = (int32_t)std::max<long long>(1, std::min<long long>(c, 1LL << 30));
  return OCTO_OK;
}

octo_status octo_width_to_cus(double util, int32_t total_cus, int32_t grain, int32_t* n_cu) {
  if (!n_cu || total_cus < 1 || grain < 1 || grain > total_cus || !(util >= 0.0)) return OCTO_EINVAL;
  const long long groups = (long long)std::ceil(util * (double)total_cus / (double)grain - 1e-9);
  const long long n = std::min<long long>(total_cus, std::max<long long>(grain, groups * grain));
  *n_cu = (int32_t)n;
  return OCTO_OK;
}

octo_status octo_choose_width(const int32_t* widths, const double* latency_ms, int32_t n, int32_t by_cost, double tol, int32_t* width) {
  if (!widths || !latency_ms || !width || n < 1 || !(tol >= 0.0)) return OCTO_EINVAL;
  std::vector<int> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::sort(order.begin(), order.end(), [&](int a, int b) { return widths[a] < widths[b]; });
  for (int i = 0; i < n; ++i)
    if (widths[i] < 1 || !(latency_ms[i] > 0.0)) return OCTO_EINVAL;
  // what a width is judged by: its latency, or what it costs in compute-unit-milliseconds
  auto score = [&](int i) { return by_cost ? (double)widths[i] * latency_ms[i] : latency_ms[i]; };
  double target;
  if (by_cost) {
    target = score(order[0]);
    for (int i : order) target = std::min(target, score(i));
  } else {
    target = score(order[n - 1]);            // the widest stream's latency
  }
  *width = widths[order[n - 1]];
  for (int i : order)
    if (score(i) <= (1.0 + tol) * target) { *width = widths[i]; break; }
  return OCTO_OK;
}

octo_status octo_late_prefix(const double* arrival_ms, int32_t n, double now_ms, double slo_ms, int32_t* n_late) {
  if (!n_late || n < 0 || (n > 0 && !arrival_ms)) return OCTO_EINVAL;
  int32_t k = 0;
  while (k < n && now_ms - arrival_ms[k] > slo_ms) ++k;
  *n_late = k;
  return OCTO_OK;
}

octo_status octo_plan_pipeline(const octo_plan_model* models, int32_t n_models, float slo_ms, double duty_ms, double cycle_share,
                               const int32_t* widths, int32_t n_widths, int32_t total_cus, const int32_t* fixed_bz,
                               octo_sched_model* out, int32_t* batches_per_cycle, float* est_latency_ms, float* est_throughput) {
  if (!models || !widths || !out || !batches_per_cycle || n_models < 1 || n_widths < 1 || n_widths > OCTO_MAX_WIDTHS || total_cus < 1 ||
      !(duty_ms > 0.0) || !(cycle_share > 0.0))
    return OCTO_EINVAL;
  std::vector<int> order(n_widths);
  std::iota(order.begin(), order.end(), 0);
  std::sort(order.begin(), order.end(), [&](int a, int b) { return widths[a] < widths[b]; });
  auto column_of = [&](int w) { for (int j = 0; j < n_widths; ++j) if (widths[j] == w) return j; return -1; };
  for (int i = 0; i < n_models; ++i)
    if (models[i].n_profile < 1 || models[i].n_profile > 8 || column_of(models[i].width) < 0) return OCTO_EINVAL;
  std::vector<octo_sched_model> trial(n_models);
  octo_sched_pipeline p{trial.data(), n_models, slo_ms};
  for (int f = 0; f < n_widths; ++f) {
    const int floor_w = widths[order[f]];
    for (int i = 0; i < n_models; ++i) {
      const octo_plan_model& m = models[i];
      const int w = std::max(floor_w, m.width);          // a profiled width: the floor or the model's own
      const int col = column_of(w);
      octo_sched_model& t = trial[i];
      t = octo_sched_model{};
      t.parent = m.parent; t.n_profile = m.n_profile;
      for (int k = 0; k < m.n_profile; ++k) { t.profile_bz[k] = m.profile_bz[k]; t.profile_ms[k] = m.profile_ms[col][k]; }
      t.rate = std::max(m.rate, 1e-3f); t.burstiness = m.burstiness; t.util = (float)w / (float)total_cus;
      t.weight_mem = m.weight_mem; t.inter_mem = m.inter_mem; t.bz = 1;
    }
    if (fixed_bz) {
      for (int i = 0; i < n_models; ++i) trial[i].bz = fixed_bz[i];
    } else {
      const octo_status st = octo_cwd_search(&p);
      if (st != OCTO_OK) return st;
    }
    double work = 0.0;
    for (int i = 0; i < n_models; ++i) {
      const octo_sched_model& t = trial[i];
      int slot = -1;
      for (int k = 0; k < t.n_profile; ++k) if (t.profile_bz[k] == t.bz) slot = k;
      if (slot < 0) return OCTO_EINVAL;                   // a batch size without a profile entry
      const octo_status st = octo_batches_per_cycle(t.rate, duty_ms, t.bz, &batches_per_cycle[i]);
      if (st != OCTO_OK) return st;
      work += (double)batches_per_cycle[i] * (double)t.profile_ms[slot];
    }
    if (work <= cycle_share * duty_ms) break;             // the widest floor is taken whatever its work
  }
  if (est_latency_ms) *est_latency_ms = octo_est_latency_ms(&p);
  if (est_throughput) *est_throughput = octo_est_throughput(&p);
  for (int i = 0; i < n_models; ++i) {
    out[i] = trial[i];
    for (int k = 0; k < out[i].n_profile; ++k)
      if (out[i].profile_bz[k] == out[i].bz) out[i].profile_ms[k] *= (float)batches_per_cycle[i];      // the portion holds k back-to-back batches
  }
  return OCTO_OK;
}

octo_status octo_scaler_create(double capacity, int32_t window, double up, double down, int32_t max_instances, octo_scaler** out) {
  if (!out || !(capacity > 0.0) || window < 1 || !(down > 0.0) || !(down < up) || max_instances < 1) return OCTO_EINVAL;
  octo_scaler* s = new (std::nothrow) octo_scaler;
  if (!s) return OCTO_ENOMEM;
  s->capacity = capacity; s->window = window; s->up = up; s->down = down; s->max_instances = max_instances;
  *out = s;
  return OCTO_OK;
}

octo_status octo_scaler_observe(octo_scaler* s, int64_t arrived, int64_t backlog, int32_t n_active, int32_t* decision) {
  if (!s || !decision || arrived < 0 || backlog < 0 || n_active < 1) return OCTO_EINVAL;
  *decision = 0;
  s->arrived.push_back(arrived);
  s->backlog.push_back(backlog);
  while ((int)s->arrived.size() > s->window) { s->arrived.pop_front(); s->backlog.pop_front(); }
  if (!s->window_full()) return OCTO_OK;
  const double mean = s->mean_arrivals();
  const double served_now = s->capacity * n_active, served_with_one_fewer = s->capacity * (n_active - 1);
  const bool overloaded = mean > s->up * served_now || (double)s->least_backlog() > served_now;
  const bool idle = mean < s->down * served_with_one_fewer && (double)s->backlog.back() <= served_with_one_fewer;
  if (n_active < s->max_instances && overloaded) { *decision = 1; s->forget(); }
  else if (n_active > 1 && idle) { *decision = -1; s->forget(); }
  return OCTO_OK;
}

octo_status octo_scaler_destroy(octo_scaler* s) {
  if (!s) return OCTO_EINVAL;
  delete s;
  return OCTO_OK;
}

}  // extern "C"
