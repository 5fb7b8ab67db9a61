// Cross-device placement of one pipeline (host only): the function ToEdge of the paper's Algorithm 1 (Sec. III-B) for two
// devices, the server and the edge device at the data source, joined by a link of given bandwidth.  The readings of what
// the paper leaves open (the estimates with the network term of Eq. (1), what "a new configuration only for m" searches,
// Overhead()) are stated at the declaration in include/octo.h.
#include <algorithm>
#include <limits>
#include <numeric>
#include <vector>

#include "../../include/octo.h"

namespace {

// The pipeline under placement: the caller's models plus the link.
class Deployment {
 public:
  Deployment(octo_place_model* m, int n, double slo_ms, double bytes_per_s, double alpha)
      : m_(m), n_(n), budget_ms_(slo_ms / 2.0), bw_(bytes_per_s), alpha_(alpha), kids_(n) {
    for (int i = 1; i < n; ++i) kids_[m[i].parent].push_back(i);
  }

  // depth-first from model i: move it to the edge if some batch size works there, descend, and undo the move if the model
  // turns out to be a poor split point
  void descend(int i) {
    const int bz_before = m_[i].bz, edge_before = m_[i].on_edge;
    const int bz = best_edge_batch(i);
    if (bz == 0) { m_[i].bz = bz_before; m_[i].on_edge = edge_before; return; }
    m_[i].bz = bz; m_[i].on_edge = 1;
    std::vector<int> order(kids_[i]);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return m_[a].burstiness < m_[b].burstiness; });
    for (int c : order) descend(c);
    bool downstream_on_edge = false;
    double out_rate = 0.0;                     // bytes per second the model's output puts on the network if the split is after it
    for (int c : kids_[i]) { downstream_on_edge |= m_[c].on_edge != 0; out_rate += (double)m_[c].rate * m_[c].in_bytes; }
    if (kids_[i].empty()) out_rate = (double)m_[i].rate * m_[i].result_bytes;
    const double in_rate = (double)m_[i].rate * m_[i].in_bytes;
    if (in_rate * alpha_ < out_rate && !downstream_on_edge) { m_[i].bz = bz_before; m_[i].on_edge = edge_before; }
  }

  double worst_latency_ms() const {
    double worst = 0.0;
    for (int leaf = 0; leaf < n_; ++leaf) {
      if (!kids_[leaf].empty()) continue;
      double sum = 0.0;
      for (int i = leaf; i >= 0; i = m_[i].parent) sum += batch_ms(i) + (m_[i].bz - 1) * 1000.0 / m_[i].rate + link_ms(i);
      worst = std::max(worst, sum);
    }
    return worst;
  }
  double throughput() const {
    double per_request_ms = 0.0;
    for (int i = 0; i < n_; ++i) per_request_ms += batch_ms(i) / m_[i].bz + link_ms(i);
    return 1000.0 / per_request_ms;
  }

 private:
  double batch_ms(int i) const {
    const float* table = m_[i].on_edge ? m_[i].edge_ms : m_[i].server_ms;
    for (int k = 0; k < m_[i].n_profile; ++k) if (m_[i].profile_bz[k] == m_[i].bz) return table[k];
    return std::numeric_limits<double>::infinity();
  }
  // a request crosses the link iff the model and what feeds it (for the root: the data source, at the edge) are on different devices
  double link_ms(int i) const {
    const int fed_from_edge = m_[i].parent < 0 ? 1 : m_[m_[i].parent].on_edge;
    return fed_from_edge != m_[i].on_edge ? 1000.0 * m_[i].in_bytes / bw_ : 0.0;
  }
  double edge_seconds_per_second() const {
    double s = 0.0;
    for (int i = 0; i < n_; ++i) if (m_[i].on_edge) s += (double)m_[i].rate * batch_ms(i) / m_[i].bz / 1000.0;
    return s;
  }
  // the profiled batch size with the largest throughput estimate among those that keep the latency estimate within half
  // the objective and the edge device within its compute (smallest on ties); 0 if none.  Leaves the model on the edge.
  int best_edge_batch(int i) {
    int best = 0;
    double best_thr = 0.0;
    m_[i].on_edge = 1;
    for (int k = 0; k < m_[i].n_profile; ++k) {            // profile_bz ascends
      m_[i].bz = m_[i].profile_bz[k];
      if (worst_latency_ms() > budget_ms_ || edge_seconds_per_second() > 1.0) continue;
      const double thr = throughput();
      if (best == 0 || thr > best_thr) { best = m_[i].bz; best_thr = thr; }
    }
    return best;
  }

  octo_place_model* m_;
  int n_;
  double budget_ms_, bw_, alpha_;
  std::vector<std::vector<int>> kids_;
};

}  // namespace

extern "C" octo_status octo_to_edge(octo_place_model* models, int32_t n_models, float slo_ms, double bandwidth_bytes_per_s, double alpha,
                                    float* est_latency_ms, float* est_throughput) {
  if (!models || n_models < 1 || !(slo_ms > 0.f) || !(bandwidth_bytes_per_s > 0.0) || !(alpha > 0.0)) return OCTO_EINVAL;
  for (int i = 0; i < n_models; ++i) {
    const octo_place_model& m = models[i];
    if (m.parent >= i || (i == 0) != (m.parent < 0) || m.n_profile < 1 || m.n_profile > 8 || !(m.rate > 0.f) || !(m.in_bytes >= 0.0) || !(m.result_bytes >= 0.0))
      return OCTO_EINVAL;
    bool has = false;
    for (int k = 0; k < m.n_profile; ++k) {
      has |= m.profile_bz[k] == m.bz;
      if (k > 0 && m.profile_bz[k] <= m.profile_bz[k - 1]) return OCTO_EINVAL;
    }
    if (!has) return OCTO_EINVAL;
    models[i].on_edge = 0;
  }
  Deployment d(models, n_models, slo_ms, bandwidth_bytes_per_s, alpha);
  d.descend(0);
  if (est_latency_ms) *est_latency_ms = (float)d.worst_latency_ms();
  if (est_throughput) *est_throughput = (float)d.throughput();
  return OCTO_OK;
}
