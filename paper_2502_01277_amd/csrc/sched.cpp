// Host-side scheduling for one GPU: the batch-size search of the paper's
// Algorithm 1 (device / GPU choice and instance counts fixed) and the portion
// scheduler of Algorithm 2 ("inference streams", Sec. III-C).  No GPU calls.
#include <algorithm>
#include <cmath>
#include <limits>
#include <set>
#include <vector>

#include "octo_internal.h"

namespace octo {
namespace {

float profile_ms(const octo_sched_model& m, int bz, bool* found) {
  for (int i = 0; i < m.n_profile; ++i)
    if (m.profile_bz[i] == bz) { *found = true; return m.profile_ms[i]; }
  *found = false;
  return 0.f;
}

double batch_ms(const octo_sched_model& m) {
  bool ok;
  float v = profile_ms(m, m.bz, &ok);
  return ok ? v : std::numeric_limits<double>::infinity();
}

}  // namespace

// Worst case of the first request of a batch (Sec. II, constraint a) along the longest root-to-leaf path:
// batch latency plus the time for bz-1 more requests to arrive.  (EstLat is not defined in the paper.)
double est_latency(const octo_sched_pipeline* p) {
  double worst = 0.0;
  for (int leaf = 0; leaf < p->n_models; ++leaf) {
    bool is_leaf = true;
    for (int j = 0; j < p->n_models; ++j) if (p->models[j].parent == leaf) is_leaf = false;
    if (!is_leaf) continue;
    double sum = 0.0;
    for (int i = leaf; i >= 0; i = p->models[i].parent) {
      const octo_sched_model& m = p->models[i];
      sum += batch_ms(m) + (m.bz - 1) * 1000.0 / m.rate;
    }
    worst = std::max(worst, sum);
  }
  return worst;
}

// Eq. (2) for one pipeline, same-device IO term dropped: 1 / sum_m (L_{m|bz} / bz), in results per second.
double est_throughput(const octo_sched_pipeline* p) {
  double s = 0.0;
  for (int i = 0; i < p->n_models; ++i) s += batch_ms(p->models[i]) / p->models[i].bz;
  return 1000.0 / s;
}

int cwd_search(octo_sched_pipeline* p) {
  const int n = p->n_models;
  for (int i = 0; i < n; ++i) p->models[i].bz = 1;
  double best = est_throughput(p);
  std::vector<int> order(n);
  for (int i = 0; i < n; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(),
                   [&](int a, int b) { return p->models[a].burstiness > p->models[b].burstiness; });
  bool adopted = true;
  while (adopted) {
    adopted = false;
    for (int i : order) {
      octo_sched_model& m = p->models[i];
      m.bz *= 2;
      bool has;
      profile_ms(m, m.bz, &has);
      if (!has || est_latency(p) > p->slo_ms / 2.0) { m.bz /= 2; continue; }
      const double thr = est_throughput(p);
      if (thr > best) { best = thr; adopted = true; }
      else m.bz /= 2;
    }
  }
  return 0;
}

namespace {
const double kInf = std::numeric_limits<double>::infinity();

// A free stretch of an inference stream's duty cycle.  Ordered by tightness, so that walking the set visits the
// smallest gap that can hold a window first ("best fit"); ties by start, then stream.
struct Gap {
  int lane; double begin, end;
  double length() const { return end - begin; }
  bool operator<(const Gap& o) const {
    if (length() != o.length()) return length() < o.length();
    if (begin != o.begin) return begin < o.begin;
    return lane < o.lane;
  }
};

// What a model asks of the GPU: a window inside the duty cycle of its pipeline, memory, and a share of compute.
struct Need { double begin, end, cycle, weights, scratch, width; };

// One GPU as Algorithm 2 sees it (Sec. III-C): inference streams ("lanes"), each with the duty cycle of the first
// pipeline placed on it, the widest portion it holds (a stream reserves that width for its whole cycle) and the largest
// intermediate buffer of its models (models of one stream run one after the other and share it); weights add up.
class GpuLedger {
 public:
  GpuLedger(int n_lanes, double mem_cap, double width_cap) : lanes_(n_lanes), mem_cap_(mem_cap), width_cap_(width_cap) {
    for (int l = 0; l < n_lanes; ++l) gaps_.insert({l, 0.0, kInf});
  }
  // the tightest gap that can take the need, or end()
  std::set<Gap>::const_iterator find(const Need& n) const {
    for (auto it = gaps_.begin(); it != gaps_.end(); ++it)
      if (admits(*it, n)) return it;
    return gaps_.end();
  }
  std::set<Gap>::const_iterator none() const { return gaps_.end(); }
  // book the need into the gap; returns the duty cycle of the gap's lane
  double book(std::set<Gap>::const_iterator it, const Need& n) {
    Gap g = *it;
    gaps_.erase(it);
    Lane& lane = lanes_[g.lane];
    if (lane.cycle == 0.0) {                 // first portion of this lane: the lane takes the pipeline's cycle, open ends close there
      lane.cycle = n.cycle;
      std::vector<Gap> open;
      for (auto q = gaps_.begin(); q != gaps_.end();)
        if (q->lane == g.lane && q->end == kInf) { open.push_back(*q); q = gaps_.erase(q); } else ++q;
      for (Gap& q : open) { q.end = n.cycle; gaps_.insert(q); }
      if (g.end == kInf) g.end = n.cycle;
    }
    weights_ += n.weights;
    lane.scratch = std::max(lane.scratch, n.scratch);
    lane.widest = std::max(lane.widest, n.width);
    if (n.begin > g.begin) gaps_.insert({g.lane, g.begin, n.begin});       // what is left before and after the window
    if (g.end > n.end) gaps_.insert({g.lane, n.end, g.end});
    return lane.cycle;
  }

 private:
  struct Lane { double cycle = 0.0, widest = 0.0, scratch = 0.0; };
  bool admits(const Gap& g, const Need& n) const {
    const Lane& lane = lanes_[g.lane];
    if (n.cycle < lane.cycle) return false;                                 // the lane repeats faster than this pipeline may wait
    const double cycle = lane.cycle > 0.0 ? lane.cycle : n.cycle;
    if (g.begin > n.begin || g.end < n.end || n.end > cycle) return false;  // the window must lie inside the gap and the cycle
    double scratch = std::max(lane.scratch, n.scratch), width = std::max(lane.widest, n.width);
    for (size_t l = 0; l < lanes_.size(); ++l)
      if ((int)l != g.lane) { scratch += lanes_[l].scratch; width += lanes_[l].widest; }
    return weights_ + n.weights + scratch <= mem_cap_ && width <= width_cap_ + 1e-12;
  }
  std::vector<Lane> lanes_;
  std::set<Gap> gaps_;
  double weights_ = 0.0, mem_cap_, width_cap_;
};
}  // namespace

// Algorithm 2 with one instance per model: pipelines in order, models in topological order; a model's window starts
// where its ancestors' batches end (a downstream model runs right after its upstream one).
int coral_schedule(octo_sched_pipeline* ps, int n_pipelines, double mem, double util_max, int n_streams,
                   octo_placement* out) {
  GpuLedger gpu(n_streams, mem, util_max);
  int o = 0;
  for (int pi = 0; pi < n_pipelines; ++pi) {
    const octo_sched_pipeline& p = ps[pi];
    for (int mi = 0; mi < p.n_models; ++mi, ++o) {
      const octo_sched_model& m = p.models[mi];
      Need need{0.0, 0.0, p.slo_ms / 2.0, m.weight_mem, m.inter_mem, m.util};
      for (int a = m.parent; a >= 0; a = p.models[a].parent) need.begin += batch_ms(p.models[a]);
      need.end = need.begin + batch_ms(m);
      out[o] = octo_placement{pi, mi, -1, 0.f, 0.f, 0.f};
      const auto gap = gpu.find(need);
      if (gap == gpu.none()) continue;
      const int lane = gap->lane;
      const double cycle = gpu.book(gap, need);
      out[o] = octo_placement{pi, mi, lane, (float)need.begin, (float)need.end, (float)cycle};
    }
  }
  return 0;
}

}  // namespace octo

extern "C" {

octo_status octo_cwd_search(octo_sched_pipeline* p) {
  if (!p || !p->models || p->n_models <= 0 || !(p->slo_ms > 0)) return OCTO_EINVAL;
  for (int i = 0; i < p->n_models; ++i) {
    const octo_sched_model& m = p->models[i];
    if (m.parent >= i || m.n_profile < 1 || m.n_profile > 8 || m.profile_bz[0] != 1 || !(m.rate > 0)) return OCTO_EINVAL;
  }
  octo::cwd_search(p);
  return OCTO_OK;
}

octo_status octo_coral_schedule(octo_sched_pipeline* ps, int32_t n_pipelines, double gpu_mem, double util_max,
                                int32_t n_streams, octo_placement* out) {
  if (!ps || !out || n_pipelines <= 0 || n_streams <= 0 || n_streams > 64) return OCTO_EINVAL;
  for (int k = 0; k < n_pipelines; ++k) {
    if (!ps[k].models || ps[k].n_models <= 0) return OCTO_EINVAL;
    for (int i = 0; i < ps[k].n_models; ++i) {
      const octo_sched_model& m = ps[k].models[i];
      bool has = false;
      for (int j = 0; j < m.n_profile && j < 8; ++j) has |= m.profile_bz[j] == m.bz;
      if (m.parent >= i || !has) return OCTO_EINVAL;
    }
  }
  octo::coral_schedule(ps, n_pipelines, gpu_mem, util_max, n_streams, out);
  return OCTO_OK;
}

float octo_est_latency_ms(const octo_sched_pipeline* p) { return p ? (float)octo::est_latency(p) : 0.f; }
float octo_est_throughput(const octo_sched_pipeline* p) { return p ? (float)octo::est_throughput(p) : 0.f; }

}  // extern "C"
