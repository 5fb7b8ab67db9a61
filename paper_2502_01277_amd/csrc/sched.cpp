// Host-side scheduling for one GPU: the batch-size search of the paper's
// Algorithm 1 (device / GPU choice and instance counts fixed) and the portion
// scheduler of Algorithm 2 ("inference streams", Sec. III-C).  No GPU calls.
#include <algorithm>
#include <cmath>
#include <limits>
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
struct Portion { int stream; double start, end; };
struct StreamState { double duty = 0.0, inter = 0.0, max_util = 0.0; };
const double kInf = std::numeric_limits<double>::infinity();

bool portion_less(const Portion& a, const Portion& b) {
  // tightest portion first ("best fit"): by length, then start, then stream
  const double la = a.end - a.start, lb = b.end - b.start;
  if (la != lb) return la < lb;
  if (a.start != b.start) return a.start < b.start;
  return a.stream < b.stream;
}
}  // namespace

int coral_schedule(octo_sched_pipeline* ps, int n_pipelines, double mem, double util_max, int n_streams,
                   octo_placement* out) {
  std::vector<StreamState> streams(n_streams);
  std::vector<Portion> free_pts;
  for (int s = 0; s < n_streams; ++s) free_pts.push_back({s, 0.0, kInf});
  std::sort(free_pts.begin(), free_pts.end(), portion_less);
  double Wg = 0.0, Ig = 0.0;
  int o = 0;
  // one instance per model, so the fairness loop over instance numbers has a single round
  for (int pi = 0; pi < n_pipelines; ++pi) {
    octo_sched_pipeline& p = ps[pi];
    for (int mi = 0; mi < p.n_models; ++mi, ++o) {
      const octo_sched_model& m = p.models[mi];
      // window: right after all upstream portions (downstream runs immediately after upstream)
      double m_start = 0.0;
      for (int a = m.parent; a >= 0; a = p.models[a].parent) m_start += batch_ms(p.models[a]);
      const double m_end = m_start + batch_ms(m);
      const double duty_r = p.slo_ms / 2.0;
      octo_placement pl = {pi, mi, -1, 0.f, 0.f, 0.f};
      for (size_t k = 0; k < free_pts.size(); ++k) {
        const Portion pt = free_pts[k];
        StreamState& st = streams[pt.stream];
        const double w_g = Wg + m.weight_mem;
        const double i_g = Ig - st.inter + std::max(st.inter, (double)m.inter_mem);
        double u_g = std::max(st.max_util, (double)m.util);
        for (int s2 = 0; s2 < n_streams; ++s2) if (s2 != pt.stream) u_g += streams[s2].max_util;
        const double cycle = st.duty > 0 ? st.duty : duty_r;
        if (!(pt.start <= m_start && pt.end >= m_end && m_end <= cycle)) continue;
        if (!(w_g + i_g <= mem && u_g <= util_max + 1e-12)) continue;
        if (!(duty_r >= st.duty)) continue;
        double pt_end = pt.end;
        if (st.duty == 0) {
          st.duty = duty_r;
          for (Portion& q : free_pts) if (q.stream == pt.stream && q.end == kInf) q.end = duty_r;
          if (pt_end == kInf) pt_end = duty_r;
        }
        Wg = w_g; Ig = i_g;
        st.inter = std::max(st.inter, (double)m.inter_mem);
        st.max_util = std::max(st.max_util, (double)m.util);
        free_pts.erase(free_pts.begin() + k);
        if (m_start > pt.start) free_pts.push_back({pt.stream, pt.start, m_start});
        if (pt_end > m_end) free_pts.push_back({pt.stream, m_end, pt_end});
        std::sort(free_pts.begin(), free_pts.end(), portion_less);
        pl.stream = pt.stream; pl.start_ms = (float)m_start; pl.end_ms = (float)m_end; pl.duty_cycle_ms = (float)st.duty;
        break;
      }
      out[o] = pl;
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
