// Slot executor: co-located serving of several pipelines on one GPU (Sec. III-C "Inference Stream", Sec. III-D).
//
// Every duty cycle, at the start of a pipeline instance's portion, the instance's detector is launched on what is
// queued for it (at most its batch size per batch, at most batches-per-cycle + 1 batches per slot); its downstream
// models follow on the streams of their own portions.  Requests come from cameras with given arrival times; a request
// already older than the objective when a batch is formed is dropped if lazy dropping is on (Sec. IV-A).  Once per
// cycle every queue with a stand-by instance asks its scaler (octo_scaler_observe) whether to switch the copy on or
// off; a copy that is switched on gets its portions from Algorithm 2 run over the scheduled pipelines followed by the
// active copies (Sec. III-D: "scheduled as described earlier"), so scheduled portions stay where they are.
//
// The loop only uses the library's public calls (octo_submit_frames, octo_run_model, octo_collect, the run-time
// rules, octo_coral_schedule, octo_stream_create_range); it owns no GPU state besides the streams it creates for
// newly placed copies and the index tables of the planted-head pools.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstring>
#include <map>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "../../include/octo.h"

namespace {

constexpr int MAX_IN_FLIGHT = 6;      // uncollected batches per instance (the library holds result slots for 7)
constexpr int CU_GRAIN = 8;

// dst[j] = pool[idx[first + j]] for j < n: rows of row_bytes, copied as 16-byte vectors (VEC) or bytes
template <bool VEC>
__global__ void gather_rows_kernel(const unsigned char* __restrict__ pool, unsigned char* __restrict__ dst, const long long* __restrict__ idx,
                                   long long first, int n, size_t row_bytes) {
  const size_t per_row = VEC ? row_bytes / 16 : row_bytes;
  const size_t total = per_row * (size_t)n;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const size_t j = i / per_row, k = i - j * per_row;
    const unsigned char* s = pool + (size_t)idx[first + (long long)j] * row_bytes;
    unsigned char* d = dst + j * row_bytes;
    if (VEC) ((uint4*)d)[k] = ((const uint4*)s)[k];
    else d[k] = s[k];
  }
}

struct Request { long long id; int pool_index; const void* frame; size_t pitch; double arrival_ms; };
struct Arrival { double t_s; int cam; int seq; };

struct Queue {
  octo_exec_queue d{};
  std::vector<const void*> head_pool;
  std::vector<size_t> head_item_bytes;
  std::vector<Arrival> merged;          // arrivals of all its cameras, by time
  size_t next_arrival = 0, arrival_mark = 0;
  long long next_id = 0;
  std::vector<Request> waiting;         // admitted, not yet in a batch (arrival order)
  long long* d_seq = nullptr;           // device: pool index of every request id
  octo_scaler* scaler = nullptr;
  int standby = -1;                     // instance index of its stand-by copy
  // statistics
  long long submitted = 0, served = 0, slo_met = 0, boxes = 0, dropped = 0;
  std::vector<float> latency_ms;
  // kept results
  struct Kept { long long id; int pool_index; int box_begin, n_boxes; };
  std::vector<Kept> kept;
  std::vector<octo_box> kept_boxes;
  std::map<long long, int> pool_of;
};

struct Instance {
  octo_exec_instance d{};
  std::vector<void*> streams;
  std::vector<void*> head_buffers;
  bool active = true;
  int inflight = 0;
  std::vector<long long> batch_last;    // id of the last frame of every uncollected batch
  float slot_ms = 0.f;
};

struct Camera {
  octo_exec_camera d{};
  std::vector<double> arrivals;
  std::vector<const void*> frames;
  std::vector<size_t> pitches;
};

}  // namespace

struct octo_executor {
  std::vector<Queue> queues;
  std::vector<Instance> inst;
  std::vector<Camera> cams;
  float duty_ms = 0.f;
  bool slotted = true, drop_late = false, keep_results = false, masked = true;
  void* plain_stream = nullptr;
  int total_cus = 0;
  // Algorithm 2's inputs for the scheduled pipelines and the streams its placements refer to
  std::vector<std::vector<octo_sched_model>> sched_models;
  std::vector<float> sched_slo;
  double gpu_mem = 0; int n_streams = 0;
  std::map<int, void*> stream_handle;
  std::map<int, std::pair<int, int>> stream_cus;
  std::vector<void*> owned_streams;
  std::vector<octo_scale_event> events;
  double t0_ms = 0;
  std::vector<octo_frame_result> fr_buf;
  std::vector<octo_box> bx_buf;
  std::string err;

  octo_status fail(octo_status s, const std::string& what) { err = what; return s; }

  // planted mode: the head tensors of requests first .. first + n - 1 of a queue go from the pool into the buffers decode reads
  octo_status gather_heads(Instance& I, const long long* d_idx, long long first, int n, void* stream) {
    if (I.head_buffers.empty()) return OCTO_OK;
    Queue& q = queues[I.d.queue];
    for (size_t l = 0; l < q.head_pool.size(); ++l) {
      const size_t rb = q.head_item_bytes[l];
      const bool vec = rb % 16 == 0 && ((uintptr_t)q.head_pool[l] % 16) == 0 && ((uintptr_t)I.head_buffers[l] % 16) == 0;
      const size_t work = (vec ? rb / 16 : rb) * (size_t)n;
      const unsigned grid = (unsigned)std::min<size_t>((work + 255) / 256, 4096);
      if (vec) hipLaunchKernelGGL(gather_rows_kernel<true>, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const unsigned char*)q.head_pool[l],
                                  (unsigned char*)I.head_buffers[l], d_idx, first, n, rb);
      else hipLaunchKernelGGL(gather_rows_kernel<false>, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const unsigned char*)q.head_pool[l],
                              (unsigned char*)I.head_buffers[l], d_idx, first, n, rb);
      if (hipGetLastError() != hipSuccess) return fail(OCTO_EHIP, "gather of planted heads failed to launch");
    }
    return OCTO_OK;
  }

  // results of finished batches of every instance -> statistics
  octo_status poll() {
    for (Instance& I : inst) {
      if (I.inflight == 0) continue;
      int32_t nf = 0, nb = 0;
      const octo_status st = octo_collect(I.d.pipe, fr_buf.data(), (int32_t)fr_buf.size(), bx_buf.data(), (int32_t)bx_buf.size(), &nf, &nb, 0);
      if (st == OCTO_ENOTREADY || nf == 0) continue;
      if (st != OCTO_OK && st != OCTO_ECAP) return fail(st, std::string("collect: ") + octo_last_error(I.d.pipe));
      Queue& q = queues[I.d.queue];
      int done = 0;
      for (int f = 0; f < nf; ++f) {
        const octo_frame_result& r = fr_buf[f];
        ++q.served; q.slo_met += r.slo_met; q.boxes += r.n_boxes;
        q.latency_ms.push_back(r.latency_ms);
        const auto it = std::find(I.batch_last.begin(), I.batch_last.end(), (long long)r.frame_id);
        if (it != I.batch_last.end()) { ++done; I.batch_last.erase(it); }
        if (keep_results) {
          const auto p = q.pool_of.find(r.frame_id);
          q.kept.push_back({(long long)r.frame_id, p == q.pool_of.end() ? -1 : p->second, (int)q.kept_boxes.size(), r.n_boxes});
          if (p != q.pool_of.end()) q.pool_of.erase(p);
          q.kept_boxes.insert(q.kept_boxes.end(), bx_buf.begin() + r.box_offset, bx_buf.begin() + r.box_offset + r.n_boxes);
        }
      }
      I.inflight -= done;
    }
    return OCTO_OK;
  }

  // requests that have arrived by now move from the camera streams into the queue
  void admit(int qi, double now_s) {
    Queue& q = queues[qi];
    size_t ptr = q.next_arrival;
    while (ptr < q.merged.size() && q.merged[ptr].t_s <= now_s) {
      const Arrival& a = q.merged[ptr];
      const Camera& c = cams[a.cam];
      const int k = a.seq % (int)c.frames.size();
      q.waiting.push_back({q.next_id++, c.d.pool_offset + k, c.frames[k], c.pitches[k], t0_ms + 1e3 * a.t_s});
      ++ptr;
    }
    q.submitted += (long long)(ptr - q.next_arrival);
    q.next_arrival = ptr;
  }

  // one batch of an instance: drop what is late, take at most bz requests, launch every model on its stream
  octo_status launch_batch(Instance& I, int* launched) {
    *launched = 0;
    Queue& q = queues[I.d.queue];
    if (drop_late && !q.waiting.empty()) {
      std::vector<double> arr(q.waiting.size());
      for (size_t i = 0; i < arr.size(); ++i) arr[i] = q.waiting[i].arrival_ms;
      int32_t late = 0;
      octo_late_prefix(arr.data(), (int32_t)arr.size(), octo_now_ms(), q.d.slo_ms, &late);
      if (late > 0) { q.waiting.erase(q.waiting.begin(), q.waiting.begin() + late); q.dropped += late; }
    }
    const int n = std::min<int>(q.d.bz, (int)q.waiting.size());
    if (n == 0 || I.inflight >= MAX_IN_FLIGHT) return OCTO_OK;
    std::vector<const void*> fr(n); std::vector<size_t> pitch(n); std::vector<double> arr(n); std::vector<int64_t> ids(n);
    for (int i = 0; i < n; ++i) { const Request& r = q.waiting[i]; fr[i] = r.frame; pitch[i] = r.pitch; arr[i] = r.arrival_ms; ids[i] = r.id; }
    octo_status st = gather_heads(I, q.d_seq, ids[0], n, I.streams[0]);      // ids in a batch are consecutive
    if (st != OCTO_OK) return st;
    if ((st = octo_submit_frames(I.d.pipe, fr.data(), pitch.data(), arr.data(), ids.data(), n)) != OCTO_OK)
      return fail(st, std::string("submit: ") + octo_last_error(I.d.pipe));
    int32_t got = 0;
    if ((st = octo_run_model(I.d.pipe, 0, I.streams[0], &got)) != OCTO_OK) return fail(st, std::string("run: ") + octo_last_error(I.d.pipe));
    if (got != n) return fail(OCTO_ESTATE, "a batch took a different number of frames than were submitted for it");
    for (int m = 1; m < (int)I.streams.size(); ++m)
      if ((st = octo_run_model(I.d.pipe, m, I.streams[m], &got)) != OCTO_OK) return fail(st, std::string("run: ") + octo_last_error(I.d.pipe));
    if (keep_results) for (int i = 0; i < n; ++i) q.pool_of[q.waiting[i].id] = q.waiting[i].pool_index;
    ++I.inflight;
    I.batch_last.push_back(ids[n - 1]);
    q.waiting.erase(q.waiting.begin(), q.waiting.begin() + n);
    *launched = n;
    return OCTO_OK;
  }

  // an instance's slot: up to batches-per-cycle + 1 batches of what is queued
  octo_status fire(Instance& I, double now_s) {
    admit(I.d.queue, now_s);
    const int k = queues[I.d.queue].d.batches_per_cycle + 1;
    for (int b = 0; b < k; ++b) {
      for (int spins = 0; I.inflight >= MAX_IN_FLIGHT && spins < 100000; ++spins) {     // result slots are full: take finished batches first
        const octo_status st = poll();
        if (st != OCTO_OK) return st;
      }
      int n = 0;
      const octo_status st = launch_batch(I, &n);
      if (st != OCTO_OK) return st;
      if (n == 0) break;
    }
    return OCTO_OK;
  }

  void* make_stream(int first, int n) {
    if (!masked) return plain_stream;
    void* h = nullptr;
    if (octo_stream_create_range(first, n, &h) != OCTO_OK) return nullptr;
    owned_streams.push_back(h);
    return h;
  }

  // Algorithm 2 over the scheduled pipelines followed by the active copies.  It visits pipelines in order, so the
  // scheduled ones get the placements they already have and the copies get what is free.  A copy whose first model finds
  // no portion is switched off again; a later model without a portion follows its parent's stream.  A stream the
  // schedule did not use yet gets the compute units after the ones in use (the last ones if the GPU is full), as wide as
  // the widest model placed on it; streams that exist keep their width.
  octo_status place_copies() {
    std::vector<int> copies;
    for (int i = 0; i < (int)inst.size(); ++i) if (inst[i].d.standby && inst[i].active) copies.push_back(i);
    if (copies.empty()) return OCTO_OK;
    const int nb = (int)sched_models.size();
    std::vector<std::vector<octo_sched_model>> models(sched_models);
    for (int ci : copies) models.push_back(sched_models[inst[ci].d.queue]);
    std::vector<octo_sched_pipeline> ps(models.size());
    int total = 0;
    for (size_t i = 0; i < models.size(); ++i) {
      ps[i].models = models[i].data(); ps[i].n_models = (int32_t)models[i].size();
      ps[i].slo_ms = sched_slo[i < (size_t)nb ? i : (size_t)inst[copies[i - nb]].d.queue];
      total += ps[i].n_models;
    }
    std::vector<octo_placement> pl(total);
    const octo_status st = octo_coral_schedule(ps.data(), (int32_t)ps.size(), gpu_mem, 1.0, n_streams, pl.data());
    if (st != OCTO_OK) return fail(st, "Algorithm 2 failed while placing a stand-by copy");
    for (size_t c = 0; c < copies.size(); ++c) {
      Instance& I = inst[copies[c]];
      const std::vector<octo_sched_model>& ms = sched_models[I.d.queue];
      const int nm = (int)ms.size();
      std::vector<const octo_placement*> mine(nm, nullptr);
      for (const octo_placement& p : pl) if (p.pipeline == nb + (int)c && p.model >= 0 && p.model < nm) mine[p.model] = &p;
      if (!mine[0] || mine[0]->stream < 0) { I.active = false; continue; }
      for (int m = 0; m < nm; ++m) {
        const int s = mine[m] ? mine[m]->stream : -1;
        if (s < 0 || stream_handle.count(s)) continue;
        double widest = 0.0;
        for (int q2 = 0; q2 < nm; ++q2) if (mine[q2] && mine[q2]->stream == s) widest = std::max<double>(widest, ms[q2].util);
        int32_t n = CU_GRAIN;
        octo_width_to_cus(widest, total_cus, CU_GRAIN, &n);
        int first = 0;
        for (const auto& kv : stream_cus) first = std::max(first, kv.second.first + kv.second.second);
        if (first + n > total_cus) first = total_cus - n;
        void* h = make_stream(first, n);
        if (!h && masked) return fail(OCTO_EHIP, "could not create a stream for a stand-by copy");
        stream_cus[s] = {first, (int)n};
        stream_handle[s] = h;
      }
      std::vector<void*> handles(nm, nullptr);
      for (int m = 0; m < nm; ++m) {
        const int s = mine[m] ? mine[m]->stream : -1;
        const int parent = ms[m].parent;
        handles[m] = s >= 0 ? stream_handle[s] : (parent >= 0 && parent < m ? handles[parent] : I.streams[0]);
      }
      I.streams = handles;
      I.slot_ms = mine[0]->start_ms;
    }
    return OCTO_OK;
  }

  // once per duty cycle: tell every queue's scaler what arrived and what is queued, and act on its decision
  octo_status autoscale(double now_s) {
    std::vector<int> ups, downs;
    for (int qi = 0; qi < (int)queues.size(); ++qi) {
      Queue& q = queues[qi];
      if (!q.scaler) continue;
      admit(qi, now_s);
      const long long arrived = (long long)(q.next_arrival - q.arrival_mark);
      q.arrival_mark = q.next_arrival;
      Instance& S = inst[q.standby];
      int32_t d = 0;
      octo_scaler_observe(q.scaler, arrived, (long long)q.waiting.size(), S.active ? 2 : 1, &d);
      if (d > 0 && !S.active) { S.active = true; ups.push_back(qi); }
      else if (d < 0 && S.active) { S.active = false; downs.push_back(qi); }
    }
    if (ups.empty() && downs.empty()) return OCTO_OK;
    const octo_status st = place_copies();      // the copies that stay may move into what a removed one has freed
    if (st != OCTO_OK) return st;
    for (int qi : downs) events.push_back({(float)now_s, qi, -1});
    for (int qi : ups) events.push_back({(float)now_s, qi, inst[queues[qi].standby].active ? 1 : 0});
    return OCTO_OK;
  }

  bool all_done() const {
    for (const Queue& q : queues) if (q.next_arrival != q.merged.size() || !q.waiting.empty()) return false;
    for (const Instance& I : inst) if (I.inflight) return false;
    return true;
  }
};

extern "C" {

octo_status octo_executor_create(const octo_exec_desc* d, octo_executor** out) {
  if (!d || !out || d->n_queues < 1 || d->n_instances < 1 || d->n_cameras < 0 || !d->queues || !d->instances || (d->n_cameras && !d->cameras) ||
      !(d->duty_ms > 0.f))
    return OCTO_EINVAL;
  octo_executor* ex = new (std::nothrow) octo_executor();
  if (!ex) return OCTO_ENOMEM;
  auto bad = [&](octo_status s) { delete ex; return s; };
  ex->duty_ms = d->duty_ms;
  ex->slotted = d->slotted != 0; ex->drop_late = d->drop_late != 0; ex->keep_results = d->keep_results != 0; ex->masked = d->masked != 0;
  ex->plain_stream = d->plain_stream;
  int32_t ncu = 0;
  if (octo_device_cu_count(&ncu) != OCTO_OK) return bad(OCTO_EHIP);
  ex->total_cus = ncu;
  ex->queues.resize(d->n_queues);
  for (int i = 0; i < d->n_queues; ++i) {
    Queue& q = ex->queues[i];
    q.d = d->queues[i];
    if (q.d.bz < 1 || q.d.batches_per_cycle < 1 || q.d.n_levels < 0 || q.d.n_levels > OCTO_MAX_LEVELS) return bad(OCTO_EINVAL);
    for (int l = 0; l < q.d.n_levels; ++l) {
      if (!q.d.head_pool || !q.d.head_item_bytes || !q.d.head_pool[l] || !q.d.head_item_bytes[l]) return bad(OCTO_EINVAL);
      q.head_pool.push_back(q.d.head_pool[l]); q.head_item_bytes.push_back(q.d.head_item_bytes[l]);
    }
    q.d.head_pool = nullptr; q.d.head_item_bytes = nullptr;
  }
  size_t frame_cap = 1, box_cap = 1;
  ex->inst.resize(d->n_instances);
  for (int i = 0; i < d->n_instances; ++i) {
    Instance& I = ex->inst[i];
    I.d = d->instances[i];
    if (!I.d.pipe || I.d.queue < 0 || I.d.queue >= d->n_queues || I.d.n_models < 1 || !I.d.streams) return bad(OCTO_EINVAL);
    I.streams.assign(I.d.streams, I.d.streams + I.d.n_models);
    Queue& q = ex->queues[I.d.queue];
    if (I.d.head_buffers) {
      if (q.head_pool.empty()) return bad(OCTO_EINVAL);
      I.head_buffers.assign(I.d.head_buffers, I.d.head_buffers + q.head_pool.size());
    } else if (!q.head_pool.empty()) {
      return bad(OCTO_EINVAL);
    }
    I.d.streams = nullptr; I.d.head_buffers = nullptr;
    I.slot_ms = I.d.slot_ms;
    I.active = !I.d.standby;
    if (I.d.standby) {
      if (q.standby >= 0 || !ex->slotted) return bad(OCTO_EINVAL);       // one copy per queue; only the slotted mode scales
      q.standby = i;
    }
    if (I.d.max_frames < 1 || I.d.max_batch < 1 || I.d.max_det < 1) return bad(OCTO_EINVAL);
    frame_cap = std::max<size_t>(frame_cap, 4 * (size_t)I.d.max_frames);
    box_cap = std::max<size_t>(box_cap, 4 * (size_t)I.d.max_frames * (size_t)I.d.max_det);
    if (octo_set_batch_size(I.d.pipe, 0, std::min(q.d.bz, I.d.max_batch)) != OCTO_OK) return bad(OCTO_EINVAL);
  }
  ex->fr_buf.resize(frame_cap); ex->bx_buf.resize(box_cap);
  for (Queue& q : ex->queues)
    if (q.standby >= 0) {
      const double cap = (double)(q.d.batches_per_cycle + 1) * q.d.bz;
      if (octo_scaler_create(cap, q.d.scaler_window > 0 ? q.d.scaler_window : 5, q.d.scaler_up > 0 ? q.d.scaler_up : 1.0,
                             q.d.scaler_down > 0 ? q.d.scaler_down : 0.75, 2, &q.scaler) != OCTO_OK) return bad(OCTO_EINVAL);
    }
  ex->cams.resize(d->n_cameras);
  for (int i = 0; i < d->n_cameras; ++i) {
    Camera& c = ex->cams[i];
    c.d = d->cameras[i];
    if (c.d.queue < 0 || c.d.queue >= d->n_queues || c.d.n_arrivals < 0 || c.d.n_frames < 1 || !c.d.d_frames || !c.d.pitch_bytes ||
        (c.d.n_arrivals && !c.d.arrivals_s)) return bad(OCTO_EINVAL);
    c.arrivals.assign(c.d.arrivals_s, c.d.arrivals_s + c.d.n_arrivals);
    c.frames.assign(c.d.d_frames, c.d.d_frames + c.d.n_frames);
    c.pitches.assign(c.d.pitch_bytes, c.d.pitch_bytes + c.d.n_frames);
    c.d.arrivals_s = nullptr; c.d.d_frames = nullptr; c.d.pitch_bytes = nullptr;
  }
  // scheduler inputs for re-placement (only needed with stand-by copies)
  if (d->sched) {
    for (int i = 0; i < d->n_queues; ++i) {
      if (!d->sched[i].models || d->sched[i].n_models < 1) return bad(OCTO_EINVAL);
      ex->sched_models.emplace_back(d->sched[i].models, d->sched[i].models + d->sched[i].n_models);
      ex->sched_slo.push_back(d->sched[i].slo_ms);
    }
    ex->gpu_mem = d->gpu_mem; ex->n_streams = d->n_streams;
  }
  for (int i = 0; i < d->n_sched_streams; ++i) {
    if (!d->stream_index || !d->stream_handle || !d->stream_first_cu || !d->stream_n_cu) return bad(OCTO_EINVAL);
    ex->stream_handle[d->stream_index[i]] = d->stream_handle[i];
    ex->stream_cus[d->stream_index[i]] = {d->stream_first_cu[i], d->stream_n_cu[i]};
  }
  for (const Queue& q : ex->queues) if (q.standby >= 0 && ex->sched_models.empty()) return bad(OCTO_EINVAL);
  // one frame through every instance on the streams it will use, so that the first served batch does not pay for
  // stream and code-object set-up
  for (Instance& I : ex->inst) {
    const Camera* cam = nullptr;
    for (const Camera& c : ex->cams) if (c.d.queue == I.d.queue) { cam = &c; break; }
    if (!cam) continue;
    long long* d_one = nullptr;
    if (!I.head_buffers.empty()) {
      const long long idx = cam->d.pool_offset;
      if (hipMalloc((void**)&d_one, sizeof idx) != hipSuccess || hipMemcpy(d_one, &idx, sizeof idx, hipMemcpyHostToDevice) != hipSuccess) return bad(OCTO_EHIP);
      if (ex->gather_heads(I, d_one, 0, 1, I.streams[0]) != OCTO_OK) { (void)hipFree(d_one); return bad(OCTO_EHIP); }
    }
    const void* f = cam->frames[0]; const size_t pitch = cam->pitches[0]; const int64_t id = -1;
    octo_status st = octo_submit_frames(I.d.pipe, &f, &pitch, nullptr, &id, 1);
    int32_t got = 0;
    for (int m = 0; st == OCTO_OK && m < (int)I.streams.size(); ++m) st = octo_run_model(I.d.pipe, m, I.streams[m], &got);
    int32_t nf = 0, nb = 0;
    if (st == OCTO_OK) st = octo_collect(I.d.pipe, ex->fr_buf.data(), (int32_t)ex->fr_buf.size(), ex->bx_buf.data(), (int32_t)ex->bx_buf.size(), &nf, &nb, 1);
    if (d_one) { (void)hipDeviceSynchronize(); (void)hipFree(d_one); }
    if (st != OCTO_OK && st != OCTO_ECAP) return bad(st);
  }
  *out = ex;
  return OCTO_OK;
}

octo_status octo_executor_serve(octo_executor* ex, double duration_s, double drain_s, double* wall_s) {
  if (!ex || !(duration_s >= 0.0) || !(drain_s >= 0.0)) return OCTO_EINVAL;
  // arrivals of every queue's cameras, merged by time; request ids are handed out in arrival order, so the pool index
  // of every request is known now: one upload per queue
  for (size_t qi = 0; qi < ex->queues.size(); ++qi) {
    Queue& q = ex->queues[qi];
    q.merged.clear();
    for (size_t ci = 0; ci < ex->cams.size(); ++ci) {
      const Camera& c = ex->cams[ci];
      if (c.d.queue != (int)qi) continue;
      for (size_t k = 0; k < c.arrivals.size(); ++k) if (c.arrivals[k] < duration_s) q.merged.push_back({c.arrivals[k], (int)ci, (int)k});
    }
    std::stable_sort(q.merged.begin(), q.merged.end(), [](const Arrival& a, const Arrival& b) {
      return a.t_s != b.t_s ? a.t_s < b.t_s : (a.cam != b.cam ? a.cam < b.cam : a.seq < b.seq); });
    q.next_arrival = q.arrival_mark = 0; q.next_id = 0; q.waiting.clear(); q.pool_of.clear();
    if (q.d_seq) { (void)hipFree(q.d_seq); q.d_seq = nullptr; }
    if (!q.head_pool.empty()) {
      std::vector<long long> seq(std::max<size_t>(1, q.merged.size()), 0);
      for (size_t i = 0; i < q.merged.size(); ++i) {
        const Camera& c = ex->cams[q.merged[i].cam];
        seq[i] = c.d.pool_offset + q.merged[i].seq % (int)c.frames.size();
      }
      if (hipMalloc((void**)&q.d_seq, seq.size() * sizeof(long long)) != hipSuccess ||
          hipMemcpy(q.d_seq, seq.data(), seq.size() * sizeof(long long), hipMemcpyHostToDevice) != hipSuccess)
        return ex->fail(OCTO_EHIP, "upload of the planted-head index table failed");
    }
  }
  const double duty = ex->duty_ms;
  ex->t0_ms = octo_now_ms() + 2.0;
  const double t_end_ms = ex->t0_ms + 1e3 * (duration_s + drain_s);
  auto nap = [] { std::this_thread::sleep_for(std::chrono::microseconds(200)); };
  auto now_s = [&] { return (octo_now_ms() - ex->t0_ms) / 1e3; };
  octo_status st = OCTO_OK;
  bool scaling = false;
  for (const Queue& q : ex->queues) scaling |= q.scaler != nullptr;
  if (ex->slotted) {
    for (long long c = 0;; ) {
      std::vector<std::pair<float, int>> order;
      for (int k = 0; k < (int)ex->inst.size(); ++k) if (ex->inst[k].active) order.push_back({ex->inst[k].slot_ms, k});
      std::sort(order.begin(), order.end());
      for (const auto& o : order) {
        const double target = ex->t0_ms + (double)c * duty + o.first;
        while (octo_now_ms() < target) { if ((st = ex->poll()) != OCTO_OK) return st; nap(); }
        if ((st = ex->fire(ex->inst[o.second], now_s())) != OCTO_OK) return st;
      }
      ++c;
      if (scaling) {
        while (octo_now_ms() < ex->t0_ms + (double)c * duty) { if ((st = ex->poll()) != OCTO_OK) return st; nap(); }     // decisions are taken on whole cycles
        if ((st = ex->autoscale(now_s())) != OCTO_OK) return st;
      }
      if ((ex->all_done() && (double)c * duty >= 1e3 * duration_s) || octo_now_ms() > t_end_ms) break;
    }
  } else {
    for (;;) {
      for (Instance& I : ex->inst) {
        ex->admit(I.d.queue, now_s());
        int n = 0;
        if ((st = ex->launch_batch(I, &n)) != OCTO_OK) return st;
      }
      if ((st = ex->poll()) != OCTO_OK) return st;
      nap();
      if ((ex->all_done() && octo_now_ms() - ex->t0_ms >= 1e3 * duration_s) || octo_now_ms() > t_end_ms) break;
    }
  }
  if (wall_s) *wall_s = now_s();
  for (int i = 0; i < 1000; ++i) {
    bool busy = false;
    for (const Instance& I : ex->inst) busy |= I.inflight != 0;
    if (!busy) break;
    if ((st = ex->poll()) != OCTO_OK) return st;
    std::this_thread::sleep_for(std::chrono::milliseconds(1));
  }
  return OCTO_OK;
}

octo_status octo_executor_stats(const octo_executor* ex, int32_t queue, octo_exec_stats* out) {
  if (!ex || !out || queue < 0 || queue >= (int)ex->queues.size()) return OCTO_EINVAL;
  const Queue& q = ex->queues[queue];
  *out = octo_exec_stats{};
  out->submitted = q.submitted; out->served = q.served; out->slo_met = q.slo_met; out->boxes = q.boxes; out->dropped = q.dropped;
  if (!q.latency_ms.empty()) {
    std::vector<float> v(q.latency_ms);
    std::sort(v.begin(), v.end());
    auto pct = [&](double p) {       // linear interpolation between order statistics
      const double pos = p / 100.0 * (double)(v.size() - 1);
      const size_t lo = (size_t)std::floor(pos), hi = std::min(v.size() - 1, lo + 1);
      return (float)(v[lo] + (pos - (double)lo) * (v[hi] - v[lo]));
    };
    out->latency_ms_p50 = pct(50.0); out->latency_ms_p99 = pct(99.0); out->latency_ms_max = v.back();
  }
  return OCTO_OK;
}

octo_status octo_executor_scale_events(const octo_executor* ex, octo_scale_event* out, int32_t cap, int32_t* n) {
  if (!ex || !n || cap < 0 || (cap > 0 && !out)) return OCTO_EINVAL;
  *n = (int32_t)ex->events.size();
  for (int i = 0; i < std::min<int>(cap, *n); ++i) out[i] = ex->events[i];
  return *n > cap ? OCTO_ECAP : OCTO_OK;
}

octo_status octo_executor_streams(const octo_executor* ex, int32_t* stream_index, int32_t* first_cu, int32_t* n_cu, int32_t cap, int32_t* n) {
  if (!ex || !n || cap < 0 || (cap > 0 && (!stream_index || !first_cu || !n_cu))) return OCTO_EINVAL;
  *n = (int32_t)ex->stream_cus.size();
  int i = 0;
  for (const auto& kv : ex->stream_cus) {
    if (i >= cap) break;
    stream_index[i] = kv.first; first_cu[i] = kv.second.first; n_cu[i] = kv.second.second; ++i;
  }
  return *n > cap ? OCTO_ECAP : OCTO_OK;
}

octo_status octo_executor_results(const octo_executor* ex, int32_t queue, int64_t* frame_ids, int32_t* pool_index, int32_t* box_offset,
                                  int32_t* n_boxes, int32_t frame_cap, octo_box* boxes, int32_t box_cap, int32_t* n_frames, int32_t* n_boxes_total) {
  if (!ex || queue < 0 || queue >= (int)ex->queues.size() || !n_frames || !n_boxes_total || frame_cap < 0 || box_cap < 0) return OCTO_EINVAL;
  const Queue& q = ex->queues[queue];
  *n_frames = (int32_t)q.kept.size(); *n_boxes_total = (int32_t)q.kept_boxes.size();
  if (*n_frames > frame_cap || *n_boxes_total > box_cap) return OCTO_ECAP;
  if ((*n_frames && (!frame_ids || !pool_index || !box_offset || !n_boxes)) || (*n_boxes_total && !boxes)) return OCTO_EINVAL;
  for (int i = 0; i < *n_frames; ++i) {
    frame_ids[i] = q.kept[i].id; pool_index[i] = q.kept[i].pool_index; box_offset[i] = q.kept[i].box_begin; n_boxes[i] = q.kept[i].n_boxes;
  }
  if (*n_boxes_total) memcpy(boxes, q.kept_boxes.data(), q.kept_boxes.size() * sizeof(octo_box));
  return OCTO_OK;
}

const char* octo_executor_last_error(const octo_executor* ex) { return ex ? ex->err.c_str() : ""; }

octo_status octo_executor_destroy(octo_executor* ex) {
  if (!ex) return OCTO_EINVAL;
  (void)hipDeviceSynchronize();
  for (void* h : ex->owned_streams) (void)octo_stream_destroy(h);
  for (Queue& q : ex->queues) {
    if (q.d_seq) (void)hipFree(q.d_seq);
    if (q.scaler) (void)octo_scaler_destroy(q.scaler);
  }
  delete ex;
  return OCTO_OK;
}

}  // extern "C"
