// Host side of libocto: pipeline construction (workspace planning, weight
// packing), the frame queue, batch formation, the launch sequence of one
// cascade pass, result collection, and the profiling / parity hooks.
// No device code lives here.
#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <string>
#include <vector>

#include "octo_internal.h"

using namespace octo;

namespace {

thread_local std::string g_create_error;

struct Arena {
  char* base = nullptr;   // nullptr: sizing pass
  size_t off = 0, cap = 0;
  bool failed = false;
  void* alloc(size_t bytes) {
    off = (off + 255) & ~(size_t)255;
    size_t at = off;
    off += bytes;
    if (base && off > cap) { failed = true; return nullptr; }
    return base ? base + at : (void*)(uintptr_t)(at + 256);   // non-null placeholder while sizing
  }
};

struct LayerPlan {
  octo_layer L{};
  int cin = 0;
  void* d_weight = nullptr;
  float* d_bias = nullptr;
  int K = 0, Kp = 0, cout_pad = 0;
  std::vector<int> copy_inputs;   // concat: inputs that could not be aliased into the output buffer
  double flops = 0, bytes = 0;    // per item
  double input_bytes = 0;         // conv: the part of `bytes` that is the input tensor
  double weight_bytes = 0;        // per launch
  int kernel_id = KID_NONE;       // which kernel the last launch of this layer used
  // First layer on a 3-channel input: run on the pixel-pair view of the 4-channel-padded input (two neighbouring
  // pixels = one 16-byte vector of 8 values), i.e. as a conv with 8 input channels, kernel width pair_kw, horizontal
  // stride 1 and horizontal padding pair_pad, on an image of half the width.
  bool pair_view = false;
  int pair_kw = 0, pair_pad = 0, pair_shift = 0;
  // The next layer is a 3x3 / stride-2 / pad-1 max-pool and the only reader of this first layer's output: the
  // convolution kernel pools its own tile and writes the pooled tensor, the pool layer does nothing (its kernel id
  // then reads KID_NONE).  Cleared for good the first time no kernel accepts the fused form.
  bool fuse_pool = false;
  // The next layer is a 1x1 convolution of the same input with the same activation (the two entry convolutions of a
  // cross-stage block): one launch computes both - the weight matrices stacked, the second layer's channels written to
  // its own tensor - so the input is read once.  The next layer then does nothing (kernel id KID_NONE).  Cleared for
  // good the first time the kernel refuses the fused form.
  bool fuse_twin = false;
  void* d_weight_twin = nullptr;
  float* d_bias_twin = nullptr;
  int twin_cout_pad = 0;
};

struct TensorPlan {
  int h = 0, w = 0, c = 0;
  bool f32 = false;        // fc output
  int root = -1;           // tensor whose buffer this one lives in (itself if not aliased)
  int coff = 0;
  int ld = 0;
  size_t root_off = 0;     // offset of the root buffer inside the activation region
  void* ptr = nullptr;     // root buffer base
};

struct ModelPlan {
  octo_model_desc d{};
  std::string name;
  std::vector<LayerPlan> layers;
  std::vector<TensorPlan> tensors;
  bool input_c4 = false;   // tensor 0 is stored with a zero fourth channel
  int cap = 0;             // item capacity
  int bz = 0;              // current batch size (root: frames per batch)
  int exec_bz = 0;         // root only: frames per execution of the detector's layers (0: the whole batch at once)
  const int* n_dyn = nullptr;
  double items_hint = 0;   // smoothed item count of recent batches (children; 0: none seen yet)
  char* act_base = nullptr;
  size_t act_bytes = 0;
  // detector
  int gh[OCTO_MAX_LEVELS]{}, gw[OCTO_MAX_LEVELS]{};
  int n_cand = 0, k_cap = 0;
  octo_cand* cand = nullptr; int* cand_count = nullptr;
  octo_cand* top = nullptr; int* top_count = nullptr;
  unsigned long long* mask = nullptr;
  int* keep = nullptr; int* n_keep = nullptr; int* flags = nullptr;
  const void* head_override[OCTO_MAX_LEVELS]{};
  // classifier
  int* labels = nullptr;   // also used by detector children (label = number of kept boxes)
  int n_logits = 0;
};

struct Batch {
  int n = 0;
  int slot = 0;
  std::vector<int64_t> ids;
  std::vector<double> arrival;
  double t_launch = 0;
  hipEvent_t done = nullptr;
  bool finalized = false;
  std::vector<hipEvent_t> stage_ev;
  std::vector<std::vector<hipEvent_t>> layer_ev;   // per model: one event before the first layer and one after each
  std::vector<bool> model_ran;
};

struct QueuedFrame { const void* ptr; size_t pitch; double arrival; int64_t id; };

constexpr int RING = 8;
constexpr int CNT_STRIDE = 32;   // candidate counters sit 128 bytes apart: same-line atomics serialise in L2

}  // namespace

struct octo_pipeline {
  octo_pipeline_desc d{};
  std::vector<ModelPlan> models;
  std::vector<octo_edge> edges;
  std::vector<int> edge_of_model;   // -1: root or detached
  int num_cu = 256;
  int max_frames = 0, max_queue = 0;
  // per edge
  octo_roi* rois[OCTO_MAX_EDGES]{}; int* n_roi[OCTO_MAX_EDGES]{}; int roi_cap[OCTO_MAX_EDGES]{}; int* roi_of[OCTO_MAX_EDGES]{};
  int* roi_cnt[OCTO_MAX_EDGES]{};
  // result block (device) and its pinned host mirrors
  char* d_result = nullptr; size_t result_bytes = 0;
  size_t off_nkeep = 0, off_flags = 0, off_nroi = 0, off_boxes = 0;
  char* h_result[RING]{};
  // frame pointer tables
  const uint8_t** d_frames[RING]{}; size_t* d_pitch[RING]{};
  char* h_tables[RING]{};
  // geometry
  int nw = 0, nh = 0, left = 0, top = 0;
  std::deque<QueuedFrame> queue;
  std::deque<Batch> inflight;
  std::vector<hipEvent_t> event_pool;
  int next_slot = 0;
  bool stage_timing = false, layer_timing = false;
  std::vector<float> last_stage_ms;
  std::vector<std::vector<float>> last_layer_ms;
  hipEvent_t ev_det = nullptr;
  std::vector<hipEvent_t> ev_child;
  std::string err;
};

namespace {

octo_status fail(octo_pipeline* p, octo_status st, const char* fmt, ...) {
  char buf[512];
  va_list ap; va_start(ap, fmt); vsnprintf(buf, sizeof buf, fmt, ap); va_end(ap);
  if (p) p->err = buf; else g_create_error = buf;
  return st;
}

#define HIPCHK(p, call)                                                                     \
  do { hipError_t e_ = (call);                                                              \
       if (e_ != hipSuccess) return fail(p, OCTO_EHIP, "%s failed: %s", #call, hipGetErrorString(e_)); } while (0)

bool valid_dtype(int dt) { return dt == OCTO_F32 || dt == OCTO_F16 || dt == OCTO_BF16; }

// ---- shape inference and validation ----------------------------------------
octo_status plan_shapes(ModelPlan& m, std::string& why) {
  const octo_model_desc& d = m.d;
  if (!valid_dtype(d.dtype) || d.in_h <= 0 || d.in_w <= 0 || d.in_c <= 0 || d.n_layers <= 0 || !d.layers) { why = "bad model header"; return OCTO_EINVAL; }
  m.tensors.assign(d.n_layers + 1, TensorPlan());
  m.tensors[0].h = d.in_h; m.tensors[0].w = d.in_w; m.tensors[0].c = d.in_c;
  m.layers.resize(d.n_layers);
  for (int i = 0; i < d.n_layers; ++i) {
    LayerPlan& lp = m.layers[i];
    lp.L = d.layers[i];
    const octo_layer& L = lp.L;
    if (L.n_in < 1 || L.n_in > OCTO_MAX_LAYER_INPUTS) { why = "layer input count"; return OCTO_EINVAL; }
    for (int k = 0; k < L.n_in; ++k) if (L.in[k] < 0 || L.in[k] > i) { why = "layer input id"; return OCTO_EINVAL; }
    const TensorPlan& x = m.tensors[L.in[0]];
    TensorPlan& y = m.tensors[i + 1];
    if (x.f32) { why = "fp32 logits cannot feed a layer"; return OCTO_EINVAL; }
    switch (L.op) {
      case OCTO_CONV: case OCTO_FC: {
        const int kh = L.op == OCTO_FC ? 1 : L.kh, kw = L.op == OCTO_FC ? 1 : L.kw;
        const int st = L.op == OCTO_FC ? 1 : L.stride, pad = L.op == OCTO_FC ? 0 : L.pad;
        if (L.cout <= 0 || kh <= 0 || kw <= 0 || st <= 0 || pad < 0 || !L.weight || !L.bias) { why = "conv parameters"; return OCTO_EINVAL; }
        if (L.op == OCTO_FC && (x.h != 1 || x.w != 1)) { why = "fc needs a 1x1 map"; return OCTO_EINVAL; }
        y.h = (x.h + 2 * pad - kh) / st + 1; y.w = (x.w + 2 * pad - kw) / st + 1; y.c = L.cout;
        if (y.h <= 0 || y.w <= 0) { why = "conv output empty"; return OCTO_EINVAL; }
        y.f32 = L.op == OCTO_FC;
        lp.cin = x.c;
        lp.L.kh = kh; lp.L.kw = kw; lp.L.stride = st; lp.L.pad = pad;
        if (L.n_in == 2) {
          const TensorPlan& r = m.tensors[L.in[1]];
          if (r.h != y.h || r.w != y.w || r.c != y.c || L.res_mode == OCTO_RES_NONE || r.f32) { why = "residual shape"; return OCTO_EINVAL; }
        } else if (L.n_in != 1 || L.res_mode != OCTO_RES_NONE) { why = "conv inputs"; return OCTO_EINVAL; }
        lp.flops = 2.0 * y.h * y.w * L.cout * x.c * kh * kw;
        const int es = dtype_size(d.dtype);
        lp.bytes = (double)es * x.h * x.w * x.c + (double)(y.f32 ? 4 : es) * y.h * y.w * y.c +
                   (L.n_in == 2 ? (double)es * y.h * y.w * y.c : 0.0);
        lp.weight_bytes = (double)es * L.cout * kh * kw * x.c + 4.0 * L.cout;
        lp.input_bytes = (double)es * x.h * x.w * x.c;
        break;
      }
      case OCTO_MAXPOOL:
        if (L.kh <= 0 || L.kh != L.kw || L.stride <= 0 || L.pad < 0 || L.pad >= L.kh) { why = "maxpool parameters"; return OCTO_EINVAL; }
        y.h = (x.h + 2 * L.pad - L.kh) / L.stride + 1; y.w = (x.w + 2 * L.pad - L.kw) / L.stride + 1; y.c = x.c;
        if (y.h <= 0 || y.w <= 0) { why = "maxpool output empty"; return OCTO_EINVAL; }
        lp.bytes = (double)dtype_size(d.dtype) * ((double)x.h * x.w * x.c + (double)y.h * y.w * y.c);
        break;
      case OCTO_UPSAMPLE2X:
        y.h = 2 * x.h; y.w = 2 * x.w; y.c = x.c;
        lp.bytes = (double)dtype_size(d.dtype) * 5.0 * x.h * x.w * x.c;
        break;
      case OCTO_CONCAT: {
        int c = 0;
        for (int k = 0; k < L.n_in; ++k) {
          const TensorPlan& t = m.tensors[L.in[k]];
          if (t.h != x.h || t.w != x.w || t.f32) { why = "concat shapes"; return OCTO_EINVAL; }
          c += t.c;
        }
        y.h = x.h; y.w = x.w; y.c = c;
        break;
      }
      case OCTO_ADD: {
        if (L.n_in != 2) { why = "add inputs"; return OCTO_EINVAL; }
        const TensorPlan& b = m.tensors[L.in[1]];
        if (b.h != x.h || b.w != x.w || b.c != x.c || b.f32) { why = "add shapes"; return OCTO_EINVAL; }
        y.h = x.h; y.w = x.w; y.c = x.c;
        lp.bytes = (double)dtype_size(d.dtype) * 3.0 * x.h * x.w * x.c;
        break;
      }
      case OCTO_GAP:
        y.h = 1; y.w = 1; y.c = x.c;
        lp.bytes = (double)dtype_size(d.dtype) * ((double)x.h * x.w * x.c + x.c);
        break;
      default: why = "unknown op"; return OCTO_EINVAL;
    }
  }
  if (d.n_outputs < 1 || d.n_outputs > OCTO_MAX_LEVELS) { why = "output count"; return OCTO_EINVAL; }
  for (int k = 0; k < d.n_outputs; ++k) if (d.outputs[k] < 1 || d.outputs[k] > d.n_layers) { why = "output id"; return OCTO_EINVAL; }
  if (d.kind == OCTO_DETECTOR) {
    if (d.n_anchors < 1 || d.n_anchors > OCTO_MAX_ANCHORS || d.n_classes < 1 || d.n_classes > 128 || d.topk < 1 || d.max_det < 1 ||
        !(d.iou_thr >= 0) || !(d.score_thr >= 0)) { why = "detector parameters"; return OCTO_EINVAL; }
    m.n_cand = 0;
    for (int l = 0; l < d.n_outputs; ++l) {
      const TensorPlan& t = m.tensors[d.outputs[l]];
      if (t.c != d.n_anchors * (5 + d.n_classes) || t.f32 || d.stride[l] <= 0) { why = "head tensor shape"; return OCTO_EINVAL; }
      m.gh[l] = t.h; m.gw[l] = t.w;
      m.n_cand += t.h * t.w * d.n_anchors;
    }
    const int k = std::min(d.topk, m.n_cand);
    m.k_cap = (k + 63) / 64 * 64;
    if (m.k_cap > 4096 || (m.n_cand > 4096 && d.topk > 2048)) { why = "topk too large (<= 2048, or <= 4096 when there are at most 4096 candidates)"; return OCTO_EINVAL; }
  } else if (d.kind == OCTO_CLASSIFIER) {
    const TensorPlan& t = m.tensors[d.outputs[0]];
    if (!t.f32 || d.n_outputs != 1) { why = "classifier output must be an fc layer"; return OCTO_EINVAL; }
    m.n_logits = t.c;
  } else { why = "model kind"; return OCTO_EINVAL; }
  return OCTO_OK;
}

// ---- activation memory: concat aliasing + liveness-based reuse --------------
void plan_activations(ModelPlan& m, bool keep_all, bool allow_fusion) {
  const int nt = (int)m.tensors.size();
  for (int t = 0; t < nt; ++t) { m.tensors[t].root = t; m.tensors[t].coff = 0; m.tensors[t].ld = m.tensors[t].c; }
  // producers of these ops can write into a channel slice of a wider buffer
  auto sliceable = [&](int t) {
    if (t == 0) return false;
    const int op = m.layers[t - 1].L.op;
    return op == OCTO_CONV || op == OCTO_MAXPOOL || op == OCTO_UPSAMPLE2X || op == OCTO_ADD;
  };
  std::vector<bool> is_output(nt, false);
  for (int k = 0; k < m.d.n_outputs; ++k) is_output[m.d.outputs[k]] = true;
  for (int i = 0; i < (int)m.layers.size(); ++i) {
    LayerPlan& lp = m.layers[i];
    if (lp.L.op != OCTO_CONCAT) continue;
    int off = 0;
    for (int k = 0; k < lp.L.n_in; ++k) {
      const int t = lp.L.in[k];
      bool dup = false;
      for (int q = 0; q < k; ++q) dup |= lp.L.in[q] == t;
      if (sliceable(t) && m.tensors[t].root == t && !is_output[t] && !dup) {
        // a concat output that was itself aliased elsewhere keeps its own buffer; members must be plain
        bool has_members = false;
        for (int q = 0; q < nt; ++q) has_members |= (q != t && m.tensors[q].root == t);
        if (!has_members) { m.tensors[t].root = i + 1; m.tensors[t].coff = off; }
        else lp.copy_inputs.push_back(k);
      } else {
        lp.copy_inputs.push_back(k);
      }
      off += m.tensors[t].c;
    }
  }
  for (int t = 0; t < nt; ++t) m.tensors[t].ld = m.tensors[m.tensors[t].root].c;
  // own buffers whose channel count is not a multiple of 8 (detector heads) get a padded pitch so that rows stay
  // 16-byte aligned; the pad elements are never written or read
  for (int t = 1; t < nt; ++t)
    if (m.tensors[t].root == t && !m.tensors[t].f32 && (m.tensors[t].c & 7)) {
      bool has_members = false;
      for (int q = 0; q < nt; ++q) has_members |= (q != t && m.tensors[q].root == t);
      if (!has_members) m.tensors[t].ld = (m.tensors[t].c + 7) & ~7;
    }
  // 3-channel input read only by stride-2 convolutions: store it with 4 channels and use the pixel-pair view
  m.input_c4 = m.d.in_c == 3 && (m.d.in_w % 2) == 0 && !is_output[0] && m.tensors[0].root == 0;
  for (int i = 0; i < (int)m.layers.size() && m.input_c4; ++i)
    for (int k = 0; k < m.layers[i].L.n_in; ++k)
      if (m.layers[i].L.in[k] == 0 && !(m.layers[i].L.op == OCTO_CONV && k == 0 && m.layers[i].L.stride == 2)) m.input_c4 = false;
  if (m.input_c4) {
    m.tensors[0].ld = 4;
    for (LayerPlan& lp : m.layers)
      if (lp.L.op == OCTO_CONV && lp.L.in[0] == 0) {
        lp.pair_view = true;
        lp.pair_shift = lp.L.pad & 1;                       // makes the leftmost tap column even
        lp.pair_kw = (lp.L.kw + lp.pair_shift + 1) / 2;
        lp.pair_pad = (lp.L.pad + lp.pair_shift) / 2;
      }
  }
  // first layer followed by a 3x3 / stride-2 / pad-1 max-pool that is the only reader of its output: fused
  for (int i = 0; i + 1 < (int)m.layers.size(); ++i) {
    LayerPlan& lp = m.layers[i];
    const octo_layer& P = m.layers[i + 1].L;
    lp.fuse_pool = false;
    if (!allow_fusion || !lp.pair_view || lp.L.op != OCTO_CONV || lp.L.n_in != 1 || is_output[i + 1] || m.tensors[i + 1].root != i + 1) continue;
    if (P.op != OCTO_MAXPOOL || P.in[0] != i + 1 || P.kh != 3 || P.stride != 2 || P.pad != 1) continue;
    int readers = 0;
    for (const LayerPlan& q : m.layers)
      for (int k = 0; k < q.L.n_in; ++k) readers += q.L.in[k] == i + 1;
    lp.fuse_pool = readers == 1;
  }
  // two 1x1 convolutions in a row that read the same tensor: one launch (16-bit types; channel counts and output
  // views in whole 16-byte vectors; no residual, not the first layer, no fp32 output)
  for (int i = 0; i < (int)m.layers.size(); ++i) m.layers[i].fuse_twin = false;
  for (int i = 0; i + 1 < (int)m.layers.size(); ++i) {
    LayerPlan& a = m.layers[i];
    const LayerPlan& b = m.layers[i + 1];
    if (!allow_fusion || dtype_size(m.d.dtype) != 2 || a.fuse_pool || (i > 0 && m.layers[i - 1].fuse_twin)) continue;
    if (a.L.op != OCTO_CONV || b.L.op != OCTO_CONV || a.L.n_in != 1 || b.L.n_in != 1 || a.L.in[0] != b.L.in[0] || a.pair_view || b.pair_view) continue;
    if (a.L.kh != 1 || a.L.kw != 1 || b.L.kh != 1 || b.L.kw != 1 || a.L.stride != 1 || b.L.stride != 1 || a.L.pad != 0 || b.L.pad != 0 || a.L.act != b.L.act) continue;
    const TensorPlan &ta = m.tensors[i + 1], &tb = m.tensors[i + 2];
    if (ta.f32 || tb.f32 || ((a.L.cout | b.L.cout | ta.ld | ta.coff | tb.ld | tb.coff) & 7)) continue;
    a.fuse_twin = true;
  }
  // lifetimes of root buffers in layer steps: tensor t is written at step t-1 (input: -1)
  std::vector<int> birth(nt, 1 << 30), death(nt, -2);
  for (int t = 0; t < nt; ++t) {
    const int r = m.tensors[t].root;
    birth[r] = std::min(birth[r], t - 1);
    death[r] = std::max(death[r], t - 1);
  }
  for (int i = 0; i < (int)m.layers.size(); ++i)
    if (m.layers[i].fuse_pool || m.layers[i].fuse_twin) {      // the next layer's output is written one step early, by this layer
      const int r = m.tensors[i + 2].root;
      birth[r] = std::min(birth[r], i);
    }
  for (int i = 0; i < (int)m.layers.size(); ++i)
    for (int k = 0; k < m.layers[i].L.n_in; ++k) {
      const int r = m.tensors[m.layers[i].L.in[k]].root;
      death[r] = std::max(death[r], i);
    }
  const int forever = (int)m.layers.size() + 1;
  for (int t = 0; t < nt; ++t) if (is_output[t] || keep_all) death[m.tensors[t].root] = forever;
  const int es = dtype_size(m.d.dtype);
  auto root_bytes = [&](int r) {
    const TensorPlan& t = m.tensors[r];
    size_t b = (size_t)m.cap * t.h * t.w * t.ld * (t.f32 ? 4 : es);
    return (b + 255) & ~(size_t)255;
  };
  struct Block { size_t off, size; };
  std::vector<Block> free_list;
  size_t top = 0, peak = 0;
  std::vector<std::vector<int>> dying(forever + 2);
  for (int r = 0; r < nt; ++r) if (m.tensors[r].root == r && death[r] < forever) dying[death[r] + 1].push_back(r);
  auto release = [&](size_t off, size_t size) {
    free_list.push_back({off, size});
    std::sort(free_list.begin(), free_list.end(), [](const Block& a, const Block& b) { return a.off < b.off; });
    for (size_t k = 0; k + 1 < free_list.size();) {
      if (free_list[k].off + free_list[k].size == free_list[k + 1].off) { free_list[k].size += free_list[k + 1].size; free_list.erase(free_list.begin() + k + 1); }
      else ++k;
    }
    if (!free_list.empty() && free_list.back().off + free_list.back().size == top) { top = free_list.back().off; free_list.pop_back(); }
  };
  // step s allocates the roots born at s after freeing those whose last reader was step s-1
  for (int s = -1; s <= (int)m.layers.size(); ++s) {
    if (s >= 0) for (int r : dying[s]) release(m.tensors[r].root_off, root_bytes(r));
    for (int r = 0; r < nt; ++r) {
      if (m.tensors[r].root != r || birth[r] != s) continue;
      const size_t need = root_bytes(r);
      int best = -1;
      for (size_t k = 0; k < free_list.size(); ++k)
        if (free_list[k].size >= need && (best < 0 || free_list[k].size < free_list[best].size)) best = (int)k;
      if (best >= 0) {
        m.tensors[r].root_off = free_list[best].off;
        free_list[best].off += need; free_list[best].size -= need;
        if (free_list[best].size == 0) free_list.erase(free_list.begin() + best);
      } else {
        m.tensors[r].root_off = top;
        top += need;
        peak = std::max(peak, top);
      }
    }
  }
  m.act_bytes = peak;
}

TensorView view_of(const ModelPlan& m, int t) {
  const TensorPlan& tp = m.tensors[t];
  const TensorPlan& rt = m.tensors[tp.root];
  TensorView v;
  v.ptr = m.act_base + rt.root_off;
  v.h = tp.h; v.w = tp.w; v.c = tp.c; v.ld = tp.ld; v.coff = tp.coff;
  return v;
}

// ---- weights ----------------------------------------------------------------
octo_status pack_weights(octo_pipeline* p, ModelPlan& m, Arena& ar) {
  const int es = dtype_size(m.d.dtype);
  for (size_t li = 0; li < m.layers.size(); ++li) {
    LayerPlan& lp = m.layers[li];
    if (lp.L.op != OCTO_CONV && lp.L.op != OCTO_FC) continue;
    const int pk_kw = lp.pair_view ? lp.pair_kw : lp.L.kw, pk_cin = lp.pair_view ? 8 : lp.cin;
    lp.K = lp.L.kh * pk_kw * pk_cin;
    const size_t elems = conv_packed_weight_elems(lp.L.cout, lp.L.kh, pk_kw, pk_cin, m.d.dtype, &lp.Kp, &lp.cout_pad);
    lp.d_weight = ar.alloc(elems * es + 512);   // slack: the conv prefetch may read a K step past the last row
    lp.d_bias = (float*)ar.alloc((size_t)lp.cout_pad * sizeof(float));
    size_t twin_elems = 0;
    int twin_kp = 0;
    if (lp.fuse_twin) {      // this layer's and the next one's weights as one matrix (both 1x1 on the same input: same K)
      twin_elems = conv_packed_weight_elems(lp.L.cout + m.layers[li + 1].L.cout, 1, 1, lp.cin, m.d.dtype, &twin_kp, &lp.twin_cout_pad);
      lp.d_weight_twin = ar.alloc(twin_elems * es + 512);
      lp.d_bias_twin = (float*)ar.alloc((size_t)lp.twin_cout_pad * sizeof(float));
    }
    if (!ar.base) continue;
    if (ar.failed) return OCTO_ENOMEM;
    std::vector<char> host(elems * es, 0);
    if (lp.pair_view) {
      // w'[k][r][j][e]: e = 4*(pixel of the pair) + channel; window column s = 2j + e/4 - shift
      const int kw = lp.L.kw, cin = lp.cin;
      for (int k = 0; k < lp.L.cout; ++k)
        for (int r = 0; r < lp.L.kh; ++r)
          for (int j = 0; j < pk_kw; ++j)
            for (int e = 0; e < 8; ++e) {
              const int sc = 2 * j + e / 4 - lp.pair_shift, c = e % 4;
              if (sc < 0 || sc >= kw || c >= cin) continue;
              memcpy(host.data() + ((size_t)k * lp.Kp + ((size_t)r * pk_kw + j) * 8 + e) * es,
                     (const char*)lp.L.weight + ((((size_t)k * lp.L.kh + r) * kw + sc) * cin + c) * es, es);
            }
    } else {
      for (int k = 0; k < lp.L.cout; ++k)
        memcpy(host.data() + (size_t)k * lp.Kp * es, (const char*)lp.L.weight + (size_t)k * lp.K * es, (size_t)lp.K * es);
    }
    HIPCHK(p, hipMemcpy(lp.d_weight, host.data(), host.size(), hipMemcpyHostToDevice));
    std::vector<float> hb(lp.cout_pad, 0.f);
    memcpy(hb.data(), lp.L.bias, (size_t)lp.L.cout * sizeof(float));
    HIPCHK(p, hipMemcpy(lp.d_bias, hb.data(), hb.size() * sizeof(float), hipMemcpyHostToDevice));
    if (lp.fuse_twin) {
      const octo_layer& N = m.layers[li + 1].L;       // not packed yet: its host arrays are still there
      std::vector<char> tw(twin_elems * es, 0);
      std::vector<float> tb(lp.twin_cout_pad, 0.f);
      for (int k = 0; k < lp.L.cout; ++k)
        memcpy(tw.data() + (size_t)k * twin_kp * es, (const char*)lp.L.weight + (size_t)k * lp.K * es, (size_t)lp.K * es);
      for (int k = 0; k < N.cout; ++k)
        memcpy(tw.data() + (size_t)(lp.L.cout + k) * twin_kp * es, (const char*)N.weight + (size_t)k * lp.K * es, (size_t)lp.K * es);
      memcpy(tb.data(), lp.L.bias, (size_t)lp.L.cout * sizeof(float));
      memcpy(tb.data() + lp.L.cout, N.bias, (size_t)N.cout * sizeof(float));
      HIPCHK(p, hipMemcpy(lp.d_weight_twin, tw.data(), tw.size(), hipMemcpyHostToDevice));
      HIPCHK(p, hipMemcpy(lp.d_bias_twin, tb.data(), tb.size() * sizeof(float), hipMemcpyHostToDevice));
    }
    lp.L.weight = nullptr; lp.L.bias = nullptr;   // caller memory is not referenced after create
  }
  return OCTO_OK;
}

// ---- one layer ----------------------------------------------------------------
hipError_t run_layer(octo_pipeline* p, ModelPlan& m, int i, int n, const int* n_dyn, hipStream_t s, ConvTiming tm = ConvTiming()) {
  LayerPlan& lp = m.layers[i];
  const octo_layer& L = lp.L;
  const TensorView x = view_of(m, L.in[0]);
  const TensorView y = view_of(m, i + 1);
  switch (L.op) {
    case OCTO_CONV: case OCTO_FC: {
      ConvArgs a{};
      a.x = x.ptr; a.w = lp.d_weight; a.bias = lp.d_bias; a.y = y.ptr; a.n_dyn = n_dyn; a.n = n;
      a.H = x.h; a.W = x.w; a.Cin = x.c; a.x_ld = x.ld; a.x_coff = x.coff;
      a.Ho = y.h; a.Wo = y.w; a.Cout = y.c; a.y_ld = y.ld; a.y_coff = y.coff;
      a.kh = L.kh; a.kw = L.kw; a.stride_h = a.stride_w = L.stride; a.pad_h = a.pad_w = L.pad; a.K = lp.K; a.Kp = lp.Kp; a.w_rows = lp.cout_pad;
      if (lp.pair_view) { a.W = x.w / 2; a.Cin = 8; a.x_ld = 8; a.kw = lp.pair_kw; a.stride_w = 1; a.pad_w = lp.pair_pad; a.pair_view = 1; }
      a.act = L.act; a.res_mode = L.res_mode; a.out_f32 = m.tensors[i + 1].f32 ? 1 : 0;
      if (L.n_in == 2) { const TensorView r = view_of(m, L.in[1]); a.res = r.ptr; a.res_ld = r.ld; a.res_coff = r.coff; }
      if (n_dyn && m.items_hint > 0) a.n_hint = std::max(1, (int)(m.items_hint + 0.999));
      if (i > 0 && m.layers[i - 1].fuse_twin) { lp.kernel_id = KID_NONE; return hipSuccess; }     // computed by the layer before
      if (lp.fuse_twin) {
        const TensorView y2 = view_of(m, i + 2);
        ConvArgs f = a;
        f.Cout = L.cout + m.layers[i + 1].L.cout; f.w = lp.d_weight_twin; f.bias = lp.d_bias_twin; f.w_rows = lp.twin_cout_pad;
        f.y2 = y2.ptr; f.y2_ld = y2.ld; f.y2_coff = y2.coff; f.split = L.cout;
        const hipError_t e = launch_conv(m.d.dtype, f, p->num_cu, s, &lp.kernel_id, tm);
        if (e != hipErrorNotSupported) return e;
        lp.fuse_twin = false;
      }
      if (lp.fuse_pool) {
        const TensorView py = view_of(m, i + 2);
        ConvArgs f = a;
        f.pool_y = py.ptr; f.pool_ho = py.h; f.pool_wo = py.w; f.pool_ld = py.ld; f.pool_coff = py.coff;
        const hipError_t e = launch_conv(m.d.dtype, f, p->num_cu, s, &lp.kernel_id, tm);
        if (e != hipErrorNotSupported) return e;
        lp.fuse_pool = false;
      }
      return launch_conv(m.d.dtype, a, p->num_cu, s, &lp.kernel_id, tm);
    }
    case OCTO_MAXPOOL: {
      if (i > 0 && m.layers[i - 1].fuse_pool) { lp.kernel_id = KID_NONE; return hipSuccess; }
      PoolArgs a{x.ptr, y.ptr, n_dyn, n, x.h, x.w, x.c, x.ld, x.coff, y.h, y.w, y.ld, y.coff, L.kh, L.stride, L.pad};
      lp.kernel_id = KID_MAXPOOL;
      return launch_maxpool(m.d.dtype, a, s);
    }
    case OCTO_UPSAMPLE2X: {
      PoolArgs a{x.ptr, y.ptr, n_dyn, n, x.h, x.w, x.c, x.ld, x.coff, y.h, y.w, y.ld, y.coff, 1, 1, 0};
      lp.kernel_id = KID_UPSAMPLE;
      return launch_upsample2x(m.d.dtype, a, s);
    }
    case OCTO_CONCAT: {
      int off = 0;
      for (int k = 0; k < L.n_in; ++k) {
        const TensorView t = view_of(m, L.in[k]);
        if (std::find(lp.copy_inputs.begin(), lp.copy_inputs.end(), k) != lp.copy_inputs.end()) {
          PoolArgs a{t.ptr, y.ptr, n_dyn, n, t.h, t.w, t.c, t.ld, t.coff, y.h, y.w, y.ld, y.coff + off, 1, 1, 0};
          lp.kernel_id = KID_COPY;
          hipError_t e = launch_copy_channels(m.d.dtype, a, s);
          if (e != hipSuccess) return e;
        }
        off += t.c;
      }
      return hipSuccess;
    }
    case OCTO_ADD: {
      const TensorView b = view_of(m, L.in[1]);
      AddArgs a{x.ptr, b.ptr, y.ptr, n_dyn, n, x.h, x.w, x.c, x.ld, x.coff, b.ld, b.coff, y.ld, y.coff, L.act};
      lp.kernel_id = KID_ADD;
      return launch_add(m.d.dtype, a, s);
    }
    case OCTO_GAP: {
      PoolArgs a{x.ptr, y.ptr, n_dyn, n, x.h, x.w, x.c, x.ld, x.coff, 1, 1, y.ld, y.coff, 1, 1, 0};
      lp.kernel_id = KID_GAP;
      return launch_gap(m.d.dtype, a, s);
    }
  }
  return hipErrorInvalidValue;
}

hipError_t run_layers(octo_pipeline* p, ModelPlan& m, int n, const int* n_dyn, hipStream_t s, std::vector<hipEvent_t>* evs = nullptr) {
  hipError_t e;
  // timing events: [0..L] bracket the layers on the stream; [L+1+2i], [L+2+2i] ride on layer i's convolution dispatch
  const int L = (int)m.layers.size();
  if (evs && (e = hipEventRecord((*evs)[0], s)) != hipSuccess) return e;
  for (int i = 0; i < L; ++i) {
    ConvTiming tm;
    if (evs) { tm.start = (*evs)[L + 1 + 2 * i]; tm.stop = (*evs)[L + 2 + 2 * i]; }
    if ((e = run_layer(p, m, i, n, n_dyn, s, tm)) != hipSuccess) return e;
    if (evs && (e = hipEventRecord((*evs)[i + 1], s)) != hipSuccess) return e;
  }
  return hipSuccess;
}

// decode -> top-k -> NMS of a detector (root or child) for n items.  The head tensors hold items 0 .. n-1 of this
// execution; their results go to slots item0 .. item0 + n - 1 of the model's per-item arrays (item0 > 0 when the
// detector of one batch runs in several executions).
hipError_t run_detect_tail(octo_pipeline* p, ModelPlan& m, int n, const int* n_dyn, hipStream_t s, hipEvent_t* evs, int item0 = 0) {
  hipError_t e = launch_fill_i32(m.cand_count + (size_t)item0 * CNT_STRIDE, 0, n * CNT_STRIDE, s);
  if (e != hipSuccess) return e;
  DecodeArgs da{};
  da.n_levels = m.d.n_outputs;
  const int es = dtype_size(m.d.dtype);
  for (int l = 0; l < m.d.n_outputs; ++l) {
    const TensorView h = view_of(m, m.d.outputs[l]);
    if (m.head_override[l]) { da.head[l] = (const char*)m.head_override[l] + (size_t)item0 * h.h * h.w * h.c * es; da.head_ld[l] = h.c; }
    else { da.head[l] = (const char*)h.ptr + (size_t)h.coff * es; da.head_ld[l] = h.ld; }
    da.gh[l] = m.gh[l]; da.gw[l] = m.gw[l]; da.stride[l] = m.d.stride[l];
    memcpy(da.anchors[l], m.d.anchors[l], sizeof da.anchors[l]);
  }
  da.n_anchors = m.d.n_anchors; da.n_classes = m.d.n_classes; da.score_thr = m.d.score_thr;
  da.n = n; da.n_dyn = n_dyn; da.cand = m.cand + (size_t)item0 * m.n_cand; da.count = m.cand_count + (size_t)item0 * CNT_STRIDE; da.cap = m.n_cand;
  da.count_stride = CNT_STRIDE; da.overflow = m.flags + item0;
  if ((e = launch_decode(m.d.dtype, da, s)) != hipSuccess) return e;
  if (evs) hipEventRecord(evs[0], s);
  TopkArgs ta{da.cand, da.count, m.n_cand, CNT_STRIDE, m.top + (size_t)item0 * m.k_cap, m.top_count + item0, std::min(m.d.topk, m.n_cand), m.k_cap, n, n_dyn};
  if ((e = launch_topk(ta, s)) != hipSuccess) return e;
  if (evs) hipEventRecord(evs[1], s);
  // the suppression bit mask is scratch of one execution: every execution uses the first n items' worth of it
  NmsArgs na{ta.out, ta.out_count, m.k_cap, m.d.iou_thr, m.d.max_det, m.mask, m.keep + (size_t)item0 * m.d.max_det, m.n_keep + item0, n, n_dyn};
  if ((e = launch_nms(na, s)) != hipSuccess) return e;
  if (evs) hipEventRecord(evs[2], s);
  return hipSuccess;
}

octo_status build(octo_pipeline* p, const octo_pipeline_desc* desc, Arena& ar) {
  std::string why;
  if (!desc || !desc->models || desc->n_models < 1 || desc->n_edges < 0 || desc->n_edges > OCTO_MAX_EDGES ||
      (desc->n_edges > 0 && !desc->edges) || desc->src_h <= 0 || desc->src_w <= 0 || desc->max_frames < 1 ||
      desc->max_rois_per_frame < 0 || !(desc->slo_ms > 0))
    return fail(p, OCTO_EINVAL, "bad pipeline description");
  if (desc->models[0].kind != OCTO_DETECTOR || desc->models[0].in_c != 3) return fail(p, OCTO_EINVAL, "models[0] must be a 3-channel detector");
  p->d = *desc;
  p->max_frames = desc->max_frames;
  p->max_queue = desc->max_queue > 0 ? desc->max_queue : 4 * desc->max_frames;
  p->edges.assign(desc->edges, desc->edges + desc->n_edges);
  p->models.resize(desc->n_models);
  std::vector<int> edge_of_model(desc->n_models, -1);
  for (int e = 0; e < desc->n_edges; ++e) {
    const octo_edge& ed = p->edges[e];
    if (ed.parent != 0 || ed.child < 1 || ed.child >= desc->n_models || edge_of_model[ed.child] >= 0)
      return fail(p, OCTO_EINVAL, "edge %d: only root-to-child edges with one edge per child are supported", e);
    edge_of_model[ed.child] = e;
  }
  for (int k = 0; k < desc->n_models; ++k) {
    ModelPlan& m = p->models[k];
    m.d = desc->models[k];
    m.name = m.d.name ? m.d.name : "";
    m.d.name = nullptr;
    // a model without an incoming edge is detached: it only runs through octo_debug_run_model
    if (k > 0 && edge_of_model[k] >= 0 && m.d.in_c != 3) return fail(p, OCTO_EINVAL, "child models take 3-channel crops");
    octo_status st = plan_shapes(m, why);
    if (st != OCTO_OK) return fail(p, st, "model %d (%s): %s", k, m.name.c_str(), why.c_str());
    m.d.layers = nullptr;
    if (k == 0) {
      m.cap = desc->max_frames;
      m.bz = m.d.batch_size > 0 ? std::min(m.d.batch_size, m.cap) : m.cap;
    } else if (edge_of_model[k] >= 0) {
      const long long ecap = (long long)desc->max_frames * desc->max_rois_per_frame;
      m.cap = (int)std::max(1LL, m.d.batch_size > 0 ? std::min<long long>(m.d.batch_size, ecap) : ecap);
      m.bz = m.cap;
    } else {
      m.cap = std::max(1, m.d.batch_size);
      m.bz = m.cap;
    }
    plan_activations(m, desc->keep_all_tensors != 0, desc->keep_all_tensors != 1);
  }
  // ---- carve the workspace ----
  for (int k = 0; k < desc->n_models; ++k) {
    ModelPlan& m = p->models[k];
    octo_status st = pack_weights(p, m, ar);
    if (st != OCTO_OK) return st == OCTO_ENOMEM ? fail(p, st, "workspace too small") : st;
    m.act_base = (char*)ar.alloc(m.act_bytes);
    if (m.d.kind == OCTO_DETECTOR) {
      m.cand = (octo_cand*)ar.alloc((size_t)m.cap * m.n_cand * sizeof(octo_cand));
      m.cand_count = (int*)ar.alloc((size_t)m.cap * CNT_STRIDE * sizeof(int));
      m.top = (octo_cand*)ar.alloc((size_t)m.cap * m.k_cap * sizeof(octo_cand));
      m.top_count = (int*)ar.alloc((size_t)m.cap * sizeof(int));
      m.mask = (unsigned long long*)ar.alloc(nms_mask_bytes(m.cap, m.k_cap));
      if (k > 0) {
        m.keep = (int*)ar.alloc((size_t)m.cap * m.d.max_det * sizeof(int));
        m.flags = (int*)ar.alloc((size_t)m.cap * sizeof(int));
      }
    }
    if (k > 0) m.labels = (int*)ar.alloc((size_t)m.cap * sizeof(int));   // detector child: n_keep doubles as label
  }
  ModelPlan& root = p->models[0];
  // result block: n_keep[max_frames] | flags[max_frames] | n_roi[OCTO_MAX_EDGES] | boxes[max_frames][max_det]
  const size_t mf = (size_t)desc->max_frames;
  p->off_nkeep = 0;
  p->off_flags = p->off_nkeep + mf * sizeof(int);
  p->off_nroi = p->off_flags + mf * sizeof(int);
  p->off_boxes = (p->off_nroi + OCTO_MAX_EDGES * sizeof(int) + 31) & ~(size_t)31;
  p->result_bytes = p->off_boxes + mf * root.d.max_det * sizeof(octo_box);
  p->d_result = (char*)ar.alloc(p->result_bytes);
  root.keep = (int*)ar.alloc(mf * root.d.max_det * sizeof(int));
  for (int e = 0; e < desc->n_edges; ++e) {
    ModelPlan& c = p->models[p->edges[e].child];
    p->roi_cap[e] = c.cap;
    p->rois[e] = (octo_roi*)ar.alloc((size_t)c.cap * sizeof(octo_roi));
    p->roi_of[e] = (int*)ar.alloc(mf * root.d.max_det * sizeof(int));
    p->roi_cnt[e] = (int*)ar.alloc(mf * sizeof(int));
  }
  for (int r = 0; r < RING; ++r) {
    p->d_frames[r] = (const uint8_t**)ar.alloc(mf * sizeof(void*));
    p->d_pitch[r] = (size_t*)ar.alloc(mf * sizeof(size_t));
  }
  if (ar.base) {
    if (ar.failed) return fail(p, OCTO_ENOMEM, "workspace too small: need %zu bytes", ar.off);
    root.n_keep = (int*)(p->d_result + p->off_nkeep);
    root.flags = (int*)(p->d_result + p->off_flags);
    for (int e = 0; e < desc->n_edges; ++e) {
      p->n_roi[e] = (int*)(p->d_result + p->off_nroi) + e;
      ModelPlan& c = p->models[p->edges[e].child];
      c.n_dyn = p->n_roi[e];
      if (c.d.kind == OCTO_DETECTOR) c.n_keep = c.labels;
    }
  }
  if (ar.base)
    for (int k = 1; k < desc->n_models; ++k)
      if (p->models[k].d.kind == OCTO_DETECTOR) p->models[k].n_keep = p->models[k].labels;
  p->edge_of_model = edge_of_model;
  letterbox_geometry(desc->src_h, desc->src_w, root.d.in_h, root.d.in_w, &p->nw, &p->nh, &p->left, &p->top);
  return OCTO_OK;
}

hipEvent_t get_event(octo_pipeline* p) {
  if (!p->event_pool.empty()) { hipEvent_t e = p->event_pool.back(); p->event_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

enum { ST_LETTERBOX = 0, ST_DET_LAYERS, ST_DECODE, ST_TOPK, ST_NMS, ST_COMPACT, ST_FIXED };
// per edge: crop, layers, tail

octo_status enqueue_root(octo_pipeline* p, hipStream_t s, int n);

octo_status start_batch(octo_pipeline* p, hipStream_t s, int* launched) {
  ModelPlan& root = p->models[0];
  const int n = (int)std::min<size_t>(p->queue.size(), (size_t)root.bz);
  *launched = n;
  if (n == 0) return OCTO_OK;
  if ((int)p->inflight.size() >= RING - 1) { *launched = 0; return fail(p, OCTO_ESTATE, "too many uncollected batches (%d)", (int)p->inflight.size()); }
  // activations and ROI tables are single-buffered: a new batch may not start before the previous one is complete
  if (!p->inflight.empty()) HIPCHK(p, hipStreamWaitEvent(s, p->inflight.back().done, 0));
  // Everything that can fail before work is enqueued happens first: a batch that cannot get its events leaves the
  // queue, the slot counter and the list of batches in flight untouched.
  Batch b;
  b.n = n; b.slot = p->next_slot;
  auto give_back = [&](Batch& x) {
    if (x.done) p->event_pool.push_back(x.done);
    for (hipEvent_t e : x.stage_ev) p->event_pool.push_back(e);
    for (auto& v : x.layer_ev) for (hipEvent_t e : v) p->event_pool.push_back(e);
    x.done = nullptr; x.stage_ev.clear(); x.layer_ev.clear();
  };
  b.done = get_event(p);
  bool ok = b.done != nullptr;
  if (ok && p->stage_timing) {
    const int ne = 1 + ST_FIXED + 3 * (int)p->edges.size();
    for (int i = 0; i < ne && ok; ++i) { hipEvent_t e = get_event(p); if (e) b.stage_ev.push_back(e); else ok = false; }
  }
  b.layer_ev.resize(p->models.size());
  if (ok && p->layer_timing)
    for (size_t k = 0; k < p->models.size() && ok; ++k)
      for (size_t i = 0; i < 3 * p->models[k].layers.size() + 1 && ok; ++i) {
        hipEvent_t e = get_event(p); if (e) b.layer_ev[k].push_back(e); else ok = false;
      }
  if (!ok) { give_back(b); *launched = 0; return fail(p, OCTO_EHIP, "hipEventCreate failed"); }
  const void** hp = (const void**)p->h_tables[b.slot];
  size_t* hpitch = (size_t*)(p->h_tables[b.slot] + (size_t)p->max_frames * sizeof(void*));
  for (int i = 0; i < n; ++i) {
    const QueuedFrame& q = p->queue[i];
    hp[i] = q.ptr; hpitch[i] = q.pitch;
    b.ids.push_back(q.id); b.arrival.push_back(q.arrival);
  }
  b.t_launch = octo_now_ms();
  b.model_ran.assign(p->models.size(), false);
  p->inflight.push_back(std::move(b));
  // If enqueueing fails half-way, the batch is withdrawn again: its frames stay queued (a later run forms the batch anew;
  // whatever part was enqueued only wrote this pipeline's own buffers), and the handle stays usable.
  const octo_status st = enqueue_root(p, s, n);
  if (st != OCTO_OK) {
    give_back(p->inflight.back());
    p->inflight.pop_back();
    *launched = 0;
    return st;
  }
  p->next_slot = (p->next_slot + 1) % RING;
  p->queue.erase(p->queue.begin(), p->queue.begin() + n);
  p->inflight.back().model_ran[0] = true;
  return OCTO_OK;
}

// Enqueues the root model's part of the newest batch in flight (copy of the frame table, letterbox, detector, decode,
// top-k, NMS, ROI compaction) on `s`.
octo_status enqueue_root(octo_pipeline* p, hipStream_t s, int n) {
  ModelPlan& root = p->models[0];
  Batch& B = p->inflight.back();
  const void** hp = (const void**)p->h_tables[B.slot];
  size_t* hpitch = (size_t*)(p->h_tables[B.slot] + (size_t)p->max_frames * sizeof(void*));
  hipEvent_t* ev = p->stage_timing ? B.stage_ev.data() : nullptr;
  HIPCHK(p, hipMemcpyAsync(p->d_frames[B.slot], hp, n * sizeof(void*), hipMemcpyHostToDevice, s));
  HIPCHK(p, hipMemcpyAsync(p->d_pitch[B.slot], hpitch, n * sizeof(size_t), hipMemcpyHostToDevice, s));
  if (ev) HIPCHK(p, hipEventRecord(ev[0], s));
  ResizeArgs ra{};
  ra.src_h = p->d.src_h; ra.src_w = p->d.src_w;
  ra.dst = view_of(root, 0).ptr; ra.dst_h = root.d.in_h; ra.dst_w = root.d.in_w; ra.dst_c = root.input_c4 ? 4 : 3;
  for (int c = 0; c < 3; ++c) { ra.scale[c] = root.d.norm_scale[c]; ra.bias[c] = root.d.norm_bias[c]; }
  ra.pad_value = root.d.pad_value;
  HIPCHK(p, launch_fill_i32((int*)p->d_result, 0, (int)((p->off_boxes) / sizeof(int)), s));   // n_keep, flags, n_roi
  // The detector runs on exec_bz frames at a time (its own batch size; by default the whole batch), every execution
  // through the same activation buffers; candidates, top-k lists and keep lists are per frame and collect in place.
  // Stage events (when enabled) bracket the last execution's stages; the letterbox and layer stages of the earlier
  // executions fall into the "letterbox" interval.
  const int chunk = root.exec_bz > 0 && root.exec_bz < n ? root.exec_bz : n;
  for (int c0 = 0; c0 < n; c0 += chunk) {
    const int cn = std::min(chunk, n - c0);
    const bool last = c0 + cn >= n;
    ra.frames = p->d_frames[B.slot] + c0; ra.pitches = p->d_pitch[B.slot] + c0; ra.n = cn; ra.n_frames = cn;
    HIPCHK(p, launch_letterbox(root.d.dtype, ra, s));
    if (ev && last) HIPCHK(p, hipEventRecord(ev[1 + ST_LETTERBOX], s));
    HIPCHK(p, run_layers(p, root, cn, nullptr, s, p->layer_timing && last ? &B.layer_ev[0] : nullptr));
    if (ev && last) HIPCHK(p, hipEventRecord(ev[1 + ST_DET_LAYERS], s));
    HIPCHK(p, run_detect_tail(p, root, cn, nullptr, s, ev && last ? ev + 1 + ST_DECODE : nullptr, c0));
  }
  CompactArgs ca{};
  ca.top = root.top; ca.k_cap = root.k_cap; ca.keep = root.keep; ca.n_keep = root.n_keep; ca.max_det = root.d.max_det; ca.n = n;
  ca.left = (float)p->left; ca.top_pad = (float)p->top;
  ca.rx = (float)p->nw / (float)p->d.src_w; ca.ry = (float)p->nh / (float)p->d.src_h;
  ca.src_w = (float)p->d.src_w; ca.src_h = (float)p->d.src_h;
  ca.n_edges = (int)p->edges.size();
  for (int e = 0; e < ca.n_edges; ++e) {
    ca.class_mask[e][0] = p->edges[e].class_mask[0]; ca.class_mask[e][1] = p->edges[e].class_mask[1];
    ca.rois[e] = p->rois[e]; ca.n_roi[e] = p->n_roi[e]; ca.roi_cap[e] = p->roi_cap[e]; ca.roi_of[e] = p->roi_of[e]; ca.roi_cnt[e] = p->roi_cnt[e];
  }
  ca.boxes = (octo_box*)(p->d_result + p->off_boxes); ca.flags = root.flags;
  HIPCHK(p, launch_compact(ca, s));
  if (ev) HIPCHK(p, hipEventRecord(ev[1 + ST_COMPACT], s));
  HIPCHK(p, hipEventRecord(p->ev_det, s));
  return OCTO_OK;
}

octo_status run_child(octo_pipeline* p, Batch& B, int e, hipStream_t s, bool wait_det) {
  ModelPlan& c = p->models[p->edges[e].child];
  hipEvent_t* ev = p->stage_timing ? B.stage_ev.data() + 1 + ST_FIXED + 3 * e : nullptr;
  if (wait_det) HIPCHK(p, hipStreamWaitEvent(s, p->ev_det, 0));
  ResizeArgs ra{};
  ra.frames = p->d_frames[B.slot]; ra.pitches = p->d_pitch[B.slot]; ra.src_h = p->d.src_h; ra.src_w = p->d.src_w;
  ra.dst = view_of(c, 0).ptr; ra.dst_h = c.d.in_h; ra.dst_w = c.d.in_w; ra.dst_c = c.input_c4 ? 4 : 3;
  for (int k = 0; k < 3; ++k) { ra.scale[k] = c.d.norm_scale[k]; ra.bias[k] = c.d.norm_bias[k]; }
  ra.n = c.cap; ra.n_dyn = c.n_dyn; ra.rois = p->rois[e]; ra.n_frames = B.n;
  HIPCHK(p, launch_crop_resize(c.d.dtype, ra, s));
  if (ev) HIPCHK(p, hipEventRecord(ev[0], s));
  HIPCHK(p, run_layers(p, c, c.cap, c.n_dyn, s, p->layer_timing ? &B.layer_ev[p->edges[e].child] : nullptr));
  if (ev) HIPCHK(p, hipEventRecord(ev[1], s));
  if (c.d.kind == OCTO_CLASSIFIER) {
    const TensorView lg = view_of(c, c.d.outputs[0]);
    HIPCHK(p, launch_argmax((const float*)lg.ptr + lg.coff, lg.ld, c.n_logits, c.n_dyn, c.cap, c.labels, s));
  } else {
    HIPCHK(p, launch_fill_i32(c.flags, 0, c.cap, s));
    HIPCHK(p, run_detect_tail(p, c, c.cap, c.n_dyn, s, nullptr));
  }
  if (ev) HIPCHK(p, hipEventRecord(ev[2], s));
  HIPCHK(p, hipEventRecord(p->ev_child[e], s));
  B.model_ran[p->edges[e].child] = true;
  return OCTO_OK;
}

// cross_stream: models of this batch may have run on other streams, so wait for their events first
octo_status finalize_batch(octo_pipeline* p, Batch& B, hipStream_t s, bool cross_stream) {
  ModelPlan& root = p->models[0];
  if (cross_stream) {
    HIPCHK(p, hipStreamWaitEvent(s, p->ev_det, 0));
    for (int e = 0; e < (int)p->edges.size(); ++e) HIPCHK(p, hipStreamWaitEvent(s, p->ev_child[e], 0));
  }
  LabelArgs la{};
  la.boxes = (octo_box*)(p->d_result + p->off_boxes); la.n_keep = root.n_keep; la.max_det = root.d.max_det; la.n = B.n;
  la.n_edges = (int)p->edges.size();
  for (int e = 0; e < la.n_edges; ++e) { la.roi_of[e] = p->roi_of[e]; la.labels[e] = p->models[p->edges[e].child].labels; la.n_roi[e] = p->n_roi[e]; }
  HIPCHK(p, launch_scatter_labels(la, s));
  const size_t bytes = p->off_boxes + (size_t)B.n * root.d.max_det * sizeof(octo_box);
  HIPCHK(p, hipMemcpyAsync(p->h_result[B.slot], p->d_result, bytes, hipMemcpyDeviceToHost, s));
  HIPCHK(p, hipEventRecord(B.done, s));
  B.finalized = true;
  return OCTO_OK;
}

}  // namespace

extern "C" {

double octo_now_ms(void) {
  using namespace std::chrono;
  return duration<double, std::milli>(steady_clock::now().time_since_epoch()).count();
}

const char* octo_last_error(const octo_pipeline* p) { return p ? p->err.c_str() : g_create_error.c_str(); }

octo_status octo_pipeline_workspace_size(const octo_pipeline_desc* desc, size_t* device_bytes) {
  if (!device_bytes) return fail(nullptr, OCTO_EINVAL, "device_bytes is NULL");
  octo_pipeline tmp;
  Arena ar;
  octo_status st = build(&tmp, desc, ar);
  if (st != OCTO_OK) { g_create_error = tmp.err; return st; }
  *device_bytes = ((ar.off + 255) & ~(size_t)255) + 256;
  return OCTO_OK;
}

octo_status octo_pipeline_create(const octo_pipeline_desc* desc, void* device_workspace, size_t bytes, octo_pipeline** out) {
  if (!out || !device_workspace || ((uintptr_t)device_workspace & 255)) return fail(nullptr, OCTO_EINVAL, "bad workspace / out pointer");
  octo_pipeline* p = new (std::nothrow) octo_pipeline;
  if (!p) return fail(nullptr, OCTO_ENOMEM, "host allocation failed");
  Arena ar;
  ar.base = (char*)device_workspace; ar.cap = bytes;
  octo_status st = build(p, desc, ar);
  if (st == OCTO_OK) {
    int dev = 0; hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) p->num_cu = prop.multiProcessorCount;
    for (int r = 0; r < RING && st == OCTO_OK; ++r) {
      if (hipHostMalloc((void**)&p->h_result[r], p->result_bytes, hipHostMallocDefault) != hipSuccess ||
          hipHostMalloc((void**)&p->h_tables[r], (size_t)p->max_frames * (sizeof(void*) + sizeof(size_t)), hipHostMallocDefault) != hipSuccess)
        st = fail(p, OCTO_ENOMEM, "pinned host allocation failed");
    }
    if (st == OCTO_OK && hipEventCreate(&p->ev_det) != hipSuccess) st = fail(p, OCTO_EHIP, "hipEventCreate failed");
    for (size_t e = 0; e < p->edges.size() && st == OCTO_OK; ++e) {
      hipEvent_t ev;
      if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) st = fail(p, OCTO_EHIP, "hipEventCreate failed");
      else p->ev_child.push_back(ev);
    }
  }
  if (st != OCTO_OK) { g_create_error = p->err; octo_pipeline_destroy(p); return st; }
  *out = p;
  return OCTO_OK;
}

octo_status octo_pipeline_destroy(octo_pipeline* p) {
  if (!p) return OCTO_EINVAL;
  for (Batch& b : p->inflight) {
    if (b.done) { hipEventSynchronize(b.done); hipEventDestroy(b.done); }
    for (hipEvent_t e : b.stage_ev) hipEventDestroy(e);
    for (auto& v : b.layer_ev) for (hipEvent_t e : v) hipEventDestroy(e);
  }
  for (hipEvent_t e : p->event_pool) hipEventDestroy(e);
  if (p->ev_det) hipEventDestroy(p->ev_det);
  for (hipEvent_t e : p->ev_child) hipEventDestroy(e);
  for (int r = 0; r < RING; ++r) { if (p->h_result[r]) hipHostFree(p->h_result[r]); if (p->h_tables[r]) hipHostFree(p->h_tables[r]); }
  delete p;
  return OCTO_OK;
}

octo_status octo_submit_frames(octo_pipeline* p, const void* const* d_frames, const size_t* pitch_bytes,
                               const double* arrival_ms, const int64_t* frame_ids, int32_t n) {
  if (!p) return OCTO_EINVAL;
  if (!d_frames || !pitch_bytes || n < 0) return fail(p, OCTO_EINVAL, "bad submit arguments");
  for (int i = 0; i < n; ++i)
    if (!d_frames[i] || pitch_bytes[i] < (size_t)3 * p->d.src_w) return fail(p, OCTO_EINVAL, "frame %d: NULL pointer or pitch below 3*src_w", i);
  if ((int)p->queue.size() + n > p->max_queue) return fail(p, OCTO_ECAP, "frame queue full (%d queued, capacity %d)", (int)p->queue.size(), p->max_queue);
  const double now = octo_now_ms();
  for (int i = 0; i < n; ++i)
    p->queue.push_back({d_frames[i], pitch_bytes[i], arrival_ms ? arrival_ms[i] : now, frame_ids ? frame_ids[i] : (int64_t)i});
  return OCTO_OK;
}

octo_status octo_set_batch_size(octo_pipeline* p, int32_t model, int32_t bz) {
  if (!p) return OCTO_EINVAL;
  if (model < 0 || model >= (int)p->models.size() || bz < 1 || bz > p->models[model].cap) return fail(p, OCTO_EINVAL, "bad model or batch size");
  // a downstream model runs once per batch on however many ROIs its parent emitted (the count stays on the device), so
  // it has no launch batch size to set: a scheduler's batch size for it only sizes its time slot
  if (model > 0) return fail(p, OCTO_EINVAL, "model %d is a downstream model: it always takes the whole ROI set of a batch", model);
  p->models[model].bz = bz;
  return OCTO_OK;
}

octo_status octo_set_detector_batch(octo_pipeline* p, int32_t frames_per_execution) {
  if (!p) return OCTO_EINVAL;
  if (frames_per_execution < 0 || frames_per_execution > p->models[0].cap) return fail(p, OCTO_EINVAL, "bad detector batch size");
  p->models[0].exec_bz = frames_per_execution;
  return OCTO_OK;
}

octo_status octo_run_model(octo_pipeline* p, int32_t model, void* hip_stream, int32_t* n_items_launched) {
  if (!p) return OCTO_EINVAL;
  if (model < 0 || model >= (int)p->models.size()) return fail(p, OCTO_EINVAL, "bad model index");
  hipStream_t s = (hipStream_t)hip_stream;
  int dummy = 0;
  int* out = n_items_launched ? n_items_launched : &dummy;
  if (model == 0) {
    if (!p->inflight.empty() && !p->inflight.back().finalized) return fail(p, OCTO_ESTATE, "previous batch still has models to run");
    octo_status st = start_batch(p, s, out);
    if (st != OCTO_OK || *out == 0) return st;
    if (p->edges.empty()) return finalize_batch(p, p->inflight.back(), s, false);
    return OCTO_OK;
  }
  if (p->inflight.empty() || p->inflight.back().finalized) { *out = 0; return OCTO_OK; }
  Batch& B = p->inflight.back();
  if (p->edge_of_model[model] < 0) return fail(p, OCTO_EINVAL, "model %d is detached", model);
  if (B.model_ran[model]) return fail(p, OCTO_ESTATE, "model %d already ran for this batch", model);
  int e = 0;
  while (p->edges[e].child != model) ++e;
  octo_status st = run_child(p, B, e, s, true);
  if (st != OCTO_OK) return st;
  *out = B.n;
  bool all = true;
  for (size_t k = 0; k < p->models.size(); ++k) all = all && (B.model_ran[k] || (k > 0 && p->edge_of_model[k] < 0));
  if (all) return finalize_batch(p, B, s, true);
  return OCTO_OK;
}

octo_status octo_run(octo_pipeline* p, void* hip_stream, int32_t* n_frames_launched) {
  if (!p) return OCTO_EINVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  int dummy = 0;
  int* out = n_frames_launched ? n_frames_launched : &dummy;
  if (!p->inflight.empty() && !p->inflight.back().finalized) return fail(p, OCTO_ESTATE, "previous batch still has models to run");
  octo_status st = start_batch(p, s, out);
  if (st != OCTO_OK || *out == 0) return st;
  Batch& B = p->inflight.back();
  for (int e = 0; e < (int)p->edges.size(); ++e)
    if ((st = run_child(p, B, e, s, false)) != OCTO_OK) return st;
  return finalize_batch(p, B, s, false);   // same stream throughout: stream order already serialises the stages
}

octo_status octo_collect(octo_pipeline* p, octo_frame_result* frames, int32_t frame_cap, octo_box* boxes, int32_t box_cap,
                         int32_t* n_frames, int32_t* n_boxes, int32_t blocking) {
  if (!p) return OCTO_EINVAL;
  if (!frames || !n_frames || !n_boxes || frame_cap < 0 || box_cap < 0 || (box_cap > 0 && !boxes)) return fail(p, OCTO_EINVAL, "bad collect arguments");
  *n_frames = 0; *n_boxes = 0;
  bool overflow = false;
  while (!p->inflight.empty()) {
    Batch& B = p->inflight.front();
    if (!B.finalized) break;
    if (blocking && *n_frames == 0) HIPCHK(p, hipEventSynchronize(B.done));
    else {
      hipError_t q = hipEventQuery(B.done);
      if (q == hipErrorNotReady) break;
      if (q != hipSuccess) return fail(p, OCTO_EHIP, "hipEventQuery failed: %s", hipGetErrorString(q));
    }
    const double t_done = octo_now_ms();
    const char* h = p->h_result[B.slot];
    const int* nk = (const int*)(h + p->off_nkeep);
    const int* fl = (const int*)(h + p->off_flags);
    const octo_box* hb = (const octo_box*)(h + p->off_boxes);
    const int max_det = p->models[0].d.max_det;
    const int* nroi = (const int*)(h + p->off_nroi);
    for (size_t e = 0; e < p->edges.size(); ++e) {
      // what the children saw: the next batches' kernels are shaped for about as many items
      ModelPlan& c = p->models[p->edges[e].child];
      const double obs = std::min(nroi[e], c.cap);
      c.items_hint = c.items_hint > 0 ? 0.75 * c.items_hint + 0.25 * obs : obs;
    }
    int total = 0;
    for (int i = 0; i < B.n; ++i) total += std::min(nk[i], max_det);
    if (*n_frames + B.n > frame_cap || *n_boxes + total > box_cap) {
      if (*n_frames == 0) return fail(p, OCTO_ECAP, "oldest batch (%d frames, %d boxes) does not fit the output arrays", B.n, total);
      break;
    }
    for (int i = 0; i < B.n; ++i) {
      octo_frame_result& fr = frames[*n_frames];
      const int k = std::min(nk[i], max_det);
      fr.frame_id = B.ids[i]; fr.n_boxes = k; fr.latency_ms = (float)(t_done - B.arrival[i]);
      fr.slo_met = fr.latency_ms <= p->d.slo_ms ? 1 : 0; fr.flags = fl[i]; fr.box_offset = *n_boxes; fr.pad_ = 0;
      if (fl[i]) overflow = true;
      memcpy(boxes + *n_boxes, hb + (size_t)i * max_det, (size_t)k * sizeof(octo_box));
      *n_boxes += k; ++*n_frames;
    }
    if (!B.stage_ev.empty()) {
      p->last_stage_ms.assign(B.stage_ev.size() - 1, 0.f);
      for (size_t k = 0; k + 1 < B.stage_ev.size(); ++k) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, B.stage_ev[k], B.stage_ev[k + 1]) == hipSuccess) p->last_stage_ms[k] = ms;
      }
      for (hipEvent_t e : B.stage_ev) p->event_pool.push_back(e);
    }
    p->last_layer_ms.assign(p->models.size(), std::vector<float>());
    for (size_t k = 0; k < B.layer_ev.size(); ++k) {
      const std::vector<hipEvent_t>& le = B.layer_ev[k];
      const size_t L = p->models[k].layers.size();
      for (size_t i = 0; i < L && le.size() == 3 * L + 1; ++i) {
        // convolutions: the kernel's own run time from the events on its dispatch; other layers: stream bracket
        // (a convolution that launched nothing - its work was done by the layer before - has no dispatch events; a
        // failed query must not stay behind as the runtime's last error either: the next launch would report it)
        const LayerPlan& lq = p->models[k].layers[i];
        const bool conv = (lq.L.op == OCTO_CONV || lq.L.op == OCTO_FC) && lq.kernel_id != KID_NONE;
        float ms = 0.f;
        if (!B.model_ran[k]) ms = 0.f;
        else if (conv && hipEventElapsedTime(&ms, le[L + 1 + 2 * i], le[L + 2 + 2 * i]) == hipSuccess) {}
        else {
          if (conv) (void)hipGetLastError();
          if (hipEventElapsedTime(&ms, le[i], le[i + 1]) != hipSuccess) { ms = 0.f; (void)hipGetLastError(); }
        }
        p->last_layer_ms[k].push_back(ms);
      }
      for (hipEvent_t e : le) p->event_pool.push_back(e);
    }
    p->event_pool.push_back(B.done);
    p->inflight.pop_front();
  }
  if (*n_frames == 0) return blocking ? fail(p, OCTO_ESTATE, "nothing in flight") : OCTO_ENOTREADY;
  return overflow ? OCTO_ECAP : OCTO_OK;
}

// Compute-unit bit i of a stream mask selects unit i / 8 of accelerator die i % 8 on this GPU (measured with a
// kernel that reads its die id under different masks).  A mask that leaves a die without units is refused here:
// the runtime does not accept it.
static const int N_XCD = 8;

octo_status octo_stream_create_masked(const uint32_t* cu_mask, int32_t n_words, void** hip_stream) {
  if (!cu_mask || n_words <= 0 || !hip_stream) return OCTO_EINVAL;
  int per_die[N_XCD] = {0};
  for (int b = 0; b < 32 * n_words; ++b)
    if (cu_mask[b / 32] >> (b % 32) & 1u) per_die[b % N_XCD]++;
  for (int d = 0; d < N_XCD; ++d)
    if (per_die[d] == 0) return OCTO_EINVAL;
  hipStream_t s = nullptr;
  if (hipExtStreamCreateWithCUMask(&s, (uint32_t)n_words, cu_mask) != hipSuccess) return OCTO_EHIP;
  *hip_stream = (void*)s;
  return OCTO_OK;
}
octo_status octo_stream_create_range(int32_t first_cu, int32_t n_cu, void** hip_stream) {
  int32_t total = 0;
  if (octo_device_cu_count(&total) != OCTO_OK) return OCTO_EHIP;
  if (first_cu < 0 || n_cu < N_XCD || first_cu % N_XCD || n_cu % N_XCD || first_cu + n_cu > total) return OCTO_EINVAL;
  std::vector<uint32_t> mask((size_t)(total + 31) / 32, 0u);
  for (int b = first_cu; b < first_cu + n_cu; ++b) mask[b / 32] |= 1u << (b % 32);
  return octo_stream_create_masked(mask.data(), (int32_t)mask.size(), hip_stream);
}
octo_status octo_stream_destroy(void* hip_stream) {
  if (!hip_stream) return OCTO_EINVAL;
  return hipStreamDestroy((hipStream_t)hip_stream) == hipSuccess ? OCTO_OK : OCTO_EHIP;
}
octo_status octo_device_cu_count(int32_t* n_cu) {
  if (!n_cu) return OCTO_EINVAL;
  int dev = 0; hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return OCTO_EHIP;
  *n_cu = prop.multiProcessorCount;
  return OCTO_OK;
}

octo_status octo_set_stage_timing(octo_pipeline* p, int32_t enable) {
  if (!p) return OCTO_EINVAL;
  p->stage_timing = enable != 0;
  return OCTO_OK;
}
octo_status octo_get_stage_ms(octo_pipeline* p, float* ms, int32_t cap, int32_t* n) {
  if (!p || !ms || !n) return OCTO_EINVAL;
  *n = (int)std::min<size_t>(p->last_stage_ms.size(), (size_t)std::max(cap, 0));
  for (int i = 0; i < *n; ++i) ms[i] = p->last_stage_ms[i];
  return OCTO_OK;
}

octo_status octo_set_layer_timing(octo_pipeline* p, int32_t enable) {
  if (!p) return OCTO_EINVAL;
  p->layer_timing = enable != 0;
  return OCTO_OK;
}

octo_status octo_get_layer_info(octo_pipeline* p, int32_t model, float* ms, int32_t* kernel_id, double* flops, double* bytes,
                                double* weight_bytes, int32_t cap, int32_t* n) {
  if (!p) return OCTO_EINVAL;
  if (model < 0 || model >= (int)p->models.size() || !n || cap < 0) return fail(p, OCTO_EINVAL, "bad arguments");
  const ModelPlan& m = p->models[model];
  *n = (int)std::min<size_t>(m.layers.size(), (size_t)cap);
  for (int i = 0; i < *n; ++i) {
    if (ms) ms[i] = (model < (int)p->last_layer_ms.size() && i < (int)p->last_layer_ms[model].size()) ? p->last_layer_ms[model][i] : 0.f;
    if (kernel_id) kernel_id[i] = m.layers[i].kernel_id;
    // two layers in one launch: the work is reported with the first, the second did nothing
    const bool first = m.layers[i].fuse_twin && i + 1 < (int)m.layers.size(), second = i > 0 && m.layers[i - 1].fuse_twin;
    if (flops) flops[i] = second ? 0.0 : m.layers[i].flops + (first ? m.layers[i + 1].flops : 0.0);
    if (bytes) bytes[i] = second ? 0.0 : m.layers[i].bytes + (first ? m.layers[i + 1].bytes - m.layers[i].input_bytes : 0.0);
    if (weight_bytes) weight_bytes[i] = second ? 0.0 : m.layers[i].weight_bytes + (first ? m.layers[i + 1].weight_bytes : 0.0);
  }
  return OCTO_OK;
}

octo_status octo_profile_layers(octo_pipeline* p, int32_t model, int32_t n, int32_t iters, void* hip_stream,
                                float* ms, double* flops, double* bytes, int32_t cap) {
  if (!p) return OCTO_EINVAL;
  if (model < 0 || model >= (int)p->models.size() || iters < 1 || !ms) return fail(p, OCTO_EINVAL, "bad profile arguments");
  ModelPlan& m = p->models[model];
  if (n < 1 || n > m.cap || cap < (int)m.layers.size()) return fail(p, OCTO_EINVAL, "bad item count or output capacity");
  hipStream_t s = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  HIPCHK(p, hipEventCreate(&e0));
  HIPCHK(p, hipEventCreate(&e1));
  for (int i = 0; i < (int)m.layers.size(); ++i) {
    HIPCHK(p, run_layer(p, m, i, n, nullptr, s));   // warm-up
    HIPCHK(p, hipEventRecord(e0, s));
    for (int it = 0; it < iters; ++it) HIPCHK(p, run_layer(p, m, i, n, nullptr, s));
    HIPCHK(p, hipEventRecord(e1, s));
    HIPCHK(p, hipEventSynchronize(e1));
    float t = 0.f;
    HIPCHK(p, hipEventElapsedTime(&t, e0, e1));
    ms[i] = t / iters;
    const bool first = m.layers[i].fuse_twin && i + 1 < (int)m.layers.size(), second = i > 0 && m.layers[i - 1].fuse_twin;
    if (flops) flops[i] = second ? 0.0 : (m.layers[i].flops + (first ? m.layers[i + 1].flops : 0.0)) * n;
    if (bytes) bytes[i] = second ? 0.0 : (m.layers[i].bytes + (first ? m.layers[i + 1].bytes - m.layers[i].input_bytes : 0.0)) * n +
                                             m.layers[i].weight_bytes + (first ? m.layers[i + 1].weight_bytes : 0.0);
  }
  hipEventDestroy(e0); hipEventDestroy(e1);
  return OCTO_OK;
}

octo_status octo_debug_tensor_shape(octo_pipeline* p, int32_t model, int32_t tensor_id, int32_t* h, int32_t* w, int32_t* c) {
  if (!p) return OCTO_EINVAL;
  if (model < 0 || model >= (int)p->models.size() || tensor_id < 0 || tensor_id >= (int)p->models[model].tensors.size() || !h || !w || !c)
    return fail(p, OCTO_EINVAL, "bad tensor reference");
  const TensorPlan& t = p->models[model].tensors[tensor_id];
  *h = t.h; *w = t.w; *c = t.c;
  return OCTO_OK;
}

octo_status octo_debug_get_tensor(octo_pipeline* p, int32_t model, int32_t tensor_id, int32_t first_item, int32_t n_items,
                                  void* host_dst, size_t bytes) {
  if (!p) return OCTO_EINVAL;
  if (model < 0 || model >= (int)p->models.size() || tensor_id < 0 || tensor_id >= (int)p->models[model].tensors.size() || !host_dst)
    return fail(p, OCTO_EINVAL, "bad tensor reference");
  ModelPlan& m = p->models[model];
  const TensorPlan& t = m.tensors[tensor_id];
  if (first_item < 0 || n_items < 0 || (long long)first_item + n_items > m.cap) return fail(p, OCTO_EINVAL, "bad item range");
  const size_t es = t.f32 ? 4 : dtype_size(m.d.dtype);
  const size_t rows = (size_t)n_items * t.h * t.w;
  if (bytes < rows * t.c * es) return fail(p, OCTO_EINVAL, "destination too small");
  HIPCHK(p, hipDeviceSynchronize());
  const TensorView v = view_of(m, tensor_id);
  if (rows == 0) return OCTO_OK;
  const char* src = (const char*)v.ptr + ((size_t)first_item * t.h * t.w * v.ld + (size_t)v.coff) * es;
  HIPCHK(p, hipMemcpy2D(host_dst, t.c * es, src, (size_t)v.ld * es, t.c * es, rows, hipMemcpyDeviceToHost));
  return OCTO_OK;
}

octo_status octo_debug_set_head(octo_pipeline* p, int32_t model, int32_t level, const void* d_head) {
  if (!p) return OCTO_EINVAL;
  if (model < 0 || model >= (int)p->models.size() || p->models[model].d.kind != OCTO_DETECTOR || level < 0 || level >= p->models[model].d.n_outputs)
    return fail(p, OCTO_EINVAL, "bad model or level");
  p->models[model].head_override[level] = d_head;
  return OCTO_OK;
}

octo_status octo_debug_run_model(octo_pipeline* p, int32_t model, const void* d_input, int32_t n, void* hip_stream) {
  if (!p) return OCTO_EINVAL;
  if (model < 0 || model >= (int)p->models.size() || !d_input) return fail(p, OCTO_EINVAL, "bad arguments");
  ModelPlan& m = p->models[model];
  if (n < 1 || n > m.cap) return fail(p, OCTO_EINVAL, "bad item count");
  hipStream_t s = (hipStream_t)hip_stream;
  const TensorPlan& t0 = m.tensors[0];
  const size_t bytes = (size_t)n * t0.h * t0.w * t0.c * dtype_size(m.d.dtype);
  if (m.input_c4) {
    HIPCHK(p, hipMemsetAsync(view_of(m, 0).ptr, 0, (size_t)n * t0.h * t0.w * 4 * dtype_size(m.d.dtype), s));
    PoolArgs ca{d_input, view_of(m, 0).ptr, nullptr, n, t0.h, t0.w, 3, 3, 0, t0.h, t0.w, 4, 0, 1, 1, 0};
    HIPCHK(p, launch_copy_channels(m.d.dtype, ca, s));
  } else {
    HIPCHK(p, hipMemcpyAsync(view_of(m, 0).ptr, d_input, bytes, hipMemcpyDeviceToDevice, s));
  }
  HIPCHK(p, run_layers(p, m, n, nullptr, s));
  if (m.d.kind == OCTO_DETECTOR) {
    if (m.flags) HIPCHK(p, launch_fill_i32(m.flags, 0, m.cap, s));
    HIPCHK(p, run_detect_tail(p, m, n, nullptr, s, nullptr));
  } else if (m.labels) {
    const TensorView lg = view_of(m, m.d.outputs[0]);
    HIPCHK(p, launch_argmax((const float*)lg.ptr + lg.coff, lg.ld, m.n_logits, nullptr, n, m.labels, s));
  }
  return OCTO_OK;
}

octo_status octo_debug_get_detections(octo_pipeline* p, int32_t model, int32_t item, int32_t* cand_count,
                                      octo_cand* top, int32_t top_cap, int32_t* n_top, int32_t* keep, int32_t keep_cap, int32_t* n_keep) {
  if (!p) return OCTO_EINVAL;
  if (model < 0 || model >= (int)p->models.size() || p->models[model].d.kind != OCTO_DETECTOR) return fail(p, OCTO_EINVAL, "bad model");
  ModelPlan& m = p->models[model];
  if (item < 0 || item >= m.cap) return fail(p, OCTO_EINVAL, "bad item");
  HIPCHK(p, hipDeviceSynchronize());
  int cc = 0, nt = 0, nk = 0;
  HIPCHK(p, hipMemcpy(&cc, m.cand_count + (size_t)item * CNT_STRIDE, sizeof(int), hipMemcpyDeviceToHost));
  HIPCHK(p, hipMemcpy(&nt, m.top_count + item, sizeof(int), hipMemcpyDeviceToHost));
  HIPCHK(p, hipMemcpy(&nk, m.n_keep + item, sizeof(int), hipMemcpyDeviceToHost));
  nk = std::min(nk, m.d.max_det);
  if (cand_count) *cand_count = cc;
  if (n_top) *n_top = nt;
  if (n_keep) *n_keep = nk;
  if (top && top_cap > 0) HIPCHK(p, hipMemcpy(top, m.top + (size_t)item * m.k_cap, (size_t)std::min(nt, top_cap) * sizeof(octo_cand), hipMemcpyDeviceToHost));
  if (keep && keep_cap > 0) HIPCHK(p, hipMemcpy(keep, m.keep + (size_t)item * m.d.max_det, (size_t)std::min(nk, keep_cap) * sizeof(int), hipMemcpyDeviceToHost));
  return OCTO_OK;
}

octo_status octo_debug_get_rois(octo_pipeline* p, int32_t edge, octo_roi* rois, int32_t cap, int32_t* n_rois) {
  if (!p) return OCTO_EINVAL;
  if (edge < 0 || edge >= (int)p->edges.size() || !n_rois) return fail(p, OCTO_EINVAL, "bad edge");
  HIPCHK(p, hipDeviceSynchronize());
  int n = 0;
  HIPCHK(p, hipMemcpy(&n, p->n_roi[edge], sizeof(int), hipMemcpyDeviceToHost));
  *n_rois = n;
  if (rois && cap > 0 && n > 0) HIPCHK(p, hipMemcpy(rois, p->rois[edge], (size_t)std::min(n, cap) * sizeof(octo_roi), hipMemcpyDeviceToHost));
  return OCTO_OK;
}

octo_status octo_debug_get_labels(octo_pipeline* p, int32_t edge, int32_t* labels, int32_t cap, int32_t* n) {
  if (!p) return OCTO_EINVAL;
  if (edge < 0 || edge >= (int)p->edges.size() || !n) return fail(p, OCTO_EINVAL, "bad edge");
  HIPCHK(p, hipDeviceSynchronize());
  int k = 0;
  HIPCHK(p, hipMemcpy(&k, p->n_roi[edge], sizeof(int), hipMemcpyDeviceToHost));
  *n = k;
  if (labels && cap > 0 && k > 0) HIPCHK(p, hipMemcpy(labels, p->models[p->edges[edge].child].labels, (size_t)std::min(k, cap) * sizeof(int), hipMemcpyDeviceToHost));
  return OCTO_OK;
}

}  // extern "C"
