// Stage-level C ABI entry points: argument checks and one launch each of the
// kernels the pipeline itself uses, on caller-owned device buffers.
#include <cmath>
#include <cstring>
#include <mutex>

#include "octo_internal.h"

using namespace octo;

// Suppression-mask memory of octo_op_nms_static: one copy per GPU, held until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress; the kernels get the device address that call returns.
static __device__ __align__(256) unsigned char scratch[OCTO_NMS_STATIC_BYTES];

namespace {
octo_status from_hip(hipError_t e) { return e == hipSuccess ? OCTO_OK : (e == hipErrorInvalidValue ? OCTO_EINVAL : OCTO_EHIP); }
bool valid_dtype(int dt) { return dt == OCTO_F32 || dt == OCTO_F16 || dt == OCTO_BF16; }

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_addr[MAX_DEVICES] = {};   // device address of `scratch` on each GPU, looked up on first use there

// Device address of the static scratch array on the current device.
octo_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return OCTO_EHIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_addr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return OCTO_EHIP;
    g_scratch_addr[dev] = p;
  }
  *out = g_scratch_addr[dev];
  return OCTO_OK;
}
}  // namespace

extern "C" {

octo_status octo_letterbox_geometry(int32_t src_h, int32_t src_w, int32_t dst_h, int32_t dst_w,
                                    int32_t* nw, int32_t* nh, int32_t* left, int32_t* top) {
  if (!nw || !nh || !left || !top || src_h <= 0 || src_w <= 0 || dst_h <= 0 || dst_w <= 0 || src_h > 16384 || src_w > 16384 || dst_h > 16384 || dst_w > 16384)
    return OCTO_EINVAL;
  int a, b, c, d;
  letterbox_geometry(src_h, src_w, dst_h, dst_w, &a, &b, &c, &d);
  *nw = a; *nh = b; *left = c; *top = d;
  return OCTO_OK;
}

octo_status octo_op_letterbox(const void* d_frame_ptrs, const void* d_pitches, int32_t n, int32_t src_h, int32_t src_w,
                              void* d_dst, int32_t dst_h, int32_t dst_w, int32_t dtype, const float* scale3, const float* bias3,
                              int32_t pad_value, void* hip_stream) {
  if (!d_frame_ptrs || !d_pitches || !d_dst || !scale3 || !bias3 || n < 0 || src_h <= 0 || src_w <= 0 || dst_h <= 0 || dst_w <= 0 ||
      !valid_dtype(dtype) || pad_value < 0 || pad_value > 255 || src_h > 16384 || src_w > 16384 || dst_h > 16384 || dst_w > 16384)
    return OCTO_EINVAL;
  ResizeArgs a{};
  a.frames = (const uint8_t* const*)d_frame_ptrs; a.pitches = (const size_t*)d_pitches; a.src_h = src_h; a.src_w = src_w;
  a.dst = d_dst; a.dst_h = dst_h; a.dst_w = dst_w; a.dst_c = 3; a.pad_value = pad_value; a.n = n; a.n_frames = n;
  for (int c = 0; c < 3; ++c) { a.scale[c] = scale3[c]; a.bias[c] = bias3[c]; }
  return from_hip(launch_letterbox(dtype, a, (hipStream_t)hip_stream));
}

octo_status octo_op_crop_resize(const void* d_frame_ptrs, const void* d_pitches, int32_t n_frames, int32_t src_h, int32_t src_w,
                                const octo_roi* d_rois, const int32_t* d_n_rois, int32_t cap,
                                void* d_dst, int32_t out_h, int32_t out_w, int32_t dtype, const float* scale3, const float* bias3,
                                void* hip_stream) {
  if (!d_frame_ptrs || !d_pitches || !d_rois || !d_n_rois || !d_dst || !scale3 || !bias3 || cap < 0 || n_frames < 1 || src_h <= 0 || src_w <= 0 ||
      out_h <= 0 || out_w <= 0 || !valid_dtype(dtype))
    return OCTO_EINVAL;
  ResizeArgs a{};
  a.frames = (const uint8_t* const*)d_frame_ptrs; a.pitches = (const size_t*)d_pitches; a.src_h = src_h; a.src_w = src_w;
  a.dst = d_dst; a.dst_h = out_h; a.dst_w = out_w; a.dst_c = 3; a.n = cap; a.n_dyn = d_n_rois; a.rois = d_rois;
  a.n_frames = n_frames;
  for (int c = 0; c < 3; ++c) { a.scale[c] = scale3[c]; a.bias[c] = bias3[c]; }
  return from_hip(launch_crop_resize(dtype, a, (hipStream_t)hip_stream));
}

// ---- E4M3 on the host ---------------------------------------------------------
namespace {
// nearest integer, ties to even, for 0 <= x <= 16 (independent of the floating-point rounding mode)
int round_half_even(float x) {
  const int r = (int)x;                       // floor for x >= 0
  const float d = x - (float)r;
  return d > 0.5f || (d == 0.5f && (r & 1)) ? r + 1 : r;
}
uint8_t e4m3_encode(float f) {
  if (f != f) return 0x7F;
  const uint8_t sign = std::signbit(f) ? 0x80 : 0x00;
  float a = std::fabs(f);
  if (a > 448.0f) a = 448.0f;
  if (a < 0.015625f) return sign | (uint8_t)round_half_even(a * 512.0f);     // below 2^-6: multiples of 2^-9; 8 is the first normal code
  int e = 0;
  const float m = std::frexp(a, &e);          // a = m * 2^e, 0.5 <= m < 1
  int q = round_half_even((m * 2.0f - 1.0f) * 8.0f), ex = e - 1;              // a = (1 + q/8) * 2^ex before rounding q
  if (q == 8) { q = 0; ++ex; }
  return sign | (uint8_t)(((ex + 7) << 3) | q);
}
float e4m3_decode(uint8_t c) {
  const int ex = (c >> 3) & 15, q = c & 7;
  if (ex == 15 && q == 7) return std::nanf("");
  const float mag = ex == 0 ? std::ldexp((float)q, -9) : std::ldexp(1.0f + (float)q / 8.0f, ex - 7);
  return (c & 0x80) ? -mag : mag;
}
int cached_cu_count() {
  static std::mutex mu;
  static int cus[MAX_DEVICES] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return 0;
  std::lock_guard<std::mutex> lock(mu);
  if (!cus[dev]) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
    cus[dev] = prop.multiProcessorCount;
  }
  return cus[dev];
}
bool conv_dtype(int dt) { return valid_dtype(dt) || dt == OCTO_F8; }
}  // namespace

octo_status octo_quantize_e4m3(const float* src, size_t n, float inv_scale, uint8_t* dst) {
  if ((!src || !dst) && n) return OCTO_EINVAL;
  for (size_t i = 0; i < n; ++i) dst[i] = e4m3_encode(src[i] * inv_scale);
  return OCTO_OK;
}
octo_status octo_dequantize_e4m3(const uint8_t* src, size_t n, float scale, float* dst) {
  if ((!src || !dst) && n) return OCTO_EINVAL;
  for (size_t i = 0; i < n; ++i) dst[i] = e4m3_decode(src[i]) * scale;
  return OCTO_OK;
}

// ---- one convolution layer ------------------------------------------------------
int32_t octo_op_conv_padded_cout(int32_t cout) { return cout > 0 ? (cout + 127) / 128 * 128 : 0; }

size_t octo_op_conv_packed_bytes(int32_t dtype, int32_t cout, int32_t kh, int32_t kw, int32_t cin) {
  if (!conv_dtype(dtype) || cout < 1 || kh < 1 || kw < 1 || cin < 1) return 0;
  // slack after the last row: the operand prefetch may read one K step past it
  return conv_packed_weight_elems(cout, kh, kw, cin, dtype, nullptr, nullptr) * (size_t)dtype_size(dtype) + 512;
}

octo_status octo_op_conv_pack(int32_t dtype, const void* w, int32_t cout, int32_t kh, int32_t kw, int32_t cin, void* packed) {
  const size_t bytes = octo_op_conv_packed_bytes(dtype, cout, kh, kw, cin);
  if (!w || !packed || !bytes) return OCTO_EINVAL;
  int kp = 0, rows = 0;
  conv_packed_weight_elems(cout, kh, kw, cin, dtype, &kp, &rows);
  const size_t es = (size_t)dtype_size(dtype), k = (size_t)kh * kw * cin;
  memset(packed, 0, bytes);
  for (int r = 0; r < cout; ++r) memcpy((char*)packed + (size_t)r * kp * es, (const char*)w + (size_t)r * k * es, k * es);
  return OCTO_OK;
}

octo_status octo_op_conv(const octo_conv_op* op, void* hip_stream, int32_t* kernel_id) {
  if (!op || !conv_dtype(op->dtype) || !op->d_x || !op->d_w || !op->d_bias || !op->d_y) return OCTO_EINVAL;
  if (op->n < 0 || op->h < 1 || op->w < 1 || op->cin < 1 || op->cout < 1 || op->kh < 1 || op->kw < 1 || op->stride < 1 || op->pad < 0) return OCTO_EINVAL;
  if (op->x_ld < op->cin || op->y_ld < op->cout || (op->d_res && op->res_ld < op->cout)) return OCTO_EINVAL;
  if (op->act < OCTO_ACT_NONE || op->act > OCTO_ACT_SILU || op->res_mode < OCTO_RES_NONE || op->res_mode > OCTO_RES_AFTER_ACT) return OCTO_EINVAL;
  if ((op->d_res != nullptr) != (op->res_mode != OCTO_RES_NONE)) return OCTO_EINVAL;
  if ((((uintptr_t)op->d_x | (uintptr_t)op->d_y | (uintptr_t)op->d_res | (uintptr_t)op->d_w) & 15) != 0) return OCTO_EINVAL;
  const int ho = (op->h + 2 * op->pad - op->kh) / op->stride + 1, wo = (op->w + 2 * op->pad - op->kw) / op->stride + 1;
  if (op->h + 2 * op->pad < op->kh || op->w + 2 * op->pad < op->kw || ho < 1 || wo < 1) return OCTO_EINVAL;
  if (op->dtype == OCTO_F8 && (!op->d_scale || op->cin % 16 || op->x_ld % 16 || !(op->y_inv_scale > 0.0f) || (op->d_res && !(op->res_scale > 0.0f)))) return OCTO_EINVAL;
  if (op->n == 0) { if (kernel_id) *kernel_id = 0; return OCTO_OK; }
  const int cus = cached_cu_count();
  if (cus < 1) return OCTO_EHIP;
  ConvArgs a{};
  int kp = 0, rows = 0;
  conv_packed_weight_elems(op->cout, op->kh, op->kw, op->cin, op->dtype, &kp, &rows);
  a.x = op->d_x; a.w = op->d_w; a.bias = op->d_bias; a.y = op->d_y; a.n = op->n;
  a.H = op->h; a.W = op->w; a.Cin = op->cin; a.x_ld = op->x_ld;
  a.Ho = ho; a.Wo = wo; a.Cout = op->cout; a.y_ld = op->y_ld;
  a.kh = op->kh; a.kw = op->kw; a.stride_h = a.stride_w = op->stride; a.pad_h = a.pad_w = op->pad;
  a.K = op->kh * op->kw * op->cin; a.Kp = kp; a.w_rows = rows;
  a.act = op->act; a.res_mode = op->res_mode; a.out_f32 = op->out_f32 ? 1 : 0;
  if (op->d_res) { a.res = op->d_res; a.res_ld = op->res_ld; }
  if (op->dtype == OCTO_F8) { a.scale = op->d_scale; a.res_scale = op->d_res ? op->res_scale : 0.0f; a.y_inv_scale = op->y_inv_scale; }
  int kid = 0;
  const hipError_t e = launch_conv(op->dtype, a, cus, (hipStream_t)hip_stream, &kid);
  if (kernel_id) *kernel_id = kid;
  return from_hip(e);
}

octo_status octo_op_decode(const octo_model_desc* model, const void* const* d_heads, int32_t n,
                           octo_cand* d_cand, int32_t* d_count, int32_t cap, void* hip_stream) {
  if (!model || !d_heads || !d_cand || !d_count || n < 0 || cap < 1 || !valid_dtype(model->dtype) || model->n_outputs < 1 ||
      model->n_outputs > OCTO_MAX_LEVELS || model->n_anchors < 1 || model->n_anchors > OCTO_MAX_ANCHORS || model->n_classes < 1)
    return OCTO_EINVAL;
  DecodeArgs a{};
  a.n_levels = model->n_outputs;
  for (int l = 0; l < a.n_levels; ++l) {
    if (!d_heads[l] || model->stride[l] <= 0 || model->in_h % model->stride[l] || model->in_w % model->stride[l]) return OCTO_EINVAL;
    a.head[l] = d_heads[l];
    a.head_ld[l] = model->n_anchors * (5 + model->n_classes);
    a.gh[l] = model->in_h / model->stride[l]; a.gw[l] = model->in_w / model->stride[l]; a.stride[l] = model->stride[l];
    memcpy(a.anchors[l], model->anchors[l], sizeof a.anchors[l]);
  }
  a.n_anchors = model->n_anchors; a.n_classes = model->n_classes; a.score_thr = model->score_thr;
  a.n = n; a.cand = d_cand; a.count = d_count; a.cap = cap; a.count_stride = 1;
  hipStream_t s = (hipStream_t)hip_stream;
  hipError_t e = launch_fill_i32(d_count, 0, n, s);
  if (e != hipSuccess) return from_hip(e);
  return from_hip(launch_decode(model->dtype, a, s));
}

octo_status octo_op_topk(const octo_cand* d_in, const int32_t* d_in_count, int32_t in_cap, int32_t n, int32_t k,
                         octo_cand* d_out, int32_t* d_out_count, int32_t k_cap, void* hip_stream) {
  if (!d_in || !d_in_count || !d_out || !d_out_count || n < 0 || k < 1 || k > k_cap || in_cap < 1) return OCTO_EINVAL;
  TopkArgs a{d_in, d_in_count, in_cap, 1, d_out, d_out_count, k, k_cap, n, nullptr};
  return from_hip(launch_topk(a, (hipStream_t)hip_stream));
}

size_t octo_op_nms_scratch_bytes(int32_t n, int32_t k_cap) { return n > 0 && k_cap > 0 ? nms_mask_bytes(n, k_cap) : 0; }

octo_status octo_op_nms(const octo_cand* d_top, const int32_t* d_top_count, int32_t k_cap, int32_t n, float iou_thr, int32_t max_det,
                        void* d_mask_scratch, int32_t* d_keep, int32_t* d_n_keep, void* hip_stream) {
  if (!d_top || !d_top_count || !d_mask_scratch || !d_keep || !d_n_keep || n < 0 || max_det < 1 || k_cap < 64 || k_cap % 64 || k_cap > 4096 ||
      !(iou_thr >= 0))
    return OCTO_EINVAL;
  NmsArgs a{d_top, d_top_count, k_cap, iou_thr, max_det, (unsigned long long*)d_mask_scratch, d_keep, d_n_keep, n, nullptr};
  return from_hip(launch_nms(a, (hipStream_t)hip_stream));
}

octo_status octo_op_nms_static(const octo_cand* d_top, const int32_t* d_top_count, int32_t k_cap, int32_t n, float iou_thr, int32_t max_det,
                               int32_t* d_keep, int32_t* d_n_keep, void* hip_stream) {
  if (!d_top || !d_top_count || !d_keep || !d_n_keep || n < 0 || max_det < 1 || k_cap < 64 || k_cap % 64 || k_cap > 4096 || !(iou_thr >= 0))
    return OCTO_EINVAL;
  if (n == 0) return OCTO_OK;
  if (nms_mask_bytes(n, k_cap) > (size_t)OCTO_NMS_STATIC_BYTES) return OCTO_ECAP;
  void* mask = nullptr;
  const octo_status st = static_scratch(&mask);
  if (st != OCTO_OK) return st;
  // every mask word the reduction reads is written by the mask kernel of the same call, so nothing is cleared
  NmsArgs a{d_top, d_top_count, k_cap, iou_thr, max_det, (unsigned long long*)mask, d_keep, d_n_keep, n, nullptr};
  return from_hip(launch_nms(a, (hipStream_t)hip_stream));
}

octo_status octo_op_compact(const octo_cand* d_top, int32_t k_cap, const int32_t* d_keep, const int32_t* d_n_keep, int32_t max_det,
                            int32_t n, int32_t src_h, int32_t src_w, int32_t in_h, int32_t in_w, const uint64_t* class_mask2,
                            octo_roi* d_rois, int32_t* d_n_rois, int32_t cap, int32_t* d_roi_of, int32_t* d_item_counts, octo_box* d_boxes, int32_t* d_flags,
                            void* hip_stream) {
  if (!d_top || !d_keep || !d_n_keep || !class_mask2 || !d_rois || !d_n_rois || !d_roi_of || !d_item_counts || n < 0 || cap < 0 || max_det < 1 || k_cap < 1 ||
      src_h <= 0 || src_w <= 0 || in_h <= 0 || in_w <= 0)
    return OCTO_EINVAL;
  int nw, nh, left, top;
  letterbox_geometry(src_h, src_w, in_h, in_w, &nw, &nh, &left, &top);
  CompactArgs a{};
  a.top = d_top; a.k_cap = k_cap; a.keep = d_keep; a.n_keep = d_n_keep; a.max_det = max_det; a.n = n;
  a.left = (float)left; a.top_pad = (float)top; a.rx = (float)nw / (float)src_w; a.ry = (float)nh / (float)src_h;
  a.src_w = (float)src_w; a.src_h = (float)src_h;
  a.n_edges = 1; a.class_mask[0][0] = class_mask2[0]; a.class_mask[0][1] = class_mask2[1];
  a.rois[0] = d_rois; a.n_roi[0] = d_n_rois; a.roi_cap[0] = cap; a.roi_of[0] = d_roi_of; a.roi_cnt[0] = d_item_counts;
  a.boxes = d_boxes; a.flags = d_flags;
  return from_hip(launch_compact(a, (hipStream_t)hip_stream));
}

}  // extern "C"
