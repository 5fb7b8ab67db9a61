// Internal declarations shared by the HIP translation units of libocto.
// Nothing here is part of the public C ABI (that is include/octo.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/octo.h"

namespace octo {

// A view of an NHWC activation tensor.  `ld` is the element distance between two
// pixels and `coff` the first channel inside that pitch, so a tensor can be a
// channel slice of a wider (concatenation) buffer.
struct TensorView {
  void* ptr = nullptr;
  int h = 0, w = 0, c = 0;
  int ld = 0, coff = 0;
};

struct ConvArgs {
  const void* x;
  const void* w;        // packed weights [cout_pad][kp]
  const float* bias;    // [cout]
  const void* res;      // optional residual (same h, w, cout as y)
  void* y;
  const int* n_dyn;     // optional: number of items actually present (device), clamped to n
  int n;                // item capacity
  int H, W, Cin, x_ld, x_coff;
  int Ho, Wo, Cout, y_ld, y_coff;
  int res_ld, res_coff;
  int kh, kw, stride_h, stride_w, pad_h, pad_w;
  int K, Kp;
  int w_rows;                     // rows of the packed weight matrix (cout padded to a multiple of 128)
  unsigned magic_howo, shift_howo, magic_wo, shift_wo; int HoWo_is_one;   // pixel index -> (image, row, column)
  unsigned magic_cin, magic_kw;   // floor(2^32 / d) + 1 for d = Cin, kw (set by launch_conv)
  int act, res_mode;
  int out_f32;          // write fp32 instead of the storage type
  int n_hint;           // host only: expected item count when it is taken on the device (0: assume n); picks the tile shape
  int pair_view;        // the layer is a 3-channel first layer run on pixel pairs of a 4-channel-padded input
  // Fused 3x3 / stride-2 / pad-1 max-pool (first-layer kernel only): when pool_y is set, only the pooled tensor is
  // written and y is not touched; launch_conv returns hipErrorNotSupported if no kernel can do that for the layer.
  void* pool_y;
  int pool_ho, pool_wo, pool_ld, pool_coff;
  // Two layers in one launch (general kernel, 16-bit types, no residual): output channels below `split` go to y as
  // usual, channels split .. Cout - 1 to y2 as its channels 0 ..; split is a multiple of 8 and 0 when unused.
  void* y2;
  int y2_ld, y2_coff, split;
  // 8-bit floating point storage only: y = act(acc * scale[c] + bias[c] (+ res * res_scale)), stored as
  // E4M3(y * y_inv_scale) unless out_f32.  scale: device, one factor per output channel, padded like the bias.
  const float* scale;
  float res_scale, y_inv_scale;
};

// element size of a storage type
inline __host__ __device__ int dtype_size(int dt) { return dt == OCTO_F32 ? 4 : (dt == OCTO_F8 ? 1 : 2); }

// ---- launchers (each enqueues on `s`, never synchronises) -------------------
// Optional pair of events attached to the convolution's own dispatch (start and end of the kernel on the device).
struct ConvTiming { hipEvent_t start = nullptr, stop = nullptr; };
hipError_t launch_conv(int dtype, const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id = nullptr, ConvTiming tm = ConvTiming());
// first-layer kernel for pixel-pair layers; hipErrorNotSupported when the layer does not fit it
hipError_t launch_stem(int dtype, const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, ConvTiming tm);
// 3x3 stride-1 kernel with the input patch in LDS; hipErrorNotSupported when the layer does not fit it
hipError_t launch_conv3x3_patch(int dtype, const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, ConvTiming tm);
// 3x3 stride-1 kernel for wide layers (patch in LDS, 192 / 256-channel tiles); hipErrorNotSupported when the layer does not fit it
hipError_t launch_conv3x3_big(int dtype, const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, ConvTiming tm);
int conv_kernel_id(int bc, int bp, int kv, int minb, bool vec, bool dma = false);
enum { KID_NONE = 0, KID_MAXPOOL = 1, KID_UPSAMPLE = 2, KID_COPY = 3, KID_ADD = 4, KID_GAP = 5 };
size_t conv_packed_weight_elems(int cout, int kh, int kw, int cin, int dtype, int* kp_out, int* cout_pad_out);

struct PoolArgs {
  const void* x; void* y; const int* n_dyn; int n;
  int H, W, C, x_ld, x_coff, Ho, Wo, y_ld, y_coff, k, stride, pad;
};
hipError_t launch_maxpool(int dtype, const PoolArgs& a, hipStream_t s);
hipError_t launch_upsample2x(int dtype, const PoolArgs& a, hipStream_t s);       // uses H, W, C, lds/coffs
hipError_t launch_copy_channels(int dtype, const PoolArgs& a, hipStream_t s);    // y[:, :, :, coff:coff+C] = x
struct AddArgs {
  const void* a; const void* b; void* y; const int* n_dyn; int n;
  int H, W, C, a_ld, a_coff, b_ld, b_coff, y_ld, y_coff, act;
};
hipError_t launch_add(int dtype, const AddArgs& a, hipStream_t s);
hipError_t launch_gap(int dtype, const PoolArgs& a, hipStream_t s);              // y [n][C] mean over H*W
hipError_t launch_argmax(const float* logits, int ld, int n_out, const int* n_dyn, int n, int* labels, hipStream_t s);
hipError_t launch_fill_i32(int* p, int value, int count, hipStream_t s);

// floor(n / d) for n < 2^31 by multiply-high and shift; built on the host
struct FastDiv { unsigned mul, shift; int is_one; };
inline FastDiv make_fastdiv(unsigned d) {
  FastDiv f{0u, 0u, d <= 1u ? 1 : 0};
  if (f.is_one) return f;
  unsigned s = 0;
  while ((1ull << s) < d) ++s;
  const unsigned long long m = ((1ull << (32 + s)) + d - 1) / d;
  if (m >> 32) { f.mul = (unsigned)(((1ull << (31 + s)) + d - 1) / d); f.shift = s - 1; }
  else { f.mul = (unsigned)m; f.shift = s; }
  return f;
}
#ifdef __HIPCC__
__device__ __forceinline__ unsigned fast_div(unsigned n, const FastDiv& f) { return f.is_one ? n : __umulhi(n, f.mul) >> f.shift; }
#endif

struct ResizeArgs {
  const uint8_t* const* frames;   // device table of frame base pointers
  const size_t* pitches;          // device table of row pitches in bytes
  int src_h, src_w;
  void* dst; int dst_h, dst_w;
  int dst_c;                      // 3, or 4: a zero fourth channel so that two neighbouring pixels form one 16-byte vector
  float scale[3], bias[3];
  int pad_value;
  int n; const int* n_dyn;
  // crop mode only
  const octo_roi* rois;
  int n_frames;                   // frames behind `frames` (ROI frame indices are clamped to it)
  FastDiv div_wq, div_h;          // set by the launchers: lanes per output row, rows per item
};
void letterbox_geometry(int src_h, int src_w, int dst_h, int dst_w, int* nw, int* nh, int* left, int* top);
hipError_t launch_letterbox(int dtype, const ResizeArgs& a, hipStream_t s);
hipError_t launch_crop_resize(int dtype, const ResizeArgs& a, hipStream_t s);

struct DecodeArgs {
  const void* head[3]; int head_ld[3];
  int n_levels; int gh[3], gw[3], stride[3]; float anchors[3][3][2];
  int n_anchors, n_classes; float score_thr;
  int n; const int* n_dyn;
  octo_cand* cand; int* count; int cap;      // per item: cand[item*cap ...], count[item*count_stride]
  int count_stride;                          // >= 1; 32 puts every item's counter on its own 128-byte line
  int* overflow;
};
hipError_t launch_decode(int dtype, const DecodeArgs& a, hipStream_t s);

struct TopkArgs {
  const octo_cand* in; const int* in_count; int in_cap;
  int in_count_stride;
  octo_cand* out; int* out_count; int k;     // out stride = k_cap
  int k_cap;
  int n; const int* n_dyn;
};
hipError_t launch_topk(const TopkArgs& a, hipStream_t s);

struct NmsArgs {
  const octo_cand* top; const int* top_count; int k_cap;     // k_cap multiple of 64
  float iou_thr; int max_det;
  unsigned long long* mask;                                  // [n][k_cap][k_cap/64]
  int* keep; int* n_keep;                                    // keep[item*max_det ...]
  int n; const int* n_dyn;
};
hipError_t launch_nms(const NmsArgs& a, hipStream_t s);
size_t nms_mask_bytes(int n, int k_cap);

struct CompactArgs {
  const octo_cand* top; int k_cap;
  const int* keep; const int* n_keep; int max_det;
  int n; const int* n_dyn;
  // geometry of the letterbox that produced the boxes (identity for child detectors)
  float left, top_pad, rx, ry, src_w, src_h;
  int n_edges; uint64_t class_mask[OCTO_MAX_EDGES][2];
  octo_roi* rois[OCTO_MAX_EDGES]; int* n_roi[OCTO_MAX_EDGES]; int roi_cap[OCTO_MAX_EDGES];
  int* roi_of[OCTO_MAX_EDGES];             // [n][max_det] -> roi id or -1 (required)
  int* roi_cnt[OCTO_MAX_EDGES];            // [n] scratch: ROIs per item (required)
  octo_box* boxes;                         // [n][max_det] final boxes in source pixels
  int* flags;                              // [n]
};
hipError_t launch_compact(const CompactArgs& a, hipStream_t s);

struct LabelArgs {
  octo_box* boxes; const int* n_keep; int max_det; int n;
  int n_edges; const int* roi_of[OCTO_MAX_EDGES]; const int* labels[OCTO_MAX_EDGES]; const int* n_roi[OCTO_MAX_EDGES];
};
hipError_t launch_scatter_labels(const LabelArgs& a, hipStream_t s);

// ---- host-side scheduling (no GPU) ------------------------------------------
int cwd_search(octo_sched_pipeline* p);
int coral_schedule(octo_sched_pipeline* ps, int n_pipelines, double mem, double util_max, int n_streams,
                   octo_placement* out);

}  // namespace octo
