// Detector post-processing: box decode + score threshold, per-item top-k,
// class-wise greedy NMS, ROI compaction and label scatter.
//
// Every decision that produces an integer (threshold, order, suppression) is
// taken in fp32 with individually rounded operations (no contraction to FMA),
// so that the keep-lists and ROI tables are a deterministic function of the
// decoded candidates.
#include "octo_internal.h"

namespace octo {

__device__ __forceinline__ int dyn_n(const int* n_dyn, int n) {
  if (!n_dyn) return n;
  int d = *n_dyn;
  return d < n ? (d < 0 ? 0 : d) : n;
}

// logistic function, fp32, correctly rounded division
__device__ __forceinline__ float sigmoidf(float z) { return __fdiv_rn(1.0f, __fadd_rn(1.0f, expf(-z))); }

// ---------------------------------------------------------------------------
// decode + threshold: one lane per candidate; kept candidates are appended to the
// item's list through a wavefront-aggregated atomic (ballot + popcount).
// ---------------------------------------------------------------------------
template <typename T>
__global__ void decode_kernel(const DecodeArgs a, int cand_per_item) {
  const int n_items = dyn_n(a.n_dyn, a.n);
  const int item = blockIdx.y;
  if (item >= n_items) return;
  const int no = 5 + a.n_classes;
  const int lane = threadIdx.x & 63;
  const int chunks = (cand_per_item + blockDim.x - 1) / blockDim.x;
  for (int ch = blockIdx.x; ch < chunks; ch += gridDim.x) {
    const int idx = ch * blockDim.x + threadIdx.x;
    bool keep = false;
    octo_cand c;
    if (idx < cand_per_item) {
      int l = 0, off = 0;
      while (l + 1 < a.n_levels && idx >= off + a.gh[l] * a.gw[l] * a.n_anchors) { off += a.gh[l] * a.gw[l] * a.n_anchors; ++l; }
      const int local = idx - off;
      const int an = local % a.n_anchors;
      const int cell = local / a.n_anchors;
      const int gx = cell % a.gw[l], gy = cell / a.gw[l];
      const T* t = (const T*)a.head[l] + ((size_t)item * a.gh[l] * a.gw[l] + cell) * a.head_ld[l] + an * no;
      const float sobj = sigmoidf((float)t[4]);
      if (sobj > a.score_thr) {   // score = sobj * s(cls) <= sobj, so nothing is lost by testing objectness first
        int cls = 0;
        float best = (float)t[5];
        for (int k = 1; k < a.n_classes; ++k) {
          float v = (float)t[5 + k];
          if (v > best) { best = v; cls = k; }
        }
        const float score = __fmul_rn(sobj, sigmoidf(best));
        if (score > a.score_thr) {
          const float st = (float)a.stride[l];
          const float sx = sigmoidf((float)t[0]), sy = sigmoidf((float)t[1]);
          const float sw = sigmoidf((float)t[2]), sh = sigmoidf((float)t[3]);
          const float cx = __fmul_rn(__fadd_rn(__fsub_rn(__fmul_rn(2.0f, sx), 0.5f), (float)gx), st);
          const float cy = __fmul_rn(__fadd_rn(__fsub_rn(__fmul_rn(2.0f, sy), 0.5f), (float)gy), st);
          const float tw = __fmul_rn(2.0f, sw), th = __fmul_rn(2.0f, sh);
          const float w = __fmul_rn(__fmul_rn(tw, tw), a.anchors[l][an][0]);
          const float h = __fmul_rn(__fmul_rn(th, th), a.anchors[l][an][1]);
          const float hw = __fmul_rn(w, 0.5f), hh = __fmul_rn(h, 0.5f);
          c.x1 = __fsub_rn(cx, hw); c.y1 = __fsub_rn(cy, hh);
          c.x2 = __fadd_rn(cx, hw); c.y2 = __fadd_rn(cy, hh);
          c.score = score; c.cls = cls; c.idx = idx; c.pad_ = 0;
          keep = true;
        }
      }
    }
    const unsigned long long m = __ballot(keep);
    if (m) {
      int base = 0;
      const int leader = __ffsll((long long)m) - 1;
      if (lane == leader) base = atomicAdd(&a.count[item], __popcll(m));
      base = __shfl(base, leader);
      if (keep) {
        const int slot = base + __popcll(m & ((1ull << lane) - 1ull));
        if (slot < a.cap) a.cand[(size_t)item * a.cap + slot] = c;
        else if (a.overflow) atomicOr(a.overflow + item, OCTO_FLAG_CAND_OVERFLOW);
      }
    }
  }
}

hipError_t launch_decode(int dtype, const DecodeArgs& a, hipStream_t s) {
  if (a.n <= 0) return hipSuccess;
  int cand = 0;
  for (int l = 0; l < a.n_levels; ++l) cand += a.gh[l] * a.gw[l] * a.n_anchors;
  int chunks = (cand + 255) / 256;
  dim3 grid(chunks > 1024 ? 1024 : chunks, a.n);
  switch (dtype) {
    case OCTO_F32: hipLaunchKernelGGL(decode_kernel<float>, grid, dim3(256), 0, s, a, cand); break;
    case OCTO_F16: hipLaunchKernelGGL(decode_kernel<_Float16>, grid, dim3(256), 0, s, a, cand); break;
    case OCTO_BF16: hipLaunchKernelGGL(decode_kernel<__bf16>, grid, dim3(256), 0, s, a, cand); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// top-k: one workgroup per item sorts (key, slot) pairs in LDS with a bitonic
// network.  key = score bits << 32 | ~idx, so descending key order is
// (score descending, idx ascending); scores are positive finite floats.
// Lists longer than the LDS capacity are folded in: the best k so far stay in
// the first k slots and the rest of the buffer is refilled.
// ---------------------------------------------------------------------------
constexpr int TOPK_P = 4096;
constexpr int TOPK_THREADS = 1024;

__device__ __forceinline__ void bitonic_desc(unsigned long long* key, unsigned* val, int P) {
  for (int size = 2; size <= P; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      __syncthreads();
      for (int t = threadIdx.x; t < P / 2; t += blockDim.x) {
        const int lo = 2 * t - (t & (stride - 1));
        const int hi = lo + stride;
        const bool desc = (lo & size) == 0;
        const unsigned long long a = key[lo], b = key[hi];
        if ((a < b) == desc) {
          key[lo] = b; key[hi] = a;
          const unsigned va = val[lo]; val[lo] = val[hi]; val[hi] = va;
        }
      }
    }
  }
  __syncthreads();
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_kernel(const TopkArgs a) {
  __shared__ unsigned long long key[TOPK_P];
  __shared__ unsigned val[TOPK_P];
  const int n_items = dyn_n(a.n_dyn, a.n);
  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    int count = a.in_count[item];
    if (count > a.in_cap) count = a.in_cap;
    if (count < 0) count = 0;
    const octo_cand* in = a.in + (size_t)item * a.in_cap;
    const int kk = count < a.k ? count : a.k;
    int consumed = 0;
    int have = 0;                       // entries carried over from the previous fold (already in slots [0, have))
    __syncthreads();
    while (true) {
      int take = count - consumed;
      if (take > TOPK_P - have) take = TOPK_P - have;
      const int filled = have + take;
      int P = 64;
      while (P < filled) P <<= 1;
      for (int t = threadIdx.x; t < P - have; t += blockDim.x) {
        unsigned long long k = 0ull; unsigned v = 0u;
        if (t < take) {
          const octo_cand c = in[consumed + t];
          k = ((unsigned long long)__float_as_uint(c.score) << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)c.idx);
          v = (unsigned)(consumed + t);
        }
        key[have + t] = k; val[have + t] = v;
      }
      bitonic_desc(key, val, P);
      consumed += take;
      if (consumed >= count) break;
      have = kk;                        // count > TOPK_P here, so kk == k <= TOPK_P / 2
    }
    octo_cand* out = a.out + (size_t)item * a.k_cap;
    for (int t = threadIdx.x; t < kk; t += blockDim.x) out[t] = in[val[t]];
    if (threadIdx.x == 0) a.out_count[item] = kk;
    __syncthreads();
  }
}

hipError_t launch_topk(const TopkArgs& a, hipStream_t s) {
  if (a.n <= 0) return hipSuccess;
  if (a.k > a.k_cap || (a.in_cap > TOPK_P && a.k > TOPK_P / 2) || a.k > TOPK_P) return hipErrorInvalidValue;
  hipLaunchKernelGGL(topk_kernel, dim3(a.n > 1024 ? 1024 : a.n), dim3(TOPK_THREADS), 0, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// NMS.  Step 1 fills, for every sorted box i and every 64-box column block, a
// 64-bit word whose bit j says "i suppresses box 64*block + j" (j later in the
// order).  Step 2 walks the order with one wavefront per item: lane w owns word
// w of the "removed" bitmap.
// ---------------------------------------------------------------------------
__device__ __forceinline__ bool suppresses(float ax1, float ay1, float ax2, float ay2, float aarea,
                                           float bx1, float by1, float bx2, float by2, float barea, float thr) {
  const float iw = fmaxf(0.0f, __fsub_rn(fminf(ax2, bx2), fmaxf(ax1, bx1)));
  const float ih = fmaxf(0.0f, __fsub_rn(fminf(ay2, by2), fmaxf(ay1, by1)));
  const float inter = __fmul_rn(iw, ih);
  const float uni = __fsub_rn(__fadd_rn(aarea, barea), inter);
  return inter > __fmul_rn(thr, uni);
}

__global__ __launch_bounds__(64) void nms_mask_kernel(const NmsArgs a) {
  const int n_items = dyn_n(a.n_dyn, a.n);
  const int item = blockIdx.z;
  if (item >= n_items) return;
  const int cb = blockIdx.x, rb = blockIdx.y;
  int count = a.top_count[item];
  if (count > a.k_cap) count = a.k_cap;
  if (cb < rb || rb * 64 >= count || cb * 64 >= count) return;
  __shared__ float bx[64][5];
  __shared__ int bcls[64];
  const octo_cand* top = a.top + (size_t)item * a.k_cap;
  const int t = threadIdx.x;
  const int j = cb * 64 + t;
  if (j < count) {
    const octo_cand c = top[j];
    bx[t][0] = c.x1; bx[t][1] = c.y1; bx[t][2] = c.x2; bx[t][3] = c.y2;
    bx[t][4] = __fmul_rn(__fsub_rn(c.x2, c.x1), __fsub_rn(c.y2, c.y1));
    bcls[t] = c.cls;
  }
  __syncthreads();
  const int i = rb * 64 + t;
  if (i >= count) return;
  const octo_cand c = top[i];
  const float area = __fmul_rn(__fsub_rn(c.x2, c.x1), __fsub_rn(c.y2, c.y1));
  unsigned long long bits = 0ull;
  const int jn = count - cb * 64 < 64 ? count - cb * 64 : 64;
  for (int q = (cb == rb ? t + 1 : 0); q < jn; ++q) {
    if (bcls[q] == c.cls && suppresses(c.x1, c.y1, c.x2, c.y2, area, bx[q][0], bx[q][1], bx[q][2], bx[q][3], bx[q][4], a.iou_thr))
      bits |= 1ull << q;
  }
  const int nb = a.k_cap / 64;
  a.mask[((size_t)item * a.k_cap + i) * nb + cb] = bits;
}

__global__ __launch_bounds__(64) void nms_reduce_kernel(const NmsArgs a) {
  const int n_items = dyn_n(a.n_dyn, a.n);
  const int lane = threadIdx.x;
  const int nb = a.k_cap / 64;
  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    int count = a.top_count[item];
    if (count > a.k_cap) count = a.k_cap;
    const unsigned long long* mask = a.mask + (size_t)item * a.k_cap * nb;
    int* keep = a.keep + (size_t)item * a.max_det;
    unsigned long long removed = 0ull;   // lane w: word w
    int n_keep = 0;
    const int nblk = (count + 63) / 64;
    for (int blk = 0; blk < nblk && n_keep < a.max_det; ++blk) {
      unsigned long long cur = __shfl(removed, blk);
      const int i = blk * 64 + lane;
      const unsigned long long diag = i < count ? mask[(size_t)i * nb + blk] : 0ull;
      const int valid = count - blk * 64 < 64 ? count - blk * 64 : 64;
      unsigned long long kept = 0ull;
      for (int t = 0; t < valid && n_keep < a.max_det; ++t) {
        const unsigned long long dt = __shfl(diag, t);
        if (!((cur >> t) & 1ull)) {
          kept |= 1ull << t;
          cur |= dt;
          if (lane == 0) keep[n_keep] = blk * 64 + t;
          ++n_keep;
        }
      }
      // fold the rows of the boxes kept in this block into the words of later blocks
      if (lane > blk && lane < nblk) {
        unsigned long long k2 = kept;
        while (k2) {
          const int t = __ffsll((long long)k2) - 1;
          k2 &= k2 - 1;
          removed |= mask[(size_t)(blk * 64 + t) * nb + lane];
        }
      }
    }
    if (lane == 0) a.n_keep[item] = n_keep;
  }
}

size_t nms_mask_bytes(int n, int k_cap) { return (size_t)n * k_cap * (k_cap / 64) * sizeof(unsigned long long); }

hipError_t launch_nms(const NmsArgs& a, hipStream_t s) {
  if (a.n <= 0) return hipSuccess;
  if (a.k_cap % 64 != 0 || a.k_cap > 4096 || a.k_cap <= 0) return hipErrorInvalidValue;
  const int nb = a.k_cap / 64;
  hipLaunchKernelGGL(nms_mask_kernel, dim3(nb, nb, a.n), dim3(64), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(nms_reduce_kernel, dim3(a.n > 2048 ? 2048 : a.n), dim3(64), 0, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// ROI compaction: per edge, an exclusive scan of per-item match counts gives
// every item its first ROI id; items then write their matching boxes in rank
// order.  Workgroup x = edge; the last workgroup writes the final box table.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float to_src(float v, float off, float r, float hi) {
  float s = __fdiv_rn(__fsub_rn(v, off), r);
  return fminf(fmaxf(s, 0.0f), hi);
}

__global__ __launch_bounds__(256) void compact_kernel(const CompactArgs a) {
  __shared__ int s_cnt[256];
  __shared__ int s_base;
  const int n_items = dyn_n(a.n_dyn, a.n);
  const int e = blockIdx.x;
  const int t = threadIdx.x;
  if (e == a.n_edges) {
    // final boxes of every item, in keep order, in source pixels
    for (long long i = t; i < (long long)n_items * a.max_det; i += blockDim.x) {
      const int item = (int)(i / a.max_det), r = (int)(i % a.max_det);
      int nk = a.n_keep[item]; if (nk > a.max_det) nk = a.max_det;
      if (r >= nk) continue;
      const octo_cand c = a.top[(size_t)item * a.k_cap + a.keep[(size_t)item * a.max_det + r]];
      octo_box b;
      b.x1 = to_src(c.x1, a.left, a.rx, a.src_w); b.x2 = to_src(c.x2, a.left, a.rx, a.src_w);
      b.y1 = to_src(c.y1, a.top_pad, a.ry, a.src_h); b.y2 = to_src(c.y2, a.top_pad, a.ry, a.src_h);
      b.score = c.score; b.cls = c.cls;
      for (int k = 0; k < OCTO_MAX_CHILD_LABELS; ++k) b.child_label[k] = -1;
      a.boxes[i] = b;
    }
    return;
  }
  const uint64_t m0 = a.class_mask[e][0], m1 = a.class_mask[e][1];
  if (t == 0) s_base = 0;
  __syncthreads();
  for (int chunk = 0; chunk < n_items; chunk += blockDim.x) {
    const int item = chunk + t;
    int cnt = 0, nk = 0;
    if (item < n_items) {
      nk = a.n_keep[item]; if (nk > a.max_det) nk = a.max_det;
      for (int r = 0; r < nk; ++r) {
        const int cls = a.top[(size_t)item * a.k_cap + a.keep[(size_t)item * a.max_det + r]].cls;
        const bool hit = cls >= 0 && cls < 128 && (((cls < 64 ? m0 : m1) >> (cls & 63)) & 1ull);
        cnt += hit ? 1 : 0;
      }
    }
    s_cnt[t] = cnt;
    __syncthreads();
    // inclusive scan (Hillis-Steele) over the chunk
    for (int off = 1; off < blockDim.x; off <<= 1) {
      int v = t >= off ? s_cnt[t - off] : 0;
      __syncthreads();
      s_cnt[t] += v;
      __syncthreads();
    }
    const int base = s_base + s_cnt[t] - cnt;
    if (item < n_items) {
      int j = base;
      for (int r = 0; r < nk; ++r) {
        const octo_cand c = a.top[(size_t)item * a.k_cap + a.keep[(size_t)item * a.max_det + r]];
        const bool hit = c.cls >= 0 && c.cls < 128 && (((c.cls < 64 ? m0 : m1) >> (c.cls & 63)) & 1ull);
        int id = -1;
        if (hit) {
          if (j < a.roi_cap[e]) {
            octo_roi o;
            o.frame = item; o.rank = r; o.cls = c.cls; o.pad_ = 0;
            o.x1 = to_src(c.x1, a.left, a.rx, a.src_w); o.x2 = to_src(c.x2, a.left, a.rx, a.src_w);
            o.y1 = to_src(c.y1, a.top_pad, a.ry, a.src_h); o.y2 = to_src(c.y2, a.top_pad, a.ry, a.src_h);
            a.rois[e][j] = o;
            id = j;
          } else if (a.flags) {
            atomicOr(a.flags + item, OCTO_FLAG_ROI_OVERFLOW);
          }
          ++j;
        }
        if (a.roi_of[e]) a.roi_of[e][(size_t)item * a.max_det + r] = id;
      }
    }
    __syncthreads();
    if (t == blockDim.x - 1) s_base += s_cnt[t];
    __syncthreads();
  }
  if (t == 0) *a.n_roi[e] = s_base < a.roi_cap[e] ? s_base : a.roi_cap[e];
}

hipError_t launch_compact(const CompactArgs& a, hipStream_t s) {
  if (a.n <= 0) return hipSuccess;
  hipLaunchKernelGGL(compact_kernel, dim3(a.n_edges + (a.boxes ? 1 : 0)), dim3(256), 0, s, a);
  return hipGetLastError();
}

__global__ void scatter_labels_kernel(const LabelArgs a) {
  const long long total = (long long)a.n * a.max_det;
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const int item = (int)(i / a.max_det), r = (int)(i % a.max_det);
    int nk = a.n_keep[item]; if (nk > a.max_det) nk = a.max_det;
    if (r >= nk) continue;
    for (int e = 0; e < a.n_edges && e < OCTO_MAX_CHILD_LABELS; ++e) {
      const int id = a.roi_of[e][i];
      a.boxes[i].child_label[e] = (id >= 0 && id < *a.n_roi[e]) ? a.labels[e][id] : -1;
    }
  }
}

hipError_t launch_scatter_labels(const LabelArgs& a, hipStream_t s) {
  if (a.n <= 0 || a.n_edges <= 0) return hipSuccess;
  long long total = (long long)a.n * a.max_det;
  unsigned g = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL(scatter_labels_kernel, dim3(g > 1024 ? 1024 : g), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace octo
