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
      if (lane == leader) base = atomicAdd(&a.count[(size_t)item * a.count_stride], __popcll(m));
      base = __shfl(base, leader);
      if (keep) {
        const int slot = base + __popcll(m & ((1ull << lane) - 1ull));
        if (slot < a.cap) a.cand[(size_t)item * a.cap + slot] = c;
        else if (a.overflow) atomicOr(a.overflow + item, OCTO_FLAG_CAND_OVERFLOW);
      }
    }
  }
}

// Streaming variant: a persistent workgroup walks over chunks of CH consecutive candidates of one level.  The
// contiguous head region of a chunk is fetched with 16-byte buffer loads (every byte of the head is read exactly
// once, fully coalesced) into registers while the previous chunk is being decoded out of LDS, so the memory
// pipeline never drains; each lane then decodes one candidate.  Same arithmetic as decode_kernel.
constexpr int DEC_LDS_BYTES = 48 * 1024;

struct DecChunk {
  int l, level_off, c_first, c_last, cell_lo, item, shift, nvec;
};

template <typename T, int CH>
__global__ __launch_bounds__(CH) void decode_stream_kernel(const DecodeArgs a, int blocks_per_item) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  __shared__ u32x4 lds[DEC_LDS_BYTES / 16];
  __shared__ int s_cnt, s_base;
  constexpr int ES = (int)sizeof(T);
  constexpr int VPT = (DEC_LDS_BYTES / 16 + CH - 1) / CH;      // vectors per lane, upper bound
  const int n_items = dyn_n(a.n_dyn, a.n);
  const int total_work = n_items * blocks_per_item;
  const int A = a.n_anchors, no = 5 + a.n_classes;
  const int lane = threadIdx.x & 63;
  const float z_min = a.score_thr <= 0.0f ? -INFINITY : (a.score_thr >= 1.0f ? INFINITY : __logf(a.score_thr / (1.0f - a.score_thr)) - 0.01f);
  u32x4 regs[VPT];

  // chunk geometry + issue of its loads.  The region is fetched through a buffer descriptor that ends where the
  // tensor (or the region) ends: vectors past the end read as zeros, so the copy needs no per-vector bounds logic.
  auto fetch = [&](int work, DecChunk& ck) {
    ck.item = work / blocks_per_item;
    int rem = work - ck.item * blocks_per_item;
    ck.l = 0; ck.level_off = 0;
    while (true) {
      const int nb = (a.gh[ck.l] * a.gw[ck.l] * A + CH - 1) / CH;
      if (rem < nb) break;
      rem -= nb; ck.level_off += a.gh[ck.l] * a.gw[ck.l] * A; ++ck.l;
    }
    const int ld = a.head_ld[ck.l];
    const int cells = a.gh[ck.l] * a.gw[ck.l];
    const int cand_l = cells * A;
    ck.c_first = rem * CH;
    ck.c_last = (ck.c_first + CH < cand_l ? ck.c_first + CH : cand_l) - 1;
    ck.cell_lo = ck.c_first / A;
    const int cell_hi = ck.c_last / A;
    const long long byte_lo = ((long long)ck.item * cells + ck.cell_lo) * ld * ES;
    const long long byte_hi = (((long long)ck.item * cells + cell_hi) * ld + (long long)A * no) * ES;
    const long long total = (long long)a.n * cells * ld * ES;
    const long long al_lo = byte_lo & ~15LL;
    ck.shift = (int)(byte_lo - al_lo);
    ck.nvec = (int)((byte_hi - al_lo + 15) / 16);
    const long long avail = total - al_lo < byte_hi - al_lo ? total - al_lo : byte_hi - al_lo;
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)a.head[ck.l] + al_lo), 0, (int)avail, 0x00020000);
#pragma unroll
    for (int q = 0; q < VPT; ++q) regs[q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (threadIdx.x + q * CH) * 16, 0, 0);
  };

  DecChunk nxt{};
  int work = blockIdx.x;
  if (work < total_work) fetch(work, nxt);
  while (work < total_work) {
    const DecChunk ck = nxt;
#pragma unroll
    for (int q = 0; q < VPT; ++q) {
      const int v = threadIdx.x + q * CH;
      if (v < ck.nvec) lds[v] = regs[q];
    }
    if (threadIdx.x == 0) s_cnt = 0;
    __syncthreads();
    const int next = work + gridDim.x;
    if (next < total_work) fetch(next, nxt);           // in flight while this chunk is decoded

    const int l = ck.l, ld = a.head_ld[l];
    const int c = ck.c_first + threadIdx.x;
    bool keep = false;
    octo_cand out;
    const int cell = c / A, an = c - cell * A;
    const int t_off = ck.shift + ((cell - ck.cell_lo) * ld + an * no) * ES;    // this lane's logits in LDS
    const T* t = (const T*)((const char*)lds + t_off);
    // objectness logits far below logit(threshold) cannot pass; skipping their sigmoid keeps the common path to one
    // LDS read and one compare (the margin covers fp32 rounding, so the kept set is unchanged)
    float sobj = 0.0f;
    if (c <= ck.c_last) { const float z = (float)t[4]; if (z > z_min) sobj = sigmoidf(z); }
    // score = sobj * s(cls) <= sobj, so only lanes whose objectness passes need their class scanned.  Such lanes are
    // rare; the wavefront scans the classes of each of them together (lane j looks at classes j and j + 64) instead
    // of one lane walking all classes alone.
    const bool pass_obj = c <= ck.c_last && sobj > a.score_thr;
    unsigned long long pend = __ballot(pass_obj);
    float best = 0.0f;
    int cls = 0;
    while (pend) {
      const int src = __ffsll((long long)pend) - 1;
      pend &= pend - 1;
      const T* ts = (const T*)((const char*)lds + __shfl(t_off, src));
      float v = lane < a.n_classes ? (float)ts[5 + lane] : -INFINITY;
      int vi = lane;
      if (lane + 64 < a.n_classes) { const float v2 = (float)ts[5 + lane + 64]; if (v2 > v) { v = v2; vi = lane + 64; } }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(v, off);
        const int oi = __shfl_xor(vi, off);
        if (ov > v || (ov == v && oi < vi)) { v = ov; vi = oi; }
      }
      if (lane == src) { best = v; cls = vi; }
    }
    if (pass_obj) {
      const float score = __fmul_rn(sobj, sigmoidf(best));
      if (score > a.score_thr) {
        const int gy = cell / a.gw[l], gx = cell - gy * a.gw[l];
        const float st = (float)a.stride[l];
        const float sx = sigmoidf((float)t[0]), sy = sigmoidf((float)t[1]);
        const float sw = sigmoidf((float)t[2]), sh = sigmoidf((float)t[3]);
        const float cx = __fmul_rn(__fadd_rn(__fsub_rn(__fmul_rn(2.0f, sx), 0.5f), (float)gx), st);
        const float cy = __fmul_rn(__fadd_rn(__fsub_rn(__fmul_rn(2.0f, sy), 0.5f), (float)gy), st);
        const float tw = __fmul_rn(2.0f, sw), th = __fmul_rn(2.0f, sh);
        const float w = __fmul_rn(__fmul_rn(tw, tw), a.anchors[l][an][0]);
        const float h = __fmul_rn(__fmul_rn(th, th), a.anchors[l][an][1]);
        const float hw = __fmul_rn(w, 0.5f), hh = __fmul_rn(h, 0.5f);
        out.x1 = __fsub_rn(cx, hw); out.y1 = __fsub_rn(cy, hh);
        out.x2 = __fadd_rn(cx, hw); out.y2 = __fadd_rn(cy, hh);
        out.score = score; out.cls = cls; out.idx = ck.level_off + c; out.pad_ = 0;
        keep = true;
      }
    }
    // kept candidates get consecutive slots: wavefront -> workgroup (LDS) -> one global atomic per chunk.  All kept
    // candidates of a frame bump the same counter, and same-address atomics serialise in L2, so they must be few.
    const unsigned long long m = __ballot(keep);
    int wslot = 0;
    if (m) {
      const int leader = __ffsll((long long)m) - 1;
      if (lane == leader) wslot = atomicAdd(&s_cnt, __popcll(m));
      wslot = __shfl(wslot, leader);
    }
    __syncthreads();
    if (threadIdx.x == 0 && s_cnt > 0) s_base = atomicAdd(&a.count[(size_t)ck.item * a.count_stride], s_cnt);
    __syncthreads();          // every lane is done with this chunk's LDS contents; s_base is visible
    if (keep) {
      const int slot = s_base + wslot + __popcll(m & ((1ull << lane) - 1ull));
      if (slot < a.cap) a.cand[(size_t)ck.item * a.cap + slot] = out;
      else if (a.overflow) atomicOr(a.overflow + ck.item, OCTO_FLAG_CAND_OVERFLOW);
    }
    work = next;
  }
}

template <typename T, int CH>
static bool decode_stream_ok(const DecodeArgs& a) {
  for (int l = 0; l < a.n_levels; ++l) {
    const long long region = ((long long)(CH / a.n_anchors + 2) * a.head_ld[l] + a.n_anchors * (5 + a.n_classes)) * sizeof(T) + 32;
    if (region > DEC_LDS_BYTES || ((uintptr_t)a.head[l] & 15)) return false;
  }
  return true;
}

template <typename T, int CH>
static hipError_t decode_t(const DecodeArgs& a, hipStream_t s) {
  int cand = 0, blocks = 0;
  for (int l = 0; l < a.n_levels; ++l) {
    cand += a.gh[l] * a.gw[l] * a.n_anchors;
    blocks += (a.gh[l] * a.gw[l] * a.n_anchors + CH - 1) / CH;
  }
  if (decode_stream_ok<T, CH>(a) && (long long)blocks * a.n < 0x7FFFFFFFLL) {
    const long long want = (long long)blocks * a.n;
    const unsigned grid = (unsigned)(want < 256 * 3 * (256 / CH) ? want : 256 * 3 * (256 / CH));   // persistent: what fits the chip at once
    hipLaunchKernelGGL((decode_stream_kernel<T, CH>), dim3(grid), dim3(CH), 0, s, a, blocks);
  } else {
    const int chunks = (cand + 255) / 256;
    hipLaunchKernelGGL(decode_kernel<T>, dim3(chunks > 1024 ? 1024 : chunks, a.n), dim3(256), 0, s, a, cand);
  }
  return hipGetLastError();
}

hipError_t launch_decode(int dtype, const DecodeArgs& a, hipStream_t s) {
  if (a.n <= 0) return hipSuccess;
  switch (dtype) {
    case OCTO_F32: return decode_t<float, 128>(a, s);
    case OCTO_F16: return decode_t<_Float16, 256>(a, s);
    case OCTO_BF16: return decode_t<__bf16, 256>(a, s);
  }
  return hipErrorInvalidValue;
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
    int count = a.in_count[(size_t)item * a.in_count_stride];
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
      // (four rows per pass, so that their loads are in flight together; a pass with fewer rows left repeats the last)
      if (lane > blk && lane < nblk) {
        unsigned long long k2 = kept;
        const unsigned long long* col = mask + (size_t)blk * 64 * nb + lane;
        while (k2) {
          int t[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            t[q] = k2 ? __ffsll((long long)k2) - 1 : t[q > 0 ? q - 1 : 0];
            k2 &= k2 - 1;                      // 0 stays 0
          }
          const unsigned long long r0 = col[(size_t)t[0] * nb], r1 = col[(size_t)t[1] * nb], r2 = col[(size_t)t[2] * nb], r3 = col[(size_t)t[3] * nb];
          removed |= (r0 | r1) | (r2 | r3);
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

// Step 1, one workgroup per (item, edge) [and one extra grid row for the final box table]: flag the kept boxes whose
// class is routed along the edge, give each its rank among the item's flagged boxes (workgroup scan) and leave the
// item's count in roi_cnt.  Step 2, same grid: the item's first ROI id is the sum of the counts of the items before
// it; every flagged box is written to that id + its rank.  Both steps are a few microseconds; the order of the ROI
// table is (item, rank), exactly that of a serial walk.
__global__ __launch_bounds__(256) void compact_count_kernel(const CompactArgs a) {
  __shared__ int s_wave[4];
  __shared__ int s_run;
  const int n_items = dyn_n(a.n_dyn, a.n);
  const int item = blockIdx.x, e = blockIdx.y;
  if (item >= n_items) return;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  int nk = a.n_keep[item]; if (nk > a.max_det) nk = a.max_det;
  if (e == a.n_edges) {
    // final boxes of the item, in keep order, in source pixels
    for (int r = t; r < nk; r += blockDim.x) {
      const octo_cand c = a.top[(size_t)item * a.k_cap + a.keep[(size_t)item * a.max_det + r]];
      octo_box b;
      b.x1 = to_src(c.x1, a.left, a.rx, a.src_w); b.x2 = to_src(c.x2, a.left, a.rx, a.src_w);
      b.y1 = to_src(c.y1, a.top_pad, a.ry, a.src_h); b.y2 = to_src(c.y2, a.top_pad, a.ry, a.src_h);
      b.score = c.score; b.cls = c.cls;
      for (int k = 0; k < OCTO_MAX_CHILD_LABELS; ++k) b.child_label[k] = -1;
      a.boxes[(size_t)item * a.max_det + r] = b;
    }
    return;
  }
  const uint64_t m0 = a.class_mask[e][0], m1 = a.class_mask[e][1];
  if (t == 0) s_run = 0;
  __syncthreads();
  for (int r0 = 0; r0 < nk; r0 += blockDim.x) {
    const int r = r0 + t;
    bool hit = false;
    if (r < nk) {
      const int cls = a.top[(size_t)item * a.k_cap + a.keep[(size_t)item * a.max_det + r]].cls;
      hit = cls >= 0 && cls < 128 && (((cls < 64 ? m0 : m1) >> (cls & 63)) & 1ull);
    }
    const unsigned long long bal = __ballot(hit);
    if (lane == 0) s_wave[wave] = __popcll(bal);
    __syncthreads();
    int before = s_run;
    for (int w = 0; w < wave; ++w) before += s_wave[w];
    const int rank = before + __popcll(bal & ((1ull << lane) - 1ull));
    if (r < nk) a.roi_of[e][(size_t)item * a.max_det + r] = hit ? rank : -1;      // rank inside the item for now
    __syncthreads();
    if (t == 0) s_run += s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
    __syncthreads();
  }
  if (t == 0) a.roi_cnt[e][item] = s_run;
}

__global__ __launch_bounds__(256) void compact_write_kernel(const CompactArgs a) {
  __shared__ int s_part[256];
  const int n_items = dyn_n(a.n_dyn, a.n);
  const int item = blockIdx.x, e = blockIdx.y;
  if (item >= n_items) return;
  const int t = threadIdx.x;
  // ROIs of all earlier items (and, in the last workgroup, the total)
  int part = 0, tot = 0;
  for (int f = t; f < n_items; f += blockDim.x) { const int c = a.roi_cnt[e][f]; tot += c; if (f < item) part += c; }
  s_part[t] = part;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) { if (t < off) s_part[t] += s_part[t + off]; __syncthreads(); }
  const int base = s_part[0];
  __syncthreads();
  if (item == n_items - 1) {
    s_part[t] = tot;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) { if (t < off) s_part[t] += s_part[t + off]; __syncthreads(); }
    if (t == 0) *a.n_roi[e] = s_part[0] < a.roi_cap[e] ? s_part[0] : a.roi_cap[e];
  }
  int nk = a.n_keep[item]; if (nk > a.max_det) nk = a.max_det;
  for (int r = t; r < nk; r += blockDim.x) {
    const int local = a.roi_of[e][(size_t)item * a.max_det + r];
    if (local < 0) continue;
    const int j = base + local;
    int id = -1;
    if (j < a.roi_cap[e]) {
      const octo_cand c = a.top[(size_t)item * a.k_cap + a.keep[(size_t)item * a.max_det + r]];
      octo_roi o;
      o.frame = item; o.rank = r; o.cls = c.cls; o.pad_ = 0;
      o.x1 = to_src(c.x1, a.left, a.rx, a.src_w); o.x2 = to_src(c.x2, a.left, a.rx, a.src_w);
      o.y1 = to_src(c.y1, a.top_pad, a.ry, a.src_h); o.y2 = to_src(c.y2, a.top_pad, a.ry, a.src_h);
      a.rois[e][j] = o;
      id = j;
    } else if (a.flags) {
      atomicOr(a.flags + item, OCTO_FLAG_ROI_OVERFLOW);
    }
    a.roi_of[e][(size_t)item * a.max_det + r] = id;
  }
}

hipError_t launch_compact(const CompactArgs& a, hipStream_t s) {
  if (a.n <= 0) return hipSuccess;
  if (a.n > 65535) return hipErrorInvalidValue;
  for (int e = 0; e < a.n_edges; ++e) if (!a.roi_of[e] || !a.roi_cnt[e]) return hipErrorInvalidValue;
  hipLaunchKernelGGL(compact_count_kernel, dim3(a.n, a.n_edges + (a.boxes ? 1 : 0)), dim3(256), 0, s, a);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess || a.n_edges == 0) return err;
  hipLaunchKernelGGL(compact_write_kernel, dim3(a.n, a.n_edges), dim3(256), 0, s, a);
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
