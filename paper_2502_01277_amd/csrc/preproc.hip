// Frame pre-processing: letterbox-resize + normalise (uint8 HWC frame -> NHWC
// tensor of the model's type) and ROI crop-resize (a variable number of source
// boxes -> fixed-size crops).  Both are bilinear with half-pixel centres, taps
// clamped to the frame, no antialias filter, one rounding to the output type.
//
// Each lane produces PX neighbouring output pixels of one row and writes them
// with 8/16-byte stores; a wavefront therefore covers a contiguous output span
// and a contiguous span of each tapped source row.
#include "octo_internal.h"

namespace octo {

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// PX pixels, contiguous; C4: every pixel is written as 4 values (RGB + 0)
template <typename T, int PX, bool C4>
__device__ __forceinline__ void store_pixels(T* dst, const float* v) {
  if (C4) {
    typedef T t4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int p = 0; p < PX; ++p) {
      const t4 o = {(T)v[3 * p], (T)v[3 * p + 1], (T)v[3 * p + 2], (T)0.0f};
      *(t4*)(dst + 4 * p) = o;
    }
  } else if (PX == 4) {
    alignas(16) T o[12];
#pragma unroll
    for (int i = 0; i < 12; ++i) o[i] = (T)v[i];
    if (sizeof(T) == 2) {
      uint2* d = (uint2*)dst; const uint2* s = (const uint2*)o;
      d[0] = s[0]; d[1] = s[1]; d[2] = s[2];
    } else {
      float4* d = (float4*)dst; const float4* s = (const float4*)o;
      d[0] = s[0]; d[1] = s[1]; d[2] = s[2];
    }
  } else {
#pragma unroll
    for (int i = 0; i < 3 * PX; ++i) dst[i] = (T)v[i];
  }
}

// 12 source bytes (4 RGB pixels) starting at pixel ws of a row, fetched with one unaligned 3-dword load
struct __attribute__((packed)) Win12 { uint32_t d0, d1, d2; };
__device__ __forceinline__ Win12 load_window(const uint8_t* row, int ws) {
  Win12 w;
  __builtin_memcpy(&w, row + 3 * ws, 12);
  return w;
}
// the three channels of the pixel that starts at byte `off` (0, 3, 6 or 9) of the window
__device__ __forceinline__ void window_pixel(const Win12& w, int off, float* rgb) {
  const unsigned long long lo = (unsigned long long)w.d0 | ((unsigned long long)w.d1 << 32);
  const unsigned long long hi = (unsigned long long)w.d1 | ((unsigned long long)w.d2 << 32);
  const unsigned v = off < 4 ? (unsigned)(lo >> (8 * off)) : (unsigned)(hi >> (8 * (off - 4)));
  rgb[0] = (float)(v & 0xFFu); rgb[1] = (float)((v >> 8) & 0xFFu); rgb[2] = (float)((v >> 16) & 0xFFu);
}

// Bilinear sample of taps (xa, xb) x (row_a, row_b); xb is xa or xa + 1 (clamping), so both taps of a row come from
// one window.  Needs src_w >= 4.
__device__ __forceinline__ void bilinear_rgb(const uint8_t* row_a, const uint8_t* row_b, int xa, int xb, int src_w, float fx, float fy,
                                             const float* scale, const float* bias, float* out) {
  const int ws = xa < src_w - 4 ? xa : src_w - 4;
  const Win12 wa = load_window(row_a, ws), wb = load_window(row_b, ws);
  float p00[3], p01[3], p10[3], p11[3];
  window_pixel(wa, 3 * (xa - ws), p00); window_pixel(wa, 3 * (xb - ws), p01);
  window_pixel(wb, 3 * (xa - ws), p10); window_pixel(wb, 3 * (xb - ws), p11);
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    float top = (1.0f - fx) * p00[c] + fx * p01[c];
    float bot = (1.0f - fx) * p10[c] + fx * p11[c];
    out[c] = ((1.0f - fy) * top + fy * bot) * scale[c] + bias[c];
  }
}

struct LetterboxGeom { int nw, nh, left, top; };

// EXACT: the source / resized size ratio is an odd integer in both directions, so every output pixel is exactly one
// source pixel (1080p -> 640x360 and 2160p -> 1280x720 are ratio 3): one window load per pixel, no interpolation.
template <typename T, int PX, bool C4, bool EXACT>
__global__ void letterbox_kernel(const ResizeArgs a, const LetterboxGeom g) {
  const int wq = a.dst_w / PX;
  int n_items = a.n;
  if (a.n_dyn) { int d = *a.n_dyn; n_items = d < a.n ? d : a.n; }
  const unsigned total = (unsigned)n_items * (unsigned)a.dst_h * (unsigned)wq;       // < 2^31 (checked by the launcher)
  T* dst = (T*)a.dst;
  const int rx = a.src_w / g.nw, ry = a.src_h / g.nh;      // only meaningful when EXACT
  for (unsigned i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
    const unsigned t = fast_div(i, a.div_wq);
    const int xq = (int)(i - t * (unsigned)wq);
    const int img = (int)fast_div(t, a.div_h);
    const int y = (int)(t - (unsigned)img * (unsigned)a.dst_h);
    float v[3 * PX];
    const int yi = y - g.top;
    const bool row_in = (unsigned)yi < (unsigned)g.nh;
    const uint8_t* base = a.frames[img];
    const size_t pitch = a.pitches[img];
    int ya = 0, yb = 0; float fy = 0.f;
    if (row_in) {
      if (EXACT) {
        ya = yb = ry * yi + (ry - 1) / 2;
      } else {
        // source y = (yi + 0.5) * Hs / nh - 0.5 = ((2 yi + 1) Hs - nh) / (2 nh), split exactly into floor and fraction
        const int num = (2 * yi + 1) * a.src_h - g.nh, den = 2 * g.nh;
        int y0 = num >= 0 ? num / den : -((-num + den - 1) / den);
        fy = (float)(num - y0 * den) / (float)den;
        ya = clampi(y0, 0, a.src_h - 1); yb = clampi(y0 + 1, 0, a.src_h - 1);
      }
    }
#pragma unroll
    for (int px = 0; px < PX; ++px) {
      const int xi = xq * PX + px - g.left;
      if (row_in && (unsigned)xi < (unsigned)g.nw) {
        if (EXACT) {
          const int xs = rx * xi + (rx - 1) / 2;
          const int ws = xs < a.src_w - 4 ? xs : a.src_w - 4;
          float rgb[3];
          window_pixel(load_window(base + (size_t)ya * pitch, ws), 3 * (xs - ws), rgb);
#pragma unroll
          for (int c = 0; c < 3; ++c) v[3 * px + c] = rgb[c] * a.scale[c] + a.bias[c];
        } else {
          const int num = (2 * xi + 1) * a.src_w - g.nw, den = 2 * g.nw;
          int x0 = num >= 0 ? num / den : -((-num + den - 1) / den);
          const float fx = (float)(num - x0 * den) / (float)den;
          const int xa = clampi(x0, 0, a.src_w - 1), xb = clampi(x0 + 1, 0, a.src_w - 1);
          bilinear_rgb(base + (size_t)ya * pitch, base + (size_t)yb * pitch, xa, xb, a.src_w, fx, fy, a.scale, a.bias, v + 3 * px);
        }
      } else {
#pragma unroll
        for (int c = 0; c < 3; ++c) v[3 * px + c] = (float)a.pad_value * a.scale[c] + a.bias[c];
      }
    }
    store_pixels<T, PX, C4>(dst + (((size_t)img * a.dst_h + y) * a.dst_w + (size_t)xq * PX) * (C4 ? 4 : 3), v);
  }
}

template <typename T, int PX, bool C4>
__global__ void crop_resize_kernel(const ResizeArgs a) {
  const int wq = a.dst_w / PX;
  int n_items = a.n;
  if (a.n_dyn) { int d = *a.n_dyn; n_items = d < a.n ? (d < 0 ? 0 : d) : a.n; }
  const unsigned total = (unsigned)n_items * (unsigned)a.dst_h * (unsigned)wq;       // < 2^31 (checked by the launcher)
  T* dst = (T*)a.dst;
  for (unsigned i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
    const unsigned t = fast_div(i, a.div_wq);
    const int xq = (int)(i - t * (unsigned)wq);
    const int roi = (int)fast_div(t, a.div_h);
    const int y = (int)(t - (unsigned)roi * (unsigned)a.dst_h);
    const octo_roi r = a.rois[roi];
    const int fr = clampi(r.frame, 0, a.n_frames - 1);
    const uint8_t* base = a.frames[fr];
    const size_t pitch = a.pitches[fr];
    const float sy = r.y1 + ((float)y + 0.5f) * ((r.y2 - r.y1) / (float)a.dst_h) - 0.5f;
    const float y0f = floorf(sy);
    const float fy = sy - y0f;
    const int ya = clampi((int)y0f, 0, a.src_h - 1), yb = clampi((int)y0f + 1, 0, a.src_h - 1);
    const float step = (r.x2 - r.x1) / (float)a.dst_w;
    float v[3 * PX];
#pragma unroll
    for (int px = 0; px < PX; ++px) {
      const float sx = r.x1 + ((float)(xq * PX + px) + 0.5f) * step - 0.5f;
      const float x0f = floorf(sx);
      const float fx = sx - x0f;
      const int xa = clampi((int)x0f, 0, a.src_w - 1), xb = clampi((int)x0f + 1, 0, a.src_w - 1);
      bilinear_rgb(base + (size_t)ya * pitch, base + (size_t)yb * pitch, xa, xb, a.src_w, fx, fy, a.scale, a.bias, v + 3 * px);
    }
    store_pixels<T, PX, C4>(dst + (((size_t)roi * a.dst_h + y) * a.dst_w + (size_t)xq * PX) * (C4 ? 4 : 3), v);
  }
}

// Crop-resize with the source rows staged in LDS.  One wavefront (a 64-thread workgroup) produces one output row of
// one ROI, 4 pixels per lane.  The two source rows it taps are first copied into LDS - only the span of pixels this
// part of the row needs, with aligned 16-byte loads - and every lane then picks its taps from there.  Sampling
// straight from global memory costs two 12-byte loads at arbitrary addresses per output pixel; for crops that are
// enlarged or mildly reduced (the usual case: objects of 24-360 pixels to 224) neighbouring lanes hit the same few
// cache lines over and over, and the kernel runs at the rate the L1 can look lines up, not at memory bandwidth.
// A span too long for the buffer (strong reduction: taps of neighbouring pixels share no lines anyway) is sampled
// directly, as in the kernel above.  Same arithmetic, so the results are identical.
constexpr int CROP_ROWBUF = 2048;     // bytes of LDS per staged source row

template <typename T, bool C4>
__global__ __launch_bounds__(64) void crop_resize_rows_kernel(const ResizeArgs a) {
  __shared__ __attribute__((aligned(16))) uint8_t srow[2][CROP_ROWBUF];
  const int wq = a.dst_w / 4;
  int n_items = a.n;
  if (a.n_dyn) { int d = *a.n_dyn; n_items = d < a.n ? (d < 0 ? 0 : d) : a.n; }
  const int lane = threadIdx.x;
  T* dst = (T*)a.dst;
  // Workgroup b runs on die b % 8, and each die has its own L2.  The rows of one ROI tap the same source lines again
  // and again (an enlarged crop reads every source row several times), so all rows of ROI r are given to die r % 8:
  // spread over the dies, each of the eight L2s fetched the ROI's pixels from memory for itself.  Within a die the
  // workgroups take consecutive rows, so the rows of one ROI are in flight together.  The grid is a multiple of 8.
  const unsigned die = blockIdx.x & 7u, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
  const unsigned die_rois = (unsigned)n_items > die ? ((unsigned)n_items - die + 7u) >> 3 : 0u;
  const unsigned die_rows = die_rois * (unsigned)a.dst_h;                  // < 2^31 (checked by the launcher)
  for (unsigned row = slot; row < die_rows; row += slots) {
    const unsigned nth = fast_div(row, a.div_h);
    const int roi = (int)(die + 8u * nth);
    const int y = (int)(row - nth * (unsigned)a.dst_h);
    const octo_roi r = a.rois[roi];
    const int fr = clampi(r.frame, 0, a.n_frames - 1);
    const uint8_t* base = a.frames[fr];
    const size_t pitch = a.pitches[fr];
    const float sy = r.y1 + ((float)y + 0.5f) * ((r.y2 - r.y1) / (float)a.dst_h) - 0.5f;
    const float y0f = floorf(sy);
    const float fy = sy - y0f;
    const int ya = clampi((int)y0f, 0, a.src_h - 1), yb = clampi((int)y0f + 1, 0, a.src_h - 1);
    const uint8_t* rowp[2] = {base + (size_t)ya * pitch, base + (size_t)yb * pitch};
    const float step = (r.x2 - r.x1) / (float)a.dst_w;
    for (int xq0 = 0; xq0 < wq; xq0 += 64) {
      // source pixels this chunk of the row taps: the coordinate is monotonic in the output pixel, so the ends bound it
      const int pa = xq0 * 4, pb = (xq0 + 64 < wq ? xq0 + 64 : wq) * 4 - 1;
      const float sa = r.x1 + ((float)pa + 0.5f) * step - 0.5f, sb = r.x1 + ((float)pb + 0.5f) * step - 0.5f;
      const int xlo = clampi((int)floorf(fminf(sa, sb)), 0, a.src_w - 1);
      const int xhi = clampi((int)floorf(fmaxf(sa, sb)) + 1, 0, a.src_w - 1);
      const int span = (xhi - xlo + 1) * 3;
      const bool staged = span > 0 && span + 32 <= CROP_ROWBUF;
      int koff[2] = {0, 0};                // LDS byte index of source pixel x in row rr: koff[rr] + 3 * x
      if (staged) {
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
          const uint8_t* p0 = rowp[rr] + 3 * xlo;
          const uint8_t* a0 = (const uint8_t*)((uintptr_t)p0 & ~(uintptr_t)15);
          const int nvec = (int)((p0 + span - a0 + 15) >> 4);
          const uint8_t* row_end = rowp[rr] + (size_t)a.src_w * 3;
          for (int v = lane; v < nvec; v += 64) {
            const uint8_t* va = a0 + 16 * v;
            uint4 q;
            if (va >= rowp[rr] && va + 16 <= row_end) {
              q = *(const uint4*)va;
            } else {
              // first or last vector of the row: never touch bytes outside the row
              alignas(16) uint8_t b[16];
#pragma unroll
              for (int e = 0; e < 16; ++e) b[e] = (va + e >= rowp[rr] && va + e < row_end) ? va[e] : (uint8_t)0;
              q = *(const uint4*)b;
            }
            *(uint4*)&srow[rr][16 * v] = q;
          }
          koff[rr] = (int)(p0 - a0) - 3 * xlo;
        }
      }
      __syncthreads();
      const int xq = xq0 + lane;
      if (xq < wq) {
        float v[12];
#pragma unroll
        for (int px = 0; px < 4; ++px) {
          const float sx = r.x1 + ((float)(xq * 4 + px) + 0.5f) * step - 0.5f;
          const float x0f = floorf(sx);
          const float fx = sx - x0f;
          const int xa = clampi((int)x0f, 0, a.src_w - 1), xb = clampi((int)x0f + 1, 0, a.src_w - 1);
          if (staged) {
            float t[2][2][3];
#pragma unroll
            for (int rr = 0; rr < 2; ++rr)
#pragma unroll
              for (int tp = 0; tp < 2; ++tp) {
                int k = koff[rr] + 3 * (tp ? xb : xa);
                k = k < 0 ? 0 : (k > CROP_ROWBUF - 8 ? CROP_ROWBUF - 8 : k);      // taps lie inside the span; non-finite boxes must not index outside the buffer
                const uint32_t* w = (const uint32_t*)&srow[rr][k & ~3];
                const unsigned u = (unsigned)((((unsigned long long)w[1] << 32) | w[0]) >> (8 * (k & 3)));
                t[rr][tp][0] = (float)(u & 0xFFu); t[rr][tp][1] = (float)((u >> 8) & 0xFFu); t[rr][tp][2] = (float)((u >> 16) & 0xFFu);
              }
#pragma unroll
            for (int c = 0; c < 3; ++c) {
              float top = (1.0f - fx) * t[0][0][c] + fx * t[0][1][c];
              float bot = (1.0f - fx) * t[1][0][c] + fx * t[1][1][c];
              v[3 * px + c] = ((1.0f - fy) * top + fy * bot) * a.scale[c] + a.bias[c];
            }
          } else {
            bilinear_rgb(rowp[0], rowp[1], xa, xb, a.src_w, fx, fy, a.scale, a.bias, v + 3 * px);
          }
        }
        store_pixels<T, 4, C4>(dst + (((size_t)roi * a.dst_h + y) * a.dst_w + (size_t)xq * 4) * (C4 ? 4 : 3), v);
      }
      __syncthreads();                   // the next chunk overwrites the staged rows
    }
  }
}

static inline unsigned resize_grid(long long work) {
  long long g = (work + 255) / 256;
  if (g < 1) g = 1;
  if (g > 256 * 32) g = 256 * 32;
  return (unsigned)g;
}

static LetterboxGeom letterbox_geom(int src_h, int src_w, int dst_h, int dst_w) {
  // scale r = min(dst_w/src_w, dst_h/src_h); resized size rounded half-up; centred with floor
  double r = (double)dst_w / src_w;
  if ((double)dst_h / src_h < r) r = (double)dst_h / src_h;
  LetterboxGeom g;
  g.nw = (int)(src_w * r + 0.5);
  g.nh = (int)(src_h * r + 0.5);
  if (g.nw < 1) g.nw = 1;
  if (g.nh < 1) g.nh = 1;
  g.left = (dst_w - g.nw) / 2;
  g.top = (dst_h - g.nh) / 2;
  return g;
}

void letterbox_geometry(int src_h, int src_w, int dst_h, int dst_w, int* nw, int* nh, int* left, int* top) {
  LetterboxGeom g = letterbox_geom(src_h, src_w, dst_h, dst_w);
  *nw = g.nw; *nh = g.nh; *left = g.left; *top = g.top;
}

// lanes per output row for the pixel-group width the dispatch below will pick
static bool resize_prepare(ResizeArgs& a) {
  const bool px4 = a.dst_w % 4 == 0 && ((uintptr_t)a.dst & 15) == 0;
  const int wq = px4 ? a.dst_w / 4 : a.dst_w;
  if ((long long)a.n * a.dst_h * wq >= 0x7FFFFFFFLL || a.dst_h < 1 || wq < 1) return false;
  a.div_wq = make_fastdiv((unsigned)wq);
  a.div_h = make_fastdiv((unsigned)a.dst_h);
  return true;
}

template <typename T, bool EXACT> static hipError_t letterbox_e(const ResizeArgs& a, const LetterboxGeom& g, hipStream_t s) {
  if (a.dst_c == 4 && ((uintptr_t)a.dst & 15) == 0 && a.dst_w % 4 == 0) {
    hipLaunchKernelGGL((letterbox_kernel<T, 4, true, EXACT>), dim3(resize_grid((long long)a.n * a.dst_h * (a.dst_w / 4))), dim3(256), 0, s, a, g);
  } else if (a.dst_c == 4) {
    hipLaunchKernelGGL((letterbox_kernel<T, 1, true, EXACT>), dim3(resize_grid((long long)a.n * a.dst_h * a.dst_w)), dim3(256), 0, s, a, g);
  } else if (a.dst_w % 4 == 0 && ((uintptr_t)a.dst & 15) == 0) {
    hipLaunchKernelGGL((letterbox_kernel<T, 4, false, EXACT>), dim3(resize_grid((long long)a.n * a.dst_h * (a.dst_w / 4))), dim3(256), 0, s, a, g);
  } else {
    hipLaunchKernelGGL((letterbox_kernel<T, 1, false, EXACT>), dim3(resize_grid((long long)a.n * a.dst_h * a.dst_w)), dim3(256), 0, s, a, g);
  }
  return hipGetLastError();
}
template <typename T> static hipError_t letterbox_t(const ResizeArgs& a, hipStream_t s) {
  const LetterboxGeom g = letterbox_geom(a.src_h, a.src_w, a.dst_h, a.dst_w);
  const bool exact = a.src_w % g.nw == 0 && a.src_h % g.nh == 0 && ((a.src_w / g.nw) & 1) && ((a.src_h / g.nh) & 1);
  return exact ? letterbox_e<T, true>(a, g, s) : letterbox_e<T, false>(a, g, s);
}
template <typename T> static hipError_t crop_t(const ResizeArgs& a, hipStream_t s) {
  // one 64-thread workgroup per output row, at most 32 per compute unit at a time; each die strides over the rows of
  // its own ROIs (every eighth), so the grid is 8 x the workgroups one die gets
  const long long die_rows = (long long)((a.n + 7) / 8) * a.dst_h;
  const unsigned row_grid = 8u * (unsigned)(die_rows < 32 * 32 ? (die_rows < 1 ? 1 : die_rows) : 32 * 32);
  if (a.dst_c == 4 && ((uintptr_t)a.dst & 15) == 0 && a.dst_w % 4 == 0) {
    hipLaunchKernelGGL((crop_resize_rows_kernel<T, true>), dim3(row_grid), dim3(64), 0, s, a);
  } else if (a.dst_c == 4) {
    hipLaunchKernelGGL((crop_resize_kernel<T, 1, true>), dim3(resize_grid((long long)a.n * a.dst_h * a.dst_w)), dim3(256), 0, s, a);
  } else if (a.dst_w % 4 == 0 && ((uintptr_t)a.dst & 15) == 0) {
    hipLaunchKernelGGL((crop_resize_rows_kernel<T, false>), dim3(row_grid), dim3(64), 0, s, a);
  } else {
    hipLaunchKernelGGL((crop_resize_kernel<T, 1, false>), dim3(resize_grid((long long)a.n * a.dst_h * a.dst_w)), dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

hipError_t launch_letterbox(int dtype, const ResizeArgs& a0, hipStream_t s) {
  if (a0.n <= 0) return hipSuccess;
  ResizeArgs a = a0;
  if ((a.dst_c != 3 && a.dst_c != 4) || a.src_w < 4 || !resize_prepare(a)) return hipErrorInvalidValue;
  switch (dtype) {
    case OCTO_F32: return letterbox_t<float>(a, s);
    case OCTO_F16: return letterbox_t<_Float16>(a, s);
    case OCTO_BF16: return letterbox_t<__bf16>(a, s);
  }
  return hipErrorInvalidValue;
}
hipError_t launch_crop_resize(int dtype, const ResizeArgs& a0, hipStream_t s) {
  if (a0.n <= 0) return hipSuccess;
  ResizeArgs a = a0;
  if ((a.dst_c != 3 && a.dst_c != 4) || a.src_w < 4 || !resize_prepare(a)) return hipErrorInvalidValue;
  switch (dtype) {
    case OCTO_F32: return crop_t<float>(a, s);
    case OCTO_F16: return crop_t<_Float16>(a, s);
    case OCTO_BF16: return crop_t<__bf16>(a, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace octo
