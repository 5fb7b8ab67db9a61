// HBM-bound glue layers on NHWC tensors: max-pool, nearest 2x upsample, channel
// copy (concatenation fallback), element-wise add, global average pool, argmax.
// Every kernel is a grid-stride loop over (pixel, channel-vector) work items so
// that an item count held in device memory can bound the work.
#include "octo_internal.h"

namespace octo {

template <typename T> __device__ __forceinline__ float ld_f32(const T* p) { return (float)*p; }
template <typename T> __device__ __forceinline__ void st_f32(T* p, float v) { *p = (T)v; }

__device__ __forceinline__ int dyn_items(const int* n_dyn, int n) {
  if (!n_dyn) return n;
  int d = *n_dyn;
  return d < n ? (d < 0 ? 0 : d) : n;
}

static inline unsigned grid_for(long long work, int block) {
  long long g = (work + block - 1) / block;
  if (g < 1) g = 1;
  if (g > 256 * 16) g = 256 * 16;
  return (unsigned)g;
}

// V = channels handled per work item (1, or 16 bytes worth)
template <typename T, int V>
__global__ void maxpool_kernel(const PoolArgs a) {
  const int cv = a.C / V;
  const long long total = (long long)dyn_items(a.n_dyn, a.n) * a.Ho * a.Wo * cv;
  const T* x = (const T*)a.x;
  T* y = (T*)a.y;
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    int c = (int)(i % cv) * V;
    long long pix = i / cv;
    int wo = (int)(pix % a.Wo);
    long long t = pix / a.Wo;
    int ho = (int)(t % a.Ho);
    long long img = t / a.Ho;
    float m[V];
#pragma unroll
    for (int e = 0; e < V; ++e) m[e] = -INFINITY;
    for (int r = 0; r < a.k; ++r) {
      int hi = ho * a.stride - a.pad + r;
      if ((unsigned)hi >= (unsigned)a.H) continue;
      for (int s = 0; s < a.k; ++s) {
        int wi = wo * a.stride - a.pad + s;
        if ((unsigned)wi >= (unsigned)a.W) continue;
        const T* p = x + ((size_t)(img * a.H + hi) * a.W + wi) * a.x_ld + a.x_coff + c;
        alignas(16) T v[V];
        if (V > 1) *(uint4*)v = *(const uint4*)p; else v[0] = *p;
#pragma unroll
        for (int e = 0; e < V; ++e) m[e] = fmaxf(m[e], (float)v[e]);
      }
    }
    alignas(16) T o[V];
#pragma unroll
    for (int e = 0; e < V; ++e) o[e] = (T)m[e];
    T* q = y + (size_t)pix * a.y_ld + a.y_coff + c;
    if (V > 1) *(uint4*)q = *(const uint4*)o; else *q = o[0];
  }
}

// Stride-1 "same" max-pool (window K, padding K / 2: the chained 5x5 pools of a spatial-pyramid block).  A work item
// owns one (image, row segment, column, 16-byte channel vector) and walks down the rows: of every input row it takes
// the maximum over the K columns of its window once and keeps the last K of those row maxima in registers, so an
// output costs K loads instead of K x K.  The row loop is unrolled K times so that the ring of row maxima is indexed
// statically.  Same result as maxpool_kernel: a maximum does not depend on the order it is taken in.
template <typename T, int K>
__global__ __launch_bounds__(256) void maxpool_rows_kernel(const PoolArgs a, int seg_rows, int n_seg) {
  constexpr int V = 16 / (int)sizeof(T), P = K / 2;
  const int cv = a.C / V;
  const long long total = (long long)dyn_items(a.n_dyn, a.n) * n_seg * a.W * cv;
  const T* x = (const T*)a.x;
  T* y = (T*)a.y;
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const int c = (int)(i % cv) * V;
    long long t = i / cv;
    const int wo = (int)(t % a.W); t /= a.W;
    const int seg = (int)(t % n_seg);
    const long long img = t / n_seg;
    const int r0 = seg * seg_rows, r1 = r0 + seg_rows < a.H ? r0 + seg_rows : a.H;
    const int s_lo = wo - P < 0 ? 0 : wo - P, s_hi = wo + P > a.W - 1 ? a.W - 1 : wo + P;
    float ring[K][V];
    // maximum of input row r over this item's window columns (a row outside the image contributes nothing)
    auto row_max = [&](int r, float (&m)[V]) {
#pragma unroll
      for (int e = 0; e < V; ++e) m[e] = -INFINITY;
      if ((unsigned)r >= (unsigned)a.H) return;
      const T* p = x + ((size_t)(img * a.H + r) * a.W) * a.x_ld + a.x_coff + c;
#pragma unroll
      for (int j = 0; j < K; ++j) {
        const int wi = s_lo + j;
        if (wi > s_hi) break;
        alignas(16) T v[V];
        *(uint4*)v = *(const uint4*)(p + (size_t)wi * a.x_ld);
#pragma unroll
        for (int e = 0; e < V; ++e) m[e] = fmaxf(m[e], (float)v[e]);
      }
    };
#pragma unroll
    for (int j = 0; j < K - 1; ++j) row_max(r0 - P + j, ring[j]);
    for (int ho = r0; ho < r1; ho += K) {
#pragma unroll
      for (int j = 0; j < K; ++j) {
        if (ho + j >= r1) break;
        row_max(ho + j + P, ring[(j + K - 1) % K]);        // replaces the row that left the window
        alignas(16) T o[V];
#pragma unroll
        for (int e = 0; e < V; ++e) {
          float m = ring[0][e];
#pragma unroll
          for (int q = 1; q < K; ++q) m = fmaxf(m, ring[q][e]);
          o[e] = (T)m;
        }
        *(uint4*)(y + ((size_t)(img * a.H + ho + j) * a.W + wo) * a.y_ld + a.y_coff + c) = *(const uint4*)o;
      }
    }
  }
}

// mode 0: nearest 2x upsample (y is 2H x 2W); mode 1: plain copy (y is H x W)
template <typename T, int V, int MODE>
__global__ void copy_kernel(const PoolArgs a) {
  const int cv = a.C / V;
  const int Ho = MODE == 0 ? 2 * a.H : a.H, Wo = MODE == 0 ? 2 * a.W : a.W;
  const long long total = (long long)dyn_items(a.n_dyn, a.n) * Ho * Wo * cv;
  const T* x = (const T*)a.x;
  T* y = (T*)a.y;
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    int c = (int)(i % cv) * V;
    long long pix = i / cv;
    int wo = (int)(pix % Wo);
    long long t = pix / Wo;
    int ho = (int)(t % Ho);
    long long img = t / Ho;
    int hi = MODE == 0 ? ho >> 1 : ho, wi = MODE == 0 ? wo >> 1 : wo;
    const T* p = x + ((size_t)(img * a.H + hi) * a.W + wi) * a.x_ld + a.x_coff + c;
    T* q = y + (size_t)pix * a.y_ld + a.y_coff + c;
    if (V > 1) *(uint4*)q = *(const uint4*)p; else *q = *p;
  }
}

template <typename T>
__global__ void add_kernel(const AddArgs a) {
  const long long total = (long long)dyn_items(a.n_dyn, a.n) * a.H * a.W * a.C;
  const T* pa = (const T*)a.a;
  const T* pb = (const T*)a.b;
  T* y = (T*)a.y;
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    int c = (int)(i % a.C);
    long long pix = i / a.C;
    float v = (float)pa[(size_t)pix * a.a_ld + a.a_coff + c] + (float)pb[(size_t)pix * a.b_ld + a.b_coff + c];
    if (a.act == OCTO_ACT_RELU) v = fmaxf(v, 0.0f);
    else if (a.act == OCTO_ACT_SILU) v = v / (1.0f + __expf(-v));
    y[(size_t)pix * a.y_ld + a.y_coff + c] = (T)v;
  }
}

// one thread per (item, channel): channels are contiguous, so a wavefront reads 64 neighbouring channels per pixel
template <typename T>
__global__ void gap_kernel(const PoolArgs a) {
  const long long total = (long long)dyn_items(a.n_dyn, a.n) * a.C;
  const T* x = (const T*)a.x;
  T* y = (T*)a.y;
  const int hw = a.H * a.W;
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    int c = (int)(i % a.C);
    long long img = i / a.C;
    const T* p = x + (size_t)img * hw * a.x_ld + a.x_coff + c;
    float s = 0.0f;
    for (int j = 0; j < hw; ++j) s += (float)p[(size_t)j * a.x_ld];
    y[(size_t)img * a.y_ld + a.y_coff + c] = (T)(s / (float)hw);
  }
}

// one wavefront per row; ties resolve to the lowest index
__global__ void argmax_kernel(const float* logits, int ld, int n_out, const int* n_dyn, int n, int* labels) {
  const int rows = dyn_items(n_dyn, n);
  const int lane = threadIdx.x & 63;
  const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int n_waves = (gridDim.x * blockDim.x) >> 6;
  for (int r = wave; r < rows; r += n_waves) {
    float best = -INFINITY;
    int bi = 0x7fffffff;
    for (int j = lane; j < n_out; j += 64) {
      float v = logits[(size_t)r * ld + j];
      if (v > best || (v == best && j < bi)) { best = v; bi = j; }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      float ob = __shfl_xor(best, off);
      int oi = __shfl_xor(bi, off);
      if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
    }
    if (lane == 0) labels[r] = bi == 0x7fffffff ? 0 : bi;
  }
}

__global__ void fill_i32_kernel(int* p, int value, int count) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < count; i += gridDim.x * blockDim.x) p[i] = value;
}

template <typename T> static bool vec_ok(const void* x, int x_ld, int x_coff, const void* y, int y_ld, int y_coff, int C) {
  constexpr int V = 16 / sizeof(T);
  return C % V == 0 && x_ld % V == 0 && x_coff % V == 0 && y_ld % V == 0 && y_coff % V == 0 &&
         ((uintptr_t)x & 15) == 0 && ((uintptr_t)y & 15) == 0;
}

template <typename T> static hipError_t maxpool_t(const PoolArgs& a, hipStream_t s) {
  constexpr int V = 16 / sizeof(T);
  if (vec_ok<T>(a.x, a.x_ld, a.x_coff, a.y, a.y_ld, a.y_coff, a.C)) {
    // Stride-1 "same" pools with enough columns to give every SIMD a wavefront: the row-walking kernel.  (With fewer
    // its serial walk down the rows is slower than the general kernel's k x k loads per output: 8 x 20 x 20 x 256 took
    // 25 us against 14.)  Row segments: several windows long, since each re-reads k - 1 rows.
    const long long columns = (long long)a.n * a.W * (a.C / V);
    long long n_seg = (262144 + columns - 1) / columns;
    if (n_seg > a.H / (2 * a.k)) n_seg = a.H / (2 * a.k);
    if (n_seg < 1) n_seg = 1;
    if (a.stride == 1 && (a.k == 5 || a.k == 3) && a.pad == a.k / 2 && a.Ho == a.H && a.Wo == a.W && a.H >= 2 * a.k && columns * n_seg >= 65536) {
      const int seg_rows = (int)((a.H + n_seg - 1) / n_seg);
      n_seg = (a.H + seg_rows - 1) / seg_rows;
      const unsigned grid = grid_for(columns * n_seg, 256);
      if (a.k == 5) hipLaunchKernelGGL((maxpool_rows_kernel<T, 5>), dim3(grid), dim3(256), 0, s, a, seg_rows, (int)n_seg);
      else hipLaunchKernelGGL((maxpool_rows_kernel<T, 3>), dim3(grid), dim3(256), 0, s, a, seg_rows, (int)n_seg);
      return hipGetLastError();
    }
    long long work = (long long)a.n * a.Ho * a.Wo * (a.C / V);
    hipLaunchKernelGGL((maxpool_kernel<T, V>), dim3(grid_for(work, 256)), dim3(256), 0, s, a);
  } else {
    long long work = (long long)a.n * a.Ho * a.Wo * a.C;
    hipLaunchKernelGGL((maxpool_kernel<T, 1>), dim3(grid_for(work, 256)), dim3(256), 0, s, a);
  }
  return hipGetLastError();
}
template <typename T, int MODE> static hipError_t copy_t(const PoolArgs& a, hipStream_t s) {
  constexpr int V = 16 / sizeof(T);
  const int mul = MODE == 0 ? 4 : 1;
  if (vec_ok<T>(a.x, a.x_ld, a.x_coff, a.y, a.y_ld, a.y_coff, a.C)) {
    long long work = (long long)a.n * a.H * a.W * mul * (a.C / V);
    hipLaunchKernelGGL((copy_kernel<T, V, MODE>), dim3(grid_for(work, 256)), dim3(256), 0, s, a);
  } else {
    long long work = (long long)a.n * a.H * a.W * mul * a.C;
    hipLaunchKernelGGL((copy_kernel<T, 1, MODE>), dim3(grid_for(work, 256)), dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

#define DISPATCH_T(dtype, EXPR_F32, EXPR_F16, EXPR_BF16) \
  switch (dtype) { case OCTO_F32: return EXPR_F32; case OCTO_F16: return EXPR_F16; case OCTO_BF16: return EXPR_BF16; } \
  return hipErrorInvalidValue;

hipError_t launch_maxpool(int dtype, const PoolArgs& a, hipStream_t s) {
  DISPATCH_T(dtype, maxpool_t<float>(a, s), maxpool_t<_Float16>(a, s), maxpool_t<__bf16>(a, s))
}
hipError_t launch_upsample2x(int dtype, const PoolArgs& a, hipStream_t s) {
  DISPATCH_T(dtype, (copy_t<float, 0>(a, s)), (copy_t<_Float16, 0>(a, s)), (copy_t<__bf16, 0>(a, s)))
}
hipError_t launch_copy_channels(int dtype, const PoolArgs& a, hipStream_t s) {
  DISPATCH_T(dtype, (copy_t<float, 1>(a, s)), (copy_t<_Float16, 1>(a, s)), (copy_t<__bf16, 1>(a, s)))
}
template <typename T> static hipError_t add_t(const AddArgs& a, hipStream_t s) {
  hipLaunchKernelGGL((add_kernel<T>), dim3(grid_for((long long)a.n * a.H * a.W * a.C, 256)), dim3(256), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_add(int dtype, const AddArgs& a, hipStream_t s) {
  DISPATCH_T(dtype, add_t<float>(a, s), add_t<_Float16>(a, s), add_t<__bf16>(a, s))
}
template <typename T> static hipError_t gap_t(const PoolArgs& a, hipStream_t s) {
  hipLaunchKernelGGL((gap_kernel<T>), dim3(grid_for((long long)a.n * a.C, 256)), dim3(256), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_gap(int dtype, const PoolArgs& a, hipStream_t s) {
  DISPATCH_T(dtype, gap_t<float>(a, s), gap_t<_Float16>(a, s), gap_t<__bf16>(a, s))
}
hipError_t launch_argmax(const float* logits, int ld, int n_out, const int* n_dyn, int n, int* labels, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(argmax_kernel, dim3(grid_for((long long)n * 64, 256)), dim3(256), 0, s, logits, ld, n_out, n_dyn, n, labels);
  return hipGetLastError();
}
hipError_t launch_fill_i32(int* p, int value, int count, hipStream_t s) {
  if (count <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_i32_kernel, dim3(grid_for(count, 256)), dim3(256), 0, s, p, value, count);
  return hipGetLastError();
}

}  // namespace octo
