// Two microbenchmarks behind the C ABI: what this GPU actually sustains for a plain streaming copy and for a
// register-only MFMA loop.  bench.py reports kernel throughput against these measured figures beside the datasheet
// peaks (a matrix-core loop with realistic operand values is clock-limited well below the datasheet rate).
#include <type_traits>
#include <vector>
#include <algorithm>

#include "octo_internal.h"
#include "mfma_common.h"

namespace octo {
namespace {

__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n_vec) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

__device__ __forceinline__ unsigned mix(unsigned x) { x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16; return x; }

// 16 independent 32x32 accumulators per wavefront (as in the convolution's largest tile), operands in registers with
// random signs and mantissas and exponents of 0.5..2: nothing but MFMA issue, at realistic operand toggling.
template <typename T>
__global__ __launch_bounds__(256, 1) void probe_mfma_kernel(float* out, int iters) {
  u32x4 a[4], b[4];
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) {
      const unsigned h1 = mix(threadIdx.x * 64 + i * 8 + j + blockIdx.x * 7919), h2 = mix(h1 + 12345);
      if constexpr (std::is_same<T, f8>::value) {
        a[i][j] = (h1 & 0x87878787u) | 0x38383838u; b[i][j] = (h2 & 0x87878787u) | 0x38383838u;      // four E4M3 per word, 1..1.875
      } else if constexpr (std::is_same<T, __bf16>::value) {
        a[i][j] = (h1 & 0x80FF80FFu) | 0x3F003F00u; b[i][j] = (h2 & 0x80FF80FFu) | 0x3F003F00u;      // two bf16 per word
      } else {
        a[i][j] = (h1 & 0x87FF87FFu) | 0x38003800u; b[i][j] = (h2 & 0x87FF87FFu) | 0x38003800u;      // two fp16 per word
      }
    }
  floatx16 c[4][4];
  for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) for (int r = 0; r < 16; ++r) c[i][j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if constexpr (std::is_same<T, f8>::value) c[i][j] = Elem<T>::mfma2(a[i], a[(i + 1) & 3], b[j], b[(j + 1) & 3], c[i][j]);   // K = 64 per instruction
        else c[i][j] = Elem<T>::mfma(a[i], b[j], c[i][j]);
      }
  }
  float s = 0.f;
  for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) for (int r = 0; r < 16; ++r) s += c[i][j][r];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

float median_ms(std::vector<float>& v) { std::sort(v.begin(), v.end()); return v[v.size() / 2]; }

}  // namespace
}  // namespace octo

using namespace octo;

extern "C" {

octo_status octo_probe_copy(const void* d_src, void* d_dst, size_t bytes, int32_t reps, void* hip_stream, double* gb_per_s) {
  if (!d_src || !d_dst || !gb_per_s || bytes < 16 || reps < 1 || reps > 1000 || (((uintptr_t)d_src | (uintptr_t)d_dst) & 15)) return OCTO_EINVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  int dev = 0; hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return OCTO_EHIP;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return OCTO_EHIP;
  if (hipEventCreate(&e1) != hipSuccess) { hipEventDestroy(e0); return OCTO_EHIP; }
  const size_t n_vec = bytes / 16;
  const unsigned grid = (unsigned)std::min<size_t>((n_vec + 255) / 256, (size_t)prop.multiProcessorCount * 16);
  std::vector<float> t;
  octo_status st = OCTO_OK;
  for (int r = 0; r < reps + 1 && st == OCTO_OK; ++r) {      // the first pass is a warm-up
    hipEventRecord(e0, s);
    hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(256), 0, s, (const u32x4*)d_src, (u32x4*)d_dst, n_vec);
    hipEventRecord(e1, s);
    float ms = 0.f;
    if (hipGetLastError() != hipSuccess || hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) st = OCTO_EHIP;
    else if (r > 0) t.push_back(ms);
  }
  hipEventDestroy(e0); hipEventDestroy(e1);
  if (st != OCTO_OK) return st;
  *gb_per_s = 2.0 * (double)(n_vec * 16) / (median_ms(t) * 1e-3) / 1e9;      // bytes read + bytes written
  return OCTO_OK;
}

octo_status octo_probe_mfma(int32_t dtype, float* d_scratch, size_t scratch_bytes, int32_t iters, int32_t reps, void* hip_stream, double* tflops) {
  if (!d_scratch || !tflops || iters < 1 || iters > 1000000 || reps < 1 || reps > 100 || (dtype != OCTO_F16 && dtype != OCTO_BF16 && dtype != OCTO_F8)) return OCTO_EINVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  int dev = 0; hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return OCTO_EHIP;
  const unsigned grid = (unsigned)prop.multiProcessorCount;
  if (scratch_bytes < (size_t)grid * 256 * sizeof(float)) return OCTO_EINVAL;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return OCTO_EHIP;
  if (hipEventCreate(&e1) != hipSuccess) { hipEventDestroy(e0); return OCTO_EHIP; }
  std::vector<float> t;
  octo_status st = OCTO_OK;
  for (int r = 0; r < reps + 1 && st == OCTO_OK; ++r) {
    hipEventRecord(e0, s);
    if (dtype == OCTO_F8) hipLaunchKernelGGL(probe_mfma_kernel<f8>, dim3(grid), dim3(256), 0, s, d_scratch, iters);
    else if (dtype == OCTO_F16) hipLaunchKernelGGL(probe_mfma_kernel<_Float16>, dim3(grid), dim3(256), 0, s, d_scratch, iters);
    else hipLaunchKernelGGL(probe_mfma_kernel<__bf16>, dim3(grid), dim3(256), 0, s, d_scratch, iters);
    hipEventRecord(e1, s);
    float ms = 0.f;
    if (hipGetLastError() != hipSuccess || hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) st = OCTO_EHIP;
    else if (r > 0) t.push_back(ms);
  }
  hipEventDestroy(e0); hipEventDestroy(e1);
  if (st != OCTO_OK) return st;
  const double flop = (double)grid * 4.0 * iters * 16.0 * (2.0 * 32 * 32 * (dtype == OCTO_F8 ? 64 : 16));
  *tflops = flop / (median_ms(t) * 1e-3) / 1e12;
  return OCTO_OK;
}

}  // extern "C"
