// Convolution as an implicit GEMM on the CDNA4 matrix cores.
//
//   y[n,p,q,k] = act(bias[k] + sum_{r,s,c} x[n, p*stride + r - pad, q*stride + s - pad, c] * w[k,r,s,c]  (+ residual))
//
// GEMM view: rows = output channels (weights, [Cout][K] with K = kh*kw*Cin contiguous),
// columns = output pixels (gathered on the fly from the NHWC input), reduction = K.
// One workgroup = 4 wavefronts (256 lanes) computes a BC x BP tile with
// v_mfma_f32_32x32x16 (fp16 / bf16) or v_mfma_f32_32x32x2 (fp32); both operands go
// global -> registers -> LDS (double buffered, one barrier per K step) and every
// lane feeds the MFMA with 16-byte LDS reads.  The grid is persistent: workgroups
// stride over the tile list, whose length may depend on an item count that lives
// in device memory (a variable number of ROIs), so no host round trip is needed.
#include "octo_internal.h"

namespace octo {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

struct alignas(16) Vec16 { uint32_t v[4]; };

template <typename T> struct Elem;
template <> struct Elem<_Float16> {
  static constexpr int N = 8;   // elements per 16-byte vector
  static __device__ __forceinline__ void mfma(const Vec16& a, const Vec16& b, floatx16& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_f16(*(const half8*)&a, *(const half8*)&b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ float to_f32(_Float16 v) { return (float)v; }
  static __device__ __forceinline__ _Float16 from_f32(float v) { return (_Float16)v; }
};
template <> struct Elem<__bf16> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void mfma(const Vec16& a, const Vec16& b, floatx16& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)&a, *(const bf16x8*)&b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ float to_f32(__bf16 v) { return (float)v; }
  static __device__ __forceinline__ __bf16 from_f32(float v) { return (__bf16)v; }
};
template <> struct Elem<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void mfma(const Vec16& a, const Vec16& b, floatx16& c) {
    const float* fa = (const float*)&a;
    const float* fb = (const float*)&b;
#pragma unroll
    for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[j], fb[j], c, 0, 0, 0);
  }
  static __device__ __forceinline__ float to_f32(float v) { return v; }
  static __device__ __forceinline__ float from_f32(float v) { return v; }
};

__device__ __forceinline__ float apply_act(float v, int act) {
  if (act == OCTO_ACT_RELU) return fmaxf(v, 0.0f);
  if (act == OCTO_ACT_SILU) return v / (1.0f + __expf(-v));
  return v;
}

constexpr int KVEC = 4;                 // 16-byte vectors per tile row along K (one K step = 64 bytes per row)
constexpr int ROWV = KVEC + 1;          // LDS row pitch in vectors (80 bytes: conflict-free 16-byte reads)
constexpr int THREADS = 256;

// BC: output channels per tile, BP: pixels per tile, WC x WP: wavefront grid (WC * WP == 4).
template <typename T, int BC, int BP, int WC, int WP, bool VEC>
__global__ __launch_bounds__(THREADS) void conv_mfma_kernel(const ConvArgs a) {
  using E = Elem<T>;
  constexpr int VN = E::N;
  constexpr int BK = KVEC * VN;          // elements per K step
  constexpr int TC = BC / WC / 32;       // 32x32 blocks per wavefront along channels
  constexpr int TP = BP / WP / 32;
  constexpr int LA = (BC * KVEC + THREADS - 1) / THREADS;  // vectors per thread per K step (weights)
  constexpr int LB = BP * KVEC / THREADS;                  // (pixels)
  static_assert(WC * WP == 4 && TC >= 1 && TP >= 1 && LB >= 1 && BP % 64 == 0 && BC % 32 == 0, "tile shape");

  __shared__ Vec16 sA[2][BC][ROWV];
  __shared__ Vec16 sB[2][BP][ROWV];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wc = wave % WC, wp = wave / WC;
  const int l32 = lane & 31, g = lane >> 5;

  int n_items = a.n;
  if (a.n_dyn) { int d = *a.n_dyn; n_items = d < a.n ? d : a.n; }
  const long long M = (long long)n_items * a.Ho * a.Wo;
  const int tiles_c = (a.Cout + BC - 1) / BC;
  const long long tiles_p = (M + BP - 1) / BP;
  const long long n_tiles = tiles_p * tiles_c;
  const int nk = a.Kp / BK;
  const T* __restrict__ xg = (const T*)a.x;
  const T* __restrict__ wg = (const T*)a.w;

  const int ld_row = tid >> 2;           // 0..63
  const int ld_kv = tid & 3;

  for (long long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const int tc = (int)(tile % tiles_c);
    const long long tp = tile / tiles_c;
    const int c0 = tc * BC;
    const long long p0 = tp * BP;

    // per-thread pixel rows for the gather
    int hi0[LB], wi0[LB];
    long long pixbase[LB];
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      long long m = p0 + ld_row + 64 * i;
      if (m < M) {
        int img = (int)(m / (a.Ho * a.Wo));
        int rem = (int)(m - (long long)img * (a.Ho * a.Wo));
        int ho = rem / a.Wo, wo = rem - ho * a.Wo;
        hi0[i] = ho * a.stride - a.pad;
        wi0[i] = wo * a.stride - a.pad;
        pixbase[i] = (long long)img * a.H * a.W;
      } else {
        hi0[i] = -1000000; wi0[i] = 0; pixbase[i] = 0;
      }
    }
    // this thread's position along K: element k = kb*BK + ld_kv*VN -> (tap r, s; channel c)
    int kc = ld_kv * VN, kr = 0, ks = 0;
    if (VEC) { while (kc >= a.Cin) { kc -= a.Cin; if (++ks == a.kw) { ks = 0; ++kr; } } }

    floatx16 acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; ++i)
#pragma unroll
      for (int j = 0; j < TP; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    Vec16 ra[LA], rb[LB];
    auto load_tiles = [&](int kb) {
#pragma unroll
      for (int i = 0; i < LA; ++i) {
        if (BC % 64 == 0 || ld_row + 64 * i < BC) {
          const T* src = wg + (size_t)(c0 + ld_row + 64 * i) * a.Kp + (size_t)kb * BK + ld_kv * VN;
          ra[i] = *(const Vec16*)src;
        }
      }
      if (VEC) {
#pragma unroll
        for (int i = 0; i < LB; ++i) {
          int hi = hi0[i] + kr, wi = wi0[i] + ks;
          Vec16 v = {{0u, 0u, 0u, 0u}};
          if (kr < a.kh && (unsigned)hi < (unsigned)a.H && (unsigned)wi < (unsigned)a.W) {
            const T* src = xg + ((size_t)(pixbase[i] + (long long)hi * a.W + wi)) * a.x_ld + a.x_coff + kc;
            v = *(const Vec16*)src;
          }
          rb[i] = v;
        }
        kc += BK;
        while (kc >= a.Cin) { kc -= a.Cin; if (++ks == a.kw) { ks = 0; ++kr; } }
      } else {
        const int kbase = kb * BK + ld_kv * VN;
#pragma unroll
        for (int i = 0; i < LB; ++i) {
          alignas(16) T tmp[VN];
#pragma unroll
          for (int e = 0; e < VN; ++e) {
            int k = kbase + e;
            float val = 0.0f;
            if (k < a.K) {
              int tap = k / a.Cin, c = k - tap * a.Cin;
              int r = tap / a.kw, s = tap - r * a.kw;
              int hi = hi0[i] + r, wi = wi0[i] + s;
              if ((unsigned)hi < (unsigned)a.H && (unsigned)wi < (unsigned)a.W)
                val = E::to_f32(xg[((size_t)(pixbase[i] + (long long)hi * a.W + wi)) * a.x_ld + a.x_coff + c]);
            }
            tmp[e] = E::from_f32(val);
          }
          rb[i] = *(const Vec16*)tmp;
        }
      }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
      for (int i = 0; i < LA; ++i)
        if (BC % 64 == 0 || ld_row + 64 * i < BC) sA[buf][ld_row + 64 * i][ld_kv] = ra[i];
#pragma unroll
      for (int i = 0; i < LB; ++i) sB[buf][ld_row + 64 * i][ld_kv] = rb[i];
    };

    __syncthreads();   // previous tile's LDS reads are done
    load_tiles(0);
    store_tiles(0);
    __syncthreads();
    for (int kb = 0; kb < nk; ++kb) {
      const int buf = kb & 1;
      if (kb + 1 < nk) load_tiles(kb + 1);
#pragma unroll
      for (int kk = 0; kk < KVEC / 2; ++kk) {
        Vec16 fa[TC], fb[TP];
#pragma unroll
        for (int i = 0; i < TC; ++i) fa[i] = sA[buf][wc * (BC / WC) + i * 32 + l32][kk * 2 + g];
#pragma unroll
        for (int j = 0; j < TP; ++j) fb[j] = sB[buf][wp * (BP / WP) + j * 32 + l32][kk * 2 + g];
#pragma unroll
        for (int i = 0; i < TC; ++i)
#pragma unroll
          for (int j = 0; j < TP; ++j) E::mfma(fa[i], fb[j], acc[i][j]);
      }
      if (kb + 1 < nk) store_tiles(buf ^ 1);
      __syncthreads();
    }

    // epilogue: lane holds pixel column l32 of each 32x32 block and 4 groups of 4 consecutive channels
    const bool vec_ok = ((a.y_ld | a.y_coff) & 3) == 0 && (!a.res || ((a.res_ld | a.res_coff) & 3) == 0);
#pragma unroll
    for (int j = 0; j < TP; ++j) {
      const long long p = p0 + wp * (BP / WP) + j * 32 + l32;
      if (p >= M) continue;
#pragma unroll
      for (int i = 0; i < TC; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int cb = c0 + wc * (BC / WC) + i * 32 + q * 8 + g * 4;
          if (cb >= a.Cout) continue;
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[i][j][q * 4 + e];
          const int nvalid = a.Cout - cb < 4 ? a.Cout - cb : 4;
#pragma unroll
          for (int e = 0; e < 4; ++e) if (e < nvalid) v[e] += a.bias[cb + e];
          float rv[4] = {0.f, 0.f, 0.f, 0.f};
          if (a.res) {
            const T* rp = (const T*)a.res + (size_t)p * a.res_ld + a.res_coff + cb;
#pragma unroll
            for (int e = 0; e < 4; ++e) if (e < nvalid) rv[e] = E::to_f32(rp[e]);
          }
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if (a.res_mode == OCTO_RES_BEFORE_ACT) v[e] = apply_act(v[e] + rv[e], a.act);
            else if (a.res_mode == OCTO_RES_AFTER_ACT) v[e] = apply_act(v[e], a.act) + rv[e];
            else v[e] = apply_act(v[e], a.act);
          }
          if (a.out_f32) {
            float* yp = (float*)a.y + (size_t)p * a.y_ld + a.y_coff + cb;
            if (vec_ok && nvalid == 4) *(floatx4*)yp = floatx4{v[0], v[1], v[2], v[3]};
            else { for (int e = 0; e < nvalid; ++e) yp[e] = v[e]; }
          } else {
            T* yp = (T*)a.y + (size_t)p * a.y_ld + a.y_coff + cb;
            if (vec_ok && nvalid == 4) {
              alignas(16) T o[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) o[e] = E::from_f32(v[e]);
              if (sizeof(T) == 2) *(uint2*)yp = *(const uint2*)o;
              else *(floatx4*)yp = *(const floatx4*)o;
            } else {
              for (int e = 0; e < nvalid; ++e) yp[e] = E::from_f32(v[e]);
            }
          }
        }
      }
    }
  }
}

size_t conv_packed_weight_elems(int cout, int kh, int kw, int cin, int dtype, int* kp_out, int* cout_pad_out) {
  const int vn = dtype == OCTO_F32 ? 4 : 8;
  const int bk = KVEC * vn;
  const int K = kh * kw * cin;
  const int kp = (K + bk - 1) / bk * bk;
  const int cp = (cout + 127) / 128 * 128;
  if (kp_out) *kp_out = kp;
  if (cout_pad_out) *cout_pad_out = cp;
  return (size_t)kp * cp;
}

template <typename T, int BC, int BP, int WC, int WP>
static hipError_t launch_cfg(const ConvArgs& a, bool vec, int num_cu, hipStream_t s) {
  const long long M = (long long)a.n * a.Ho * a.Wo;
  const long long tiles = ((M + BP - 1) / BP) * ((a.Cout + BC - 1) / BC);
  if (tiles <= 0) return hipSuccess;
  long long grid = tiles;
  const long long cap = (long long)num_cu * 2;      // two resident workgroups per CU (LDS / register bound)
  if (grid > cap) grid = cap;
  if (vec) hipLaunchKernelGGL((conv_mfma_kernel<T, BC, BP, WC, WP, true>), dim3((unsigned)grid), dim3(THREADS), 0, s, a);
  else hipLaunchKernelGGL((conv_mfma_kernel<T, BC, BP, WC, WP, false>), dim3((unsigned)grid), dim3(THREADS), 0, s, a);
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_typed(const ConvArgs& a, int num_cu, hipStream_t s) {
  constexpr int VN = Elem<T>::N;
  const bool vec = (a.Cin % VN == 0) && (a.x_ld % VN == 0) && (a.x_coff % VN == 0) && (((uintptr_t)a.x & 15) == 0);
  const long long M = (long long)a.n * a.Ho * a.Wo;
  // Tile choice: wide channel tiles only when there are enough channels; fall back to smaller pixel tiles when
  // the layer has too few tiles to occupy every CU.
  if (a.Cout <= 32) return launch_cfg<T, 32, 128, 1, 4>(a, vec, num_cu, s);
  if (a.Cout <= 64) {
    return launch_cfg<T, 64, 128, 2, 2>(a, vec, num_cu, s);
  }
  const long long t128 = ((M + 127) / 128) * ((a.Cout + 127) / 128);
  if (t128 >= 2LL * num_cu) return launch_cfg<T, 128, 128, 2, 2>(a, vec, num_cu, s);
  return launch_cfg<T, 64, 64, 2, 2>(a, vec, num_cu, s);
}

hipError_t launch_conv(int dtype, const ConvArgs& a, int num_cu, hipStream_t s) {
  switch (dtype) {
    case OCTO_F16: return launch_typed<_Float16>(a, num_cu, s);
    case OCTO_BF16: return launch_typed<__bf16>(a, num_cu, s);
    case OCTO_F32: return launch_typed<float>(a, num_cu, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace octo
