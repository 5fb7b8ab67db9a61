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
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte operand vector
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename T> struct Elem;
template <> struct Elem<_Float16> {
  static constexpr int N = 8;   // elements per 16-byte vector
  static __device__ __forceinline__ floatx16 mfma(u32x4 a, u32x4 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
  }
};
template <> struct Elem<__bf16> {
  static constexpr int N = 8;
  static __device__ __forceinline__ floatx16 mfma(u32x4 a, u32x4 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};
template <> struct Elem<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ floatx16 mfma(u32x4 a, u32x4 b, floatx16 c) {
    const floatx4 fa = __builtin_bit_cast(floatx4, a), fb = __builtin_bit_cast(floatx4, b);
#pragma unroll
    for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[j], fb[j], c, 0, 0, 0);
    return c;
  }
};

// four consecutive output values: residual, activation, conversion and one 8/16-byte store
template <typename T>
__device__ __forceinline__ floatx4 load4(const T* p) {
  if constexpr (sizeof(T) == 4) {
    return *(const floatx4*)p;
  } else {
    typedef T t4 __attribute__((ext_vector_type(4)));
    const t4 v = __builtin_bit_cast(t4, *(const u32x2*)p);
    return floatx4{(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
  }
}
template <typename T>
__device__ __forceinline__ void store4(T* p, floatx4 v) {
  if constexpr (sizeof(T) == 4) {
    *(floatx4*)p = v;
  } else {
    typedef T t4 __attribute__((ext_vector_type(4)));
    const t4 o = {(T)v[0], (T)v[1], (T)v[2], (T)v[3]};
    *(u32x2*)p = __builtin_bit_cast(u32x2, o);
  }
}
__device__ __forceinline__ float silu(float v) { return v / (1.0f + __expf(-v)); }

constexpr int THREADS = 256;

// BC: output channels per tile, BP: pixels per tile, WC x WP: wavefront grid (WC * WP == 4),
// KV: 16-byte vectors per tile row and K step (one K step = KV*16 bytes of K per row).
template <typename T, int BC, int BP, int WC, int WP, int KV, bool VEC>
__global__ __launch_bounds__(THREADS) void conv_mfma_kernel(const ConvArgs a) {
  using E = Elem<T>;
  constexpr int VN = E::N;
  constexpr int BK = KV * VN;            // elements per K step
  constexpr int ROWV = KV + 1;           // LDS row pitch in vectors: (16*KV + 16) bytes keeps 16-byte reads conflict-free
  constexpr int RP = THREADS / KV;       // tile rows covered by one pass of the 256 loader lanes
  constexpr int TC = BC / WC / 32;       // 32x32 blocks per wavefront along channels
  constexpr int TP = BP / WP / 32;
  constexpr int LA = (BC + RP - 1) / RP; // vectors per lane per K step (weights)
  constexpr int LB = BP / RP;            // (pixels)
  static_assert(WC * WP == 4 && TC >= 1 && TP >= 1 && LB >= 1 && BP % RP == 0 && BC % 32 == 0, "tile shape");

  __shared__ u32x4 sA[2][BC][ROWV];
  __shared__ u32x4 sB[2][BP][ROWV];
  __shared__ float sBias[BC];

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
  const T* __restrict__ xg = (const T*)a.x + a.x_coff;
  const T* __restrict__ wg = (const T*)a.w;
  const int HoWo = a.Ho * a.Wo;

  const int ld_row = tid / KV;
  const int ld_kv = tid % KV;
  const bool vec_ok = ((a.y_ld | a.y_coff) & 3) == 0 && (!a.res || ((a.res_ld | a.res_coff) & 3) == 0);
  const bool is_silu = a.act == OCTO_ACT_SILU;
  const float act_lo = a.act == OCTO_ACT_RELU ? 0.0f : -INFINITY;
  const float res_pre = a.res_mode == OCTO_RES_BEFORE_ACT ? 1.0f : 0.0f;
  const float res_post = a.res_mode == OCTO_RES_AFTER_ACT ? 1.0f : 0.0f;

  for (long long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const int tc = (int)(tile % tiles_c);
    const long long tp = tile / tiles_c;
    const int c0 = tc * BC;
    const long long p0 = tp * BP;

    // per-lane pixel rows of the gather: pointer to the (possibly out-of-image) pixel of tap (0, 0)
    int hi0[LB], wi0[LB];
    const T* rowp[LB];
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      const long long m = p0 + ld_row + RP * i;
      if (m < M) {
        const int img = (int)(m / HoWo);
        const int rem = (int)(m - (long long)img * HoWo);
        const int ho = rem / a.Wo, wo = rem - ho * a.Wo;
        hi0[i] = ho * a.stride - a.pad;
        wi0[i] = wo * a.stride - a.pad;
        rowp[i] = xg + (((long long)img * a.H + hi0[i]) * a.W + wi0[i]) * a.x_ld;
      } else {
        hi0[i] = -1000000; wi0[i] = 0; rowp[i] = xg;
      }
    }
    const T* wrow[LA];
#pragma unroll
    for (int i = 0; i < LA; ++i) wrow[i] = wg + (size_t)(c0 + ld_row + RP * i) * a.Kp + ld_kv * VN;
    floatx16 acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; ++i)
#pragma unroll
      for (int j = 0; j < TP; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    u32x4 ra[LA], rb[LB];
    bool rb_ok[LB];

    // Operands of K step KB: global -> registers.  The loads are unconditional (an out-of-image tap reads a safe
    // address and is zeroed when it is written to LDS) so that they stay in flight during the MFMA work.
    // Element k = KB*BK + ld_kv*VN of the reduction is channel c of tap (r, s): k = (r*kw + s)*Cin + c; the two
    // divisions use precomputed reciprocals (exact for k < 65536).
#define OCTO_CONV_LOAD(KB)                                                                                          \
    {                                                                                                               \
      _Pragma("unroll") for (int i = 0; i < LA; ++i)                                                                \
        if (BC % RP == 0 || ld_row + RP * i < BC) ra[i] = *(const u32x4*)(wrow[i] + (size_t)(KB) * BK);             \
      if (VEC) {                                                                                                    \
        const unsigned k = (unsigned)(KB) * BK + ld_kv * VN;                                                        \
        const unsigned tap = __umulhi(k, a.magic_cin);                                                              \
        const int c = (int)(k - tap * a.Cin);                                                                       \
        const int r = a.kw == 1 ? (int)tap : (int)__umulhi(tap, a.magic_kw);                                        \
        const int s2 = (int)tap - r * a.kw;                                                                         \
        const int delta = (r * a.W + s2) * a.x_ld + c;                                                              \
        const bool tap_ok = k < (unsigned)a.K;                                                                      \
        _Pragma("unroll") for (int i = 0; i < LB; ++i) {                                                            \
          const bool ok = tap_ok & ((unsigned)(hi0[i] + r) < (unsigned)a.H) & ((unsigned)(wi0[i] + s2) < (unsigned)a.W); \
          const T* src = ok ? rowp[i] + delta : xg;                                                                 \
          rb[i] = *(const u32x4*)src;                                                                               \
          rb_ok[i] = ok;                                                                                            \
        }                                                                                                           \
      } else {                                                                                                      \
        const int kbase = (KB) * BK + ld_kv * VN;                                                                   \
        _Pragma("unroll") for (int i = 0; i < LB; ++i) {                                                            \
          typedef T tv __attribute__((ext_vector_type(VN)));                                                        \
          tv pk;                                                                                                    \
          _Pragma("unroll") for (int e = 0; e < VN; ++e) {                                                          \
            const int k = kbase + e;                                                                                \
            T val = (T)0.0f;                                                                                        \
            if (k < a.K) {                                                                                          \
              const int tap = k / a.Cin, c = k - tap * a.Cin;                                                       \
              const int r = tap / a.kw, s2 = tap - r * a.kw;                                                        \
              if ((unsigned)(hi0[i] + r) < (unsigned)a.H && (unsigned)(wi0[i] + s2) < (unsigned)a.W)                \
                val = rowp[i][(r * a.W + s2) * a.x_ld + c];                                                         \
            }                                                                                                       \
            pk[e] = val;                                                                                            \
          }                                                                                                         \
          rb[i] = __builtin_bit_cast(u32x4, pk);                                                                    \
          rb_ok[i] = true;                                                                                          \
        }                                                                                                           \
      }                                                                                                             \
    }

    __syncthreads();   // the previous tile's LDS reads are done
    if (tid < BC) sBias[tid] = a.bias[c0 + tid];     // bias is padded to a multiple of 128 channels
    OCTO_CONV_LOAD(0)
    for (int kb = 0; kb < nk; ++kb) {
      const int buf = kb & 1;
      // operands of step kb: registers -> LDS
#pragma unroll
      for (int i = 0; i < LA; ++i)
        if (BC % RP == 0 || ld_row + RP * i < BC) sA[buf][ld_row + RP * i][ld_kv] = ra[i];
#pragma unroll
      for (int i = 0; i < LB; ++i) sB[buf][ld_row + RP * i][ld_kv] = rb_ok[i] ? rb[i] : u32x4{0u, 0u, 0u, 0u};
      __syncthreads();
      if (kb + 1 < nk) OCTO_CONV_LOAD(kb + 1)
#pragma unroll
      for (int kk = 0; kk < KV / 2; ++kk) {
        u32x4 fa[TC], fb[TP];
#pragma unroll
        for (int i = 0; i < TC; ++i) fa[i] = sA[buf][wc * (BC / WC) + i * 32 + l32][kk * 2 + g];
#pragma unroll
        for (int j = 0; j < TP; ++j) fb[j] = sB[buf][wp * (BP / WP) + j * 32 + l32][kk * 2 + g];
#pragma unroll
        for (int i = 0; i < TC; ++i)
#pragma unroll
          for (int j = 0; j < TP; ++j) acc[i][j] = E::mfma(fa[i], fb[j], acc[i][j]);
      }
    }
#undef OCTO_CONV_LOAD

    // epilogue: a lane holds pixel column l32 of each 32x32 block and 4 groups of 4 consecutive channels
#pragma unroll
    for (int j = 0; j < TP; ++j) {
      const long long p = p0 + wp * (BP / WP) + j * 32 + l32;
      if (p >= M) continue;
#pragma unroll
      for (int i = 0; i < TC; ++i) {
        const int cblk = wc * (BC / WC) + i * 32 + g * 4;     // channel (inside the tile) of this lane's group q = 0
        if (vec_ok && c0 + cblk + 28 <= a.Cout) {
          // fast path: all four 4-channel groups are inside the tensor and 8/16-byte accesses are aligned
          floatx4 rv[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) rv[q] = floatx4{0.f, 0.f, 0.f, 0.f};
          if (a.res) {
            const T* rp = (const T*)a.res + (size_t)p * a.res_ld + a.res_coff + c0 + cblk;
#pragma unroll
            for (int q = 0; q < 4; ++q) rv[q] = load4<T>(rp + q * 8);
          }
          const size_t o = (size_t)p * a.y_ld + a.y_coff + c0 + cblk;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const floatx4 b4 = *(const floatx4*)&sBias[cblk + q * 8];
            floatx4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = fmaxf(acc[i][j][q * 4 + e] + b4[e] + res_pre * rv[q][e], act_lo);
            if (is_silu) {
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] = silu(v[e]);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += res_post * rv[q][e];
            if (a.out_f32) store4<float>((float*)a.y + o + q * 8, v);
            else store4<T>((T*)a.y + o + q * 8, v);
          }
        } else {
          // edge path: channel tail of the tensor or unaligned pitch - element by element
#pragma unroll
          for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int cl = cblk + q * 8 + e;
              const int c = c0 + cl;
              if (c < a.Cout) {
                float r = 0.f;
                if (a.res) r = (float)((const T*)a.res)[(size_t)p * a.res_ld + a.res_coff + c];
                float t = fmaxf(acc[i][j][q * 4 + e] + sBias[cl] + res_pre * r, act_lo);
                if (is_silu) t = silu(t);
                t += res_post * r;
                const size_t o = (size_t)p * a.y_ld + a.y_coff + c;
                if (a.out_f32) ((float*)a.y)[o] = t; else ((T*)a.y)[o] = (T)t;
              }
            }
          }
        }
      }
    }
  }
}

// kernel id of a conv tile configuration: 1000 + BC*10 ... kept readable: BC, BP and the gather flavour
int conv_kernel_id(int bc, int bp, bool vec) { return 100000 + bc * 1000 + bp * 2 + (vec ? 1 : 0); }

size_t conv_packed_weight_elems(int cout, int kh, int kw, int cin, int dtype, int* kp_out, int* cout_pad_out) {
  const int vn = dtype == OCTO_F32 ? 4 : 8;
  const int bk = 8 * vn;   // largest K step of any tile configuration
  const int K = kh * kw * cin;
  const int kp = (K + bk - 1) / bk * bk;
  const int cp = (cout + 127) / 128 * 128;
  if (kp_out) *kp_out = kp;
  if (cout_pad_out) *cout_pad_out = cp;
  return (size_t)kp * cp;
}

template <typename T, int BC, int BP, int WC, int WP, int KV = 4>
static hipError_t launch_cfg(const ConvArgs& a, bool vec, int num_cu, hipStream_t s, int* kernel_id) {
  if (kernel_id) *kernel_id = conv_kernel_id(BC, BP, vec);
  const long long M = (long long)a.n * a.Ho * a.Wo;
  const long long tiles = ((M + BP - 1) / BP) * ((a.Cout + BC - 1) / BC);
  if (tiles <= 0) return hipSuccess;
  long long grid = tiles;
  const long long cap = (long long)num_cu * 2;      // two resident workgroups per CU (LDS / register bound)
  if (grid > cap) grid = cap;
  if (vec) hipLaunchKernelGGL((conv_mfma_kernel<T, BC, BP, WC, WP, KV, true>), dim3((unsigned)grid), dim3(THREADS), 0, s, a);
  else hipLaunchKernelGGL((conv_mfma_kernel<T, BC, BP, WC, WP, KV, false>), dim3((unsigned)grid), dim3(THREADS), 0, s, a);
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_typed(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id) {
  constexpr int VN = Elem<T>::N;
  const bool vec = (a.Cin % VN == 0) && (a.x_ld % VN == 0) && (a.x_coff % VN == 0) && (((uintptr_t)a.x & 15) == 0);
  const long long M = (long long)a.n * a.Ho * a.Wo;
  // Tile choice: wide channel tiles only when there are enough channels; fall back to smaller pixel tiles when
  // the layer has too few tiles to occupy every CU.
  if (a.Cout <= 32) return launch_cfg<T, 32, 128, 1, 4>(a, vec, num_cu, s, kernel_id);
  if (a.Cout <= 64) {
    return launch_cfg<T, 64, 128, 2, 2>(a, vec, num_cu, s, kernel_id);
  }
  const long long t128 = ((M + 127) / 128) * ((a.Cout + 127) / 128);
  if (t128 >= 2LL * num_cu) return launch_cfg<T, 128, 128, 2, 2>(a, vec, num_cu, s, kernel_id);
  return launch_cfg<T, 64, 64, 2, 2>(a, vec, num_cu, s, kernel_id);
}

hipError_t launch_conv(int dtype, const ConvArgs& a0, int num_cu, hipStream_t s, int* kernel_id) {
  ConvArgs a = a0;
  if (a.Cin < 1 || a.kw < 1 || a.Kp >= 65536) return hipErrorInvalidValue;
  a.magic_cin = a.Cin > 1 ? (unsigned)((1ull << 32) / (unsigned)a.Cin) + 1u : 0u;
  a.magic_kw = a.kw > 1 ? (unsigned)((1ull << 32) / (unsigned)a.kw) + 1u : 0u;
  switch (dtype) {
    case OCTO_F16: return launch_typed<_Float16>(a, num_cu, s, kernel_id);
    case OCTO_BF16: return launch_typed<__bf16>(a, num_cu, s, kernel_id);
    case OCTO_F32: return launch_typed<float>(a, num_cu, s, kernel_id);
  }
  return hipErrorInvalidValue;
}

}  // namespace octo
