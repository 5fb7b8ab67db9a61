// Pieces shared by the matrix-core kernels: 16-byte operand vectors, the MFMA instruction per storage type, packed
// loads / stores of four values, the fast SiLU and the buffer-load constants.
#pragma once
#include <type_traits>

#include "octo_internal.h"

namespace octo {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte operand vector
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

// One byte of 8-bit floating point, OCP E4M3: sign, 4 exponent bits (bias 7), 3 mantissa bits; no infinities, 0x7F and
// 0xFF are NaN, the largest finite value is 448.  The conversion instructions of this GPU use that format.
struct f8 { uint8_t bits; };
constexpr float F8_MAX = 448.0f;

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
template <> struct Elem<f8> {
  static constexpr int N = 16;
  // K = 64 per instruction: a lane supplies 32 consecutive bytes per operand, here two 16-byte vectors.  Which K
  // indices they are does not matter as long as both operands use the same ones.
  static __device__ __forceinline__ floatx16 mfma2(u32x4 a0, u32x4 a1, u32x4 b0, u32x4 b1, floatx16 c) {
    const i32x8 a = {(int)a0[0], (int)a0[1], (int)a0[2], (int)a0[3], (int)a1[0], (int)a1[1], (int)a1[2], (int)a1[3]};
    const i32x8 b = {(int)b0[0], (int)b0[1], (int)b0[2], (int)b0[3], (int)b1[0], (int)b1[1], (int)b1[2], (int)b1[3]};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);   // formats 0 = E4M3, scales 2^0
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

// E4M3 <-> fp32.  Encoding rounds to nearest even and saturates at +-448 (the clamp comes first, so the conversion
// instruction never sees a value it would have to turn into NaN); NaN stays NaN.
__device__ __forceinline__ uint32_t f8_pack4(floatx4 v) {
  int w = 0;
  w = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_amdgcn_fmed3f(v[0], -F8_MAX, F8_MAX), __builtin_amdgcn_fmed3f(v[1], -F8_MAX, F8_MAX), w, false);
  w = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_amdgcn_fmed3f(v[2], -F8_MAX, F8_MAX), __builtin_amdgcn_fmed3f(v[3], -F8_MAX, F8_MAX), w, true);
  return (uint32_t)w;
}
__device__ __forceinline__ floatx4 f8_unpack4(uint32_t w) {
  return floatx4{__builtin_amdgcn_cvt_f32_fp8((int)w, 0), __builtin_amdgcn_cvt_f32_fp8((int)w, 1),
                 __builtin_amdgcn_cvt_f32_fp8((int)w, 2), __builtin_amdgcn_cvt_f32_fp8((int)w, 3)};
}
template <typename T> __device__ __forceinline__ float to_f32(T v) {
  if constexpr (std::is_same<T, f8>::value) return __builtin_amdgcn_cvt_f32_fp8((int)v.bits, 0);
  else return (float)v;
}
template <typename T> __device__ __forceinline__ T from_f32(float f) {
  if constexpr (std::is_same<T, f8>::value) {
    const float c = __builtin_amdgcn_fmed3f(f, -F8_MAX, F8_MAX);
    return f8{(uint8_t)(__builtin_amdgcn_cvt_pk_fp8_f32(c, c, 0, false) & 0xFF)};
  } else {
    return (T)f;
  }
}

template <typename T>
__device__ __forceinline__ floatx4 load4(const T* p) {
  if constexpr (sizeof(T) == 4) {
    return *(const floatx4*)p;
  } else if constexpr (sizeof(T) == 1) {
    return f8_unpack4(*(const uint32_t*)p);
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
  } else if constexpr (sizeof(T) == 1) {
    *(uint32_t*)p = f8_pack4(v);
  } else {
    typedef T t4 __attribute__((ext_vector_type(4)));
    const t4 o = {(T)v[0], (T)v[1], (T)v[2], (T)v[3]};
    *(u32x2*)p = __builtin_bit_cast(u32x2, o);
  }
}
// floor(n / d) for n < 2^31 with magic = ceil(2^(32+shift) / d) (fits 32 bits for the shift chosen on the host)
__device__ __forceinline__ unsigned udiv(unsigned n, unsigned magic, unsigned shift) { return __umulhi(n, magic) >> shift; }
// x * sigmoid(x) with the hardware exp2 / reciprocal (about 1 ulp each: far below the storage precision)
__device__ __forceinline__ float silu(float v) { return v * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(v * -1.4426950408889634f)); }

// Epilogue arithmetic of four values, specialised at compile time by where the residual enters (OCTO_RES_*) and whether
// the activation is SiLU (otherwise max with act_lo: 0 for ReLU, -inf for none).  The epilogue is vector arithmetic that
// competes with the matrix pipe for issue slots - 64 values per lane and tile - so terms that a layer does not have are
// compiled out instead of being multiplied by zero.
template <int RES, bool SILU>
__device__ __forceinline__ floatx4 finish4(floatx4 acc, floatx4 bias, floatx4 res, float act_lo) {
  floatx4 v;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    float t = acc[e] + bias[e];
    if (RES == OCTO_RES_BEFORE_ACT) t += res[e];
    t = SILU ? silu(t) : fmaxf(t, act_lo);
    if (RES == OCTO_RES_AFTER_ACT) t += res[e];
    v[e] = t;
  }
  return v;
}
template <int RES, bool SILU>
__device__ __forceinline__ float finish1(float acc, float bias, float res, float act_lo) {
  float t = acc + bias;
  if (RES == OCTO_RES_BEFORE_ACT) t += res;
  t = SILU ? silu(t) : fmaxf(t, act_lo);
  if (RES == OCTO_RES_AFTER_ACT) t += res;
  return t;
}
// Calls f(residual mode, SiLU?) with both as compile-time constants (std::integral_constant) for a uniform run-time pair.
template <typename F>
__device__ __forceinline__ void with_epilogue_mode(int res_mode, bool is_silu, F&& f) {
  using std::integral_constant;
  if (is_silu) {
    if (res_mode == OCTO_RES_BEFORE_ACT) f(integral_constant<int, OCTO_RES_BEFORE_ACT>{}, integral_constant<bool, true>{});
    else if (res_mode == OCTO_RES_AFTER_ACT) f(integral_constant<int, OCTO_RES_AFTER_ACT>{}, integral_constant<bool, true>{});
    else f(integral_constant<int, OCTO_RES_NONE>{}, integral_constant<bool, true>{});
  } else {
    if (res_mode == OCTO_RES_BEFORE_ACT) f(integral_constant<int, OCTO_RES_BEFORE_ACT>{}, integral_constant<bool, false>{});
    else if (res_mode == OCTO_RES_AFTER_ACT) f(integral_constant<int, OCTO_RES_AFTER_ACT>{}, integral_constant<bool, false>{});
    else f(integral_constant<int, OCTO_RES_NONE>{}, integral_constant<bool, false>{});
  }
}

constexpr int THREADS = 256;
constexpr unsigned BUF_FLAGS = 0x00020000u;      // raw buffer, 32-bit data format
constexpr int OOB = (int)0x80000000;             // offset beyond any buffer range: the load returns zeros
constexpr long long BUF_MAX = 0x7FFFFFFFLL;


}  // namespace octo
