// First-layer convolution (3 input channels, stride 2) on the matrix cores.
//
// The input is stored with 4 channels, so two neighbouring pixels form one 16-byte vector of 8 values, and a
// stride-2 convolution becomes a stride-1 convolution over pixel pairs with a kernel of KH x PKW pairs (see
// pipeline.hip, which also re-packs the weights as [Cout][(row, pair, 8 values)]).  The general implicit-GEMM kernel
// gathers every K vector of every output pixel from global memory: for a 7x7 kernel that is 28 loads of 16 bytes per
// output pixel, almost all of them re-reads.  Here a workgroup instead
//   - keeps the weight matrix in registers for its lifetime (it is persistent over tiles): every lane holds the
//     MFMA A fragments of its row of each 32-channel block, all K steps of them (112 registers for 64 channels x 7x7).
//     Out of LDS they cost as many bytes per MFMA as the pixel operand, and the two together are exactly what a
//     compute unit's LDS delivers at the full MFMA rate - with two workgroups per unit the loop ran at half of it,
//   - loads the input patch of an 8 x 32 output tile once (21 x 35 pair vectors for 7x7), zero-filled outside the image,
//   - feeds the MFMA B operand straight from the patch: for kernel tap (r, s) output pixel (y, x) needs patch vector
//     (2y + r, x + s), so the 32 lanes of a block read 32 consecutive vectors (bank-conflict free),
//   - stages the output tile in LDS (over the patch) and writes it with 16-byte stores along the channels.
// One K step of the MFMA (16 values) is two pair vectors; with an odd number of vectors the last half step multiplies
// a zero weight column.
#include "mfma_common.h"
#include <hip/hip_ext.h>

namespace octo {

constexpr int STEM_TH = 8, STEM_TW = 32;   // output tile: rows x columns
constexpr int STEM_POOL_COLS = 15;          // pooled columns per strip (their windows span 31 of the tile's 32 columns)

// 16-bit floating-point patterns (two per word) <-> signed 16-bit integers of the same order; its own inverse
__device__ __forceinline__ unsigned order_key16x2(unsigned x) {
  typedef short s16x2 __attribute__((ext_vector_type(2)));
  return x ^ (__builtin_bit_cast(unsigned, __builtin_bit_cast(s16x2, x) >> 15) & 0x7FFF7FFFu);     // negative: magnitude bits flipped
}
__device__ __forceinline__ unsigned max_i16x2(unsigned a, unsigned b) {
  typedef short s16x2 __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(s16x2, a), __builtin_bit_cast(s16x2, b)));
}

// POOL: the layer's output feeds nothing but a 3x3 / stride-2 / pad-1 max-pool, and only the pooled tensor is written
// (a.pool_y).  A workgroup then owns a strip of the image - 15 pooled columns, i.e. convolution columns 30 sx - 1 ..
// 30 sx + 30 - and walks down it tile by tile: the tile staged in LDS plus its predecessor's last row (kept in a
// second LDS buffer) hold every window of four pooled rows, so no convolution row is computed twice; along the
// columns neighbouring strips overlap by two columns of 32.  The maximum is taken on the rounded 16-bit values, as an
// integer maximum of order-preserving keys.
template <typename T, int BC, int KH, int PKW, bool POOL>
__global__ __launch_bounds__(THREADS, 2) void stem_conv_kernel(const ConvArgs a) {
  using E = Elem<T>;
  static_assert(sizeof(T) == 2 && E::N == 8, "pixel pairs are 16-byte vectors of 8 values");
  constexpr int TH = STEM_TH, TW = STEM_TW, BP = TH * TW;
  constexpr int NV = KH * PKW;                 // K vectors
  constexpr int NJ = (NV + 1) / 2;             // MFMA steps
  constexpr int PH = (TH - 1) * 2 + KH, PW = TW + PKW - 1, PVEC = PH * PW;
  constexpr int PLOADS = (PVEC + THREADS - 1) / THREADS;
  constexpr int TC = BC / 32;
  constexpr int OPITCH = BC * 2 + 16;          // bytes per staged output pixel
  constexpr int REGION_VECS = (PLOADS * THREADS > BP * OPITCH / 16) ? PLOADS * THREADS : BP * OPITCH / 16;
  __shared__ u32x4 sR[REGION_VECS];            // input patch, then the staged output tile
  __shared__ u32x4 sCarry[POOL ? 2 * TW * OPITCH / 16 : 1];   // last row of the previous tile of the strip (two buffers, alternating)
  __shared__ float sBias[BC];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
  int n_items = a.n;
  if (a.n_dyn) { int d = *a.n_dyn; n_items = d < a.n ? d : a.n; }
  const int tiles_y = (a.Ho + TH - 1) / TH;
  const int tiles_x = POOL ? (a.pool_wo + STEM_POOL_COLS - 1) / STEM_POOL_COLS : (a.Wo + TW - 1) / TW;
  // unit of work: a tile, or (POOL) a strip of tiles_y tiles
  const int per_img = POOL ? tiles_x : tiles_x * tiles_y;
  const int tiles_per_unit = POOL ? tiles_y : 1;
  const long long n_units = (long long)n_items * per_img;
  const T* __restrict__ xg = (const T*)a.x + a.x_coff;
  const long long img_elems = (long long)a.H * a.W * a.x_ld;
  const bool is_silu = a.act == OCTO_ACT_SILU;
  const float act_lo = a.act == OCTO_ACT_RELU ? 0.0f : -INFINITY;

  // weights -> registers, once: row i * 32 + l32 of the packed matrix, K vector 2 j + g of step j (rows beyond Cout
  // are zero in the packed matrix; the half step past an odd number of vectors multiplies zeros)
  u32x4 wreg[TC][NJ];
  {
    const long long w_bytes = (long long)a.w_rows * a.Kp * 2;
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, (int)(w_bytes < BUF_MAX ? w_bytes : BUF_MAX), BUF_FLAGS);
#pragma unroll
    for (int i = 0; i < TC; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int v = 2 * j + g;
        wreg[i][j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, v < NV ? ((i * 32 + l32) * a.Kp + v * 8) * 2 : OOB, 0, 0);
      }
    if (tid < BC) sBias[tid] = a.bias[tid];
  }

  const long long per_die = (n_units + 7) >> 3;      // contiguous chunk of the unit list per die (see conv.hip)
  const long long t_end = per_die * 8;
  auto unit_of = [&](long long t) -> long long { return (t & 7) * per_die + (t >> 3); };
  auto next_valid = [&](long long t) -> long long {
    while (t < t_end && unit_of(t) >= n_units) t += gridDim.x;
    return t;
  };
  // (position in the unit list, tile of the unit) -> image, tile row and column
  auto locate = [&](long long t, int k, int& img, int& ty, int& tx) {
    const long long unit = unit_of(t);
    img = (int)(unit / per_img);
    const int rem = (int)(unit - (long long)img * per_img);
    ty = POOL ? k : rem / tiles_x;
    tx = POOL ? rem : rem - ty * tiles_x;
  };
  // global loads of a tile's input patch (zeros outside the image); one image per buffer: 32-bit offsets suffice
  u32x4 pv[PLOADS];
  auto load_patch = [&](long long t, int k) {
    int img, ty, tx;
    locate(t, k, img, ty, tx);
    const int iy0 = ty * TH * 2 - a.pad_h, ix0 = (POOL ? tx * (2 * STEM_POOL_COLS) - 1 : tx * TW) - a.pad_w;   // patch origin in input rows / pairs
    const long long img_bytes = img_elems * 2;
    const __amdgpu_buffer_rsrc_t rsrc_x =
        __builtin_amdgcn_make_buffer_rsrc((void*)(xg + (long long)img * img_elems), 0, (int)(img_bytes < BUF_MAX ? img_bytes : BUF_MAX), BUF_FLAGS);
#pragma unroll
    for (int i = 0; i < PLOADS; ++i) {
      const int q = i * THREADS + tid;
      const int prow = q / PW, pcol = q - prow * PW;
      const int iy = iy0 + prow, ix = ix0 + pcol;
      const bool ok = q < PVEC && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
      pv[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, ok ? (iy * a.W + ix) * a.x_ld * 2 : OOB, 0, 0);
    }
  };

  long long t = next_valid(blockIdx.x);
  int k = 0;
  if (t < t_end) load_patch(t, k);
  while (t < t_end) {
    int img, ty, tx;
    locate(t, k, img, ty, tx);
    const int oy0 = ty * TH, ox0 = POOL ? tx * (2 * STEM_POOL_COLS) - 1 : tx * TW;
    __syncthreads();                     // the previous tile's staged output has been written out / pooled
#pragma unroll
    for (int i = 0; i < PLOADS; ++i) sR[i * THREADS + tid] = pv[i];
    __syncthreads();

    floatx16 acc[TC][2];
#pragma unroll
    for (int i = 0; i < TC; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int prow0 = (wave * 2) * 2 * PW + l32;       // patch vector of tap (0, 0) for this lane's pixel of block 0
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int v0 = 2 * j, v1 = 2 * j + 1 < NV ? 2 * j + 1 : NV - 1;   // a half step past the end re-reads a valid vector: its weights are zero
      const int off0 = (v0 / PKW) * PW + (v0 % PKW), off1 = (v1 / PKW) * PW + (v1 % PKW);
      const int boff = prow0 + (g ? off1 : off0);
      u32x4 fb[2];
#pragma unroll
      for (int tp = 0; tp < 2; ++tp) fb[tp] = sR[boff + tp * 2 * PW];
#pragma unroll
      for (int i = 0; i < TC; ++i)
#pragma unroll
        for (int tp = 0; tp < 2; ++tp) acc[i][tp] = E::mfma(wreg[i][j], fb[tp], acc[i][tp]);
    }

    // the next tile's patch is fetched while this one is staged and written (or pooled)
    long long nt = t;
    int nk = k + 1;
    if (nk == tiles_per_unit) { nk = 0; nt = next_valid(t + gridDim.x); }
    if (nt < t_end) load_patch(nt, nk);

    __syncthreads();                     // everyone is done with the patch: the region now stages the output
#pragma unroll
    for (int tp = 0; tp < 2; ++tp) {
      const int pl = (wave * 2 + tp) * TW + l32;
      // the tile's last row also goes to the carry buffer that the strip's next tile reads
      char* carry = POOL && wave * 2 + tp == TH - 1 ? (char*)sCarry + (size_t)(((k + 1) & 1) * TW + l32) * OPITCH : nullptr;
#pragma unroll
      for (int i = 0; i < TC; ++i) {
        const int cblk = i * 32 + g * 4;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const floatx4 b4 = *(const floatx4*)&sBias[cblk + q * 8];
          floatx4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = fmaxf(acc[i][tp][q * 4 + e] + b4[e], act_lo);
          if (is_silu) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = silu(v[e]);
          }
          if constexpr (POOL) {              // staged as order keys: the pooling pass is then a plain integer maximum
            typedef T t4 __attribute__((ext_vector_type(4)));
            const t4 h = {(T)v[0], (T)v[1], (T)v[2], (T)v[3]};
            u32x2 kk = __builtin_bit_cast(u32x2, h);
            kk[0] = order_key16x2(kk[0]); kk[1] = order_key16x2(kk[1]);
            *(u32x2*)((char*)sR + (size_t)pl * OPITCH + (size_t)(cblk + q * 8) * 2) = kk;
            if (carry) *(u32x2*)(carry + (size_t)(cblk + q * 8) * 2) = kk;
          } else {
            store4<T>((T*)((char*)sR + (size_t)pl * OPITCH) + cblk + q * 8, v);
          }
        }
      }
    }
    __syncthreads();
    constexpr int VPR = BC / 8;                  // 16-byte vectors per pixel
    if constexpr (POOL) {
      // pooled rows 4 ty .. 4 ty + 3: window rows 2 py - 1 .. 2 py + 1 = staged rows -1 (the carry) .. 7; window columns
      // 2 pc .. 2 pc + 2 of the tile (convolution column = ox0 + tile column)
      constexpr int POOL_ROWS = TH / 2;
      for (int item = tid; item < POOL_ROWS * STEM_POOL_COLS * VPR; item += THREADS) {
        const int v = item % VPR, pp = item / VPR;
        const int pr = pp / STEM_POOL_COLS, pc = pp - pr * STEM_POOL_COLS;
        const int py = ty * POOL_ROWS + pr, px = tx * STEM_POOL_COLS + pc;
        if (py >= a.pool_ho || px >= a.pool_wo || v * 8 >= a.Cout) continue;
        u32x4 best = {0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u};      // smallest key
#pragma unroll
        for (int dr = 0; dr < 3; ++dr) {
          const int r = 2 * pr + dr - 1;         // staged row, -1: the carry
          const int oy = oy0 + r;
          if (oy < 0 || oy >= a.Ho) continue;
          const char* row = r < 0 ? (const char*)sCarry + (size_t)((k & 1) * TW) * OPITCH : (const char*)sR + (size_t)(r * TW) * OPITCH;
#pragma unroll
          for (int dc = 0; dc < 3; ++dc) {
            const int col = 2 * pc + dc;
            const int ox = ox0 + col;
            if (ox < 0 || ox >= a.Wo) continue;
            const u32x4 val = *(const u32x4*)(row + (size_t)col * OPITCH + (size_t)v * 16);
#pragma unroll
            for (int e = 0; e < 4; ++e) best[e] = max_i16x2(best[e], val[e]);
          }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) best[e] = order_key16x2(best[e]);
        T* yp = (T*)a.pool_y + (((size_t)img * a.pool_ho + py) * a.pool_wo + px) * a.pool_ld + a.pool_coff + v * 8;
        if (v * 8 + 8 <= a.Cout) {
          *(u32x4*)yp = best;
        } else {
          typedef T tv __attribute__((ext_vector_type(8)));
          const tv tvv = __builtin_bit_cast(tv, best);
#pragma unroll
          for (int e = 0; e < 8; ++e) if (v * 8 + e < a.Cout) yp[e] = tvv[e];
        }
      }
    } else {
    constexpr int PPP = THREADS / VPR;           // pixels per pass
    const int v = tid % VPR, pr = tid / VPR;
    const int c = v * 8;
#pragma unroll
    for (int ps = 0; ps < BP / PPP; ++ps) {
      const int pl = ps * PPP + pr;
      const int oy = oy0 + pl / TW, ox = ox0 + pl % TW;
      if (oy < a.Ho && ox < a.Wo && c < a.Cout) {
        const u32x4 val = *(const u32x4*)((const char*)sR + (size_t)pl * OPITCH + (size_t)v * 16);
        T* yp = (T*)a.y + (((size_t)img * a.Ho + oy) * a.Wo + ox) * a.y_ld + a.y_coff + c;
        if (c + 8 <= a.Cout) {
          *(u32x4*)yp = val;
        } else {
          typedef T tv __attribute__((ext_vector_type(8)));
          const tv tvv = __builtin_bit_cast(tv, val);
#pragma unroll
          for (int e = 0; e < 8; ++e) if (c + e < a.Cout) yp[e] = tvv[e];
        }
      }
    }
    }
    t = nt; k = nk;
  }
}

int stem_kernel_id(int bc, int kh, int pkw, bool pool) { return 1900000000 + (pool ? 1000000 : 0) + bc * 1000 + kh * 10 + pkw; }

template <typename T, int BC, int KH, int PKW, bool POOL>
static hipError_t launch_stem_cfg(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm) {
  if (kernel_id) *kernel_id = stem_kernel_id(BC, KH, PKW, POOL);
  const long long units = POOL ? (long long)a.n * ((a.pool_wo + STEM_POOL_COLS - 1) / STEM_POOL_COLS)
                               : (long long)a.n * ((a.Wo + STEM_TW - 1) / STEM_TW) * ((a.Ho + STEM_TH - 1) / STEM_TH);
  if (units <= 0) return hipSuccess;
  long long grid = (units + 7) / 8 * 8;
  const long long cap = (long long)num_cu * 2;
  if (grid > cap) grid = cap;
  if (tm.start && tm.stop)
    hipExtLaunchKernelGGL((stem_conv_kernel<T, BC, KH, PKW, POOL>), dim3((unsigned)grid), dim3(THREADS), 0, s, tm.start, tm.stop, 0, a);
  else
    hipLaunchKernelGGL((stem_conv_kernel<T, BC, KH, PKW, POOL>), dim3((unsigned)grid), dim3(THREADS), 0, s, a);
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_stem_typed(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm) {
  if (a.pool_y) {
    if (a.kh == 7 && a.kw == 4 && a.Cout <= 64) return launch_stem_cfg<T, 64, 7, 4, true>(a, num_cu, s, kernel_id, tm);
    return hipErrorNotSupported;
  }
  if (a.kh == 7 && a.kw == 4 && a.Cout <= 64) return launch_stem_cfg<T, 64, 7, 4, false>(a, num_cu, s, kernel_id, tm);
  if (a.kh == 6 && a.kw == 3 && a.Cout <= 32) return launch_stem_cfg<T, 32, 6, 3, false>(a, num_cu, s, kernel_id, tm);
  if (a.kh == 6 && a.kw == 3 && a.Cout <= 64) return launch_stem_cfg<T, 64, 6, 3, false>(a, num_cu, s, kernel_id, tm);
  if (a.kh == 3 && a.kw == 2 && a.Cout <= 32) return launch_stem_cfg<T, 32, 3, 2, false>(a, num_cu, s, kernel_id, tm);
  return hipErrorNotSupported;
}

// Pixel-pair first layers in the 16-bit types, stride 2, with one of the kernel shapes above, 16-byte aligned output
// rows and no residual; anything else is left to the general kernel (hipErrorNotSupported).  With a fused max-pool:
// the 7x7 shape only, pooled size (Ho + 1) / 2 x (Wo + 1) / 2, 16-byte aligned pooled rows.
hipError_t launch_stem(int dtype, const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, ConvTiming tm) {
  if (!a.pair_view || (dtype != OCTO_F16 && dtype != OCTO_BF16) || a.stride_h != 2 || a.stride_w != 1 || a.Cin != 8 || a.x_ld != 8 || a.res || a.out_f32)
    return hipErrorNotSupported;
  if (a.pool_y) {
    if (a.pool_ho != (a.Ho + 1) / 2 || a.pool_wo != (a.Wo + 1) / 2 || ((a.pool_ld | a.pool_coff) & 7) || ((uintptr_t)a.pool_y & 15)) return hipErrorNotSupported;
  } else if (((a.y_ld | a.y_coff) & 7) || ((uintptr_t)a.y & 15)) {
    return hipErrorNotSupported;
  }
  if (((uintptr_t)a.x & 15) || (a.x_coff & 7)) return hipErrorNotSupported;
  if ((long long)a.H * a.W * 16 > BUF_MAX || a.w_rows < 64) return hipErrorNotSupported;
  return dtype == OCTO_F16 ? launch_stem_typed<_Float16>(a, num_cu, s, kernel_id, tm) : launch_stem_typed<__bf16>(a, num_cu, s, kernel_id, tm);
}

}  // namespace octo
