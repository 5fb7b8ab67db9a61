// 3x3, stride-1, pad-1 convolution with the input patch of a tile held in LDS.
//
// The general implicit-GEMM kernel (conv.hip) fetches the pixel operand of every K step from global memory, so a
// 3x3 layer reads each input pixel nine times through the vector memory path; for layers with few output channels
// that path, not the matrix cores, sets the pace.  Here a workgroup computes an 8 x 32 block of output pixels for 64
// output channels and
//   - loads the (8+2) x (32+2) input patch once per slice of CS input channels (zero-filled outside the image) straight
//     into LDS, 16-byte vectors XOR-swizzled per pixel so that 32 lanes reading the same channel vector of 32
//     neighbouring pixels hit different banks,
//   - streams the weights of one (tap, channel slice) at a time - a run of CS contiguous K values per output channel -
//     straight from global memory into a two-stage LDS ring (buffer loads with the LDS bit, issued one step ahead),
//   - feeds the MFMA pixel operand from the patch: tap (r, s) of output pixel (y, x) is patch pixel (y + r, x + s).
// Per step a wave issues 16 MFMAs (CS = 64) between two barriers, twice as many as the general kernel's 64x128 tile,
// with a third fewer LDS reads per MFMA.  Used for layers with at most 64 output channels on wide images (+20-25 %
// there); with more output channels the general kernel's 128x128 tile re-uses the pixel operand enough and is faster.  Epilogue as in conv.hip: bias, residual, activation, output tile staged in
// LDS (over the patch) and written with 16-byte stores along the channels.
#include "mfma_common.h"
#include <hip/hip_ext.h>

namespace octo {

constexpr int P3_TH = 8, P3_TW = 32;       // output tile: rows x columns

// wait until at most N of this wave's vector-memory operations are outstanding
template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }

// BC output channels per tile (64: four waves of 64 channels x 2 pixel rows; 128: 2 x 2 waves of 64 channels x 4 rows)
template <typename T, int CS, int BC>
__global__ __launch_bounds__(THREADS, 2) void conv3x3_patch_kernel(const ConvArgs a) {
  using E = Elem<T>;
  static_assert(sizeof(T) == 2 && (CS == 32 || CS == 64) && (BC == 64 || BC == 128), "16-bit types, channel slices of 32 or 64");
  constexpr int TH = P3_TH, TW = P3_TW, BP = TH * TW;
  constexpr int WC = BC / 64, WP = 4 / WC;     // wave grid: channels x pixel rows
  constexpr int TPW = TH / WP;                 // pixel rows (32-pixel blocks) per wave
  constexpr int PH = TH + 2, PW = TW + 2, NPIX = PH * PW;
  constexpr int SPP = CS / 8;                  // 16-byte vectors (slots) per patch pixel
  constexpr int PPW = 16 / SPP;                // patch pixels per 256 bytes of LDS
  constexpr int PVEC = NPIX * SPP;
  constexpr int PLOADS = (PVEC + THREADS - 1) / THREADS;
  constexpr int KV = SPP;                      // vectors per weight-tile row
  constexpr int RPW = 16 / KV;                 // weight-tile rows per 256 bytes
  constexpr int RP = THREADS / KV;             // weight-tile rows per pass of all lanes
  constexpr int LA = BC / RP;                  // passes (direct-to-LDS loads per lane and step)
  static_assert(BC % RP == 0, "whole passes");
  constexpr int ASTAGE = BC * KV;              // vectors per ring stage
  constexpr int OPITCH = 64 * 2 + 16;          // the output tile is staged 64 channels at a time
  constexpr int REGION_VECS = (PLOADS * THREADS > BP * OPITCH / 16) ? PLOADS * THREADS : BP * OPITCH / 16;
  constexpr int NS = 4;                        // weight ring: the tile of tap t + NS - 1 is requested while tap t is computed
  __shared__ u32x4 sA[NS * ASTAGE];
  __shared__ u32x4 sR[REGION_VECS];            // input patch slice, then the staged output tile
  __shared__ float sBias[BC];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
  const int wc = wave % WC, wp = wave / WC;
  int n_items = a.n;
  if (a.n_dyn) { int d = *a.n_dyn; n_items = d < a.n ? d : a.n; }
  const int tiles_x = (a.Wo + TW - 1) / TW, tiles_y = (a.Ho + TH - 1) / TH;
  const int tiles_c = (a.Cout + BC - 1) / BC;
  const int per_img = tiles_x * tiles_y * tiles_c;
  const long long n_tiles = (long long)n_items * per_img;
  const T* __restrict__ xg = (const T*)a.x + a.x_coff;
  const long long img_elems = (long long)a.H * a.W * a.x_ld;
  const bool is_silu = a.act == OCTO_ACT_SILU;
  const float act_lo = a.act == OCTO_ACT_RELU ? 0.0f : -INFINITY;
  const int n_slices = a.Cin / CS;

  // weight tile: lane -> (row, slot); the slot holds logical vector slot ^ ((row / RPW) % KV)
  const int ld_row = tid / KV, ld_kv = tid % KV;
  const int lkv = ld_kv ^ ((ld_row / RPW) % KV);
  const int rsw = (l32 / RPW) % KV;
  const long long w_bytes = (long long)a.w_rows * a.Kp * 2;
  const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, (int)(w_bytes < BUF_MAX ? w_bytes : BUF_MAX), BUF_FLAGS);
  const unsigned lds_wave = (unsigned)__builtin_amdgcn_readfirstlane((int)((unsigned)(uintptr_t)sA + (unsigned)wave * 1024u));
  constexpr unsigned PASS_BYTES = RP * KV * 16, STAGE_BYTES = ASTAGE * 16;
  const unsigned patch_wave = (unsigned)__builtin_amdgcn_readfirstlane((int)((unsigned)(uintptr_t)sR + (unsigned)wave * 1024u));

  const long long per_die = (n_tiles + 7) >> 3;        // contiguous chunk of the tile list per die (see conv.hip)
  for (long long t = blockIdx.x; t < per_die * 8; t += gridDim.x) {
    const long long tile = (t & 7) * per_die + (t >> 3);
    if (tile >= n_tiles) continue;
    const int img = (int)(tile / per_img);
    int rem = (int)(tile - (long long)img * per_img);
    const int tc = rem % tiles_c; rem /= tiles_c;      // channel tiles of the same pixels are neighbours in the list
    const int ty = rem / tiles_x, tx = rem - ty * tiles_x;
    const int oy0 = ty * TH, ox0 = tx * TW, c0 = tc * BC;
    const long long img_bytes = img_elems * 2;
    const __amdgpu_buffer_rsrc_t rsrc_x =
        __builtin_amdgcn_make_buffer_rsrc((void*)(xg + (long long)img * img_elems), 0, (int)(img_bytes < BUF_MAX ? img_bytes : BUF_MAX), BUF_FLAGS);
    int woff[LA];
#pragma unroll
    for (int i = 0; i < LA; ++i) woff[i] = ((c0 + ld_row + RP * i) * a.Kp + lkv * 8) * 2;

    floatx16 acc[2][TPW];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < TPW; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // The residual values this lane will add are requested now and converted in the epilogue, so that their trip to
    // memory runs beside the patch's instead of after the main loop.
    u32x2 rraw[TPW][2][4];
#pragma unroll
    for (int tp = 0; tp < TPW; ++tp)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) rraw[tp][i][q] = u32x2{0u, 0u};
    if (a.res && a.res_mode != OCTO_RES_NONE) {
#pragma unroll
      for (int tp = 0; tp < TPW; ++tp) {
        const int oy = oy0 + wp * TPW + tp, ox = ox0 + l32;
        if (oy < a.Ho && ox < a.Wo) {
          const T* rp = (const T*)a.res + (((size_t)img * a.Ho + oy) * a.Wo + ox) * a.res_ld + a.res_coff + c0 + wc * 64 + g * 4;
#pragma unroll
          for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q)
              if (c0 + wc * 64 + g * 4 + i * 32 + q * 8 + 4 <= a.Cout) rraw[tp][i][q] = *(const u32x2*)(rp + i * 32 + q * 8);
        }
      }
    }

    // this lane's pixel of block tp = 0 at tap (0, 0): patch pixel index; its slot swizzle changes with the tap
    const int ppix0 = (wp * TPW) * PW + l32;

#define OCTO_P3_WEIGHTS(KOFF_BYTES, STAGE)                                                                          \
    {                                                                                                               \
      const unsigned sbase = lds_wave + (unsigned)(STAGE) * STAGE_BYTES;                                            \
      const int koff = (KOFF_BYTES);                                                                                \
      _Pragma("unroll") for (int i = 0; i < LA; ++i)                                                                \
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"                      \
                     :: "s"(sbase + i * PASS_BYTES), "v"(woff[i]), "s"(rsrc_w), "s"(koff) : "memory");               \
    }

    for (int sl = 0; sl < n_slices; ++sl) {
      const int cs0 = sl * CS;
      __syncthreads();                   // everyone is done with the previous patch slice / staged output tile
      if (sl == 0 && tid < BC) sBias[tid] = a.bias[c0 + tid];
      // patch slice: global -> LDS directly.  A lane's LDS slot is fixed by its lane id (vector q = pass * 256 + tid of
      // the patch), so it fetches the channel vector that belongs in that slot under the per-pixel swizzle.
#pragma unroll
      for (int i = 0; i < PLOADS; ++i) {
        const int q = i * THREADS + tid;
        const int pix = q / SPP, slot = q - pix * SPP;
        const int cv = slot ^ ((pix / PPW) % SPP);
        const int prow = pix / PW, pcol = pix - prow * PW;
        const int iy = oy0 - 1 + prow, ix = ox0 - 1 + pcol;
        const bool ok = q < PVEC && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
        const int off = ok ? ((iy * a.W + ix) * a.x_ld + cs0 + cv * 8) * 2 : OOB;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                     :: "s"(patch_wave + i * (THREADS * 16)), "v"(off), "s"(rsrc_x) : "memory");
      }
#pragma unroll
      for (int t = 0; t < NS - 1; ++t) OCTO_P3_WEIGHTS((t * a.Cin + cs0) * 2, t)   // taps 0 .. NS-2 of this slice
#pragma unroll 1
      for (int tap = 0; tap < 9; ++tap) {
        // This wave's part of the patch and of tap's weight tile has landed: loads complete in the order they were
        // issued, and the only ones issued after them are the weight tiles of the following taps (LA loads each) -
        // NS - 2 of them, fewer at the end.  A step of 16 MFMAs is shorter than a trip to the L2, so a ring of two
        // stages left every tap waiting for its weights.
        if (tap <= 9 - NS + 1) wait_vmcnt<(NS - 2) * LA>();
        else if (tap == 9 - NS + 2 && NS > 3) wait_vmcnt<(NS - 3) * LA>();
        else wait_vmcnt<0>();
        __syncthreads();                                              // ... everyone's; the stage read at tap - 1 is free
        if (tap + NS - 1 < 9) OCTO_P3_WEIGHTS(((tap + NS - 1) * a.Cin + cs0) * 2, (tap + NS - 1) % NS)
        const u32x4* pa = sA + (tap % NS) * ASTAGE;
        const int r = tap / 3, s = tap - 3 * r;
        const int pp = ppix0 + r * PW + s;                            // patch pixel of block 0; block 1 is one row down
#pragma unroll
        for (int kc = 0; kc < CS / 16; ++kc) {
          u32x4 fa[2], fb[TPW];
#pragma unroll
          for (int i = 0; i < 2; ++i) fa[i] = pa[(wc * 64 + i * 32 + l32) * KV + ((2 * kc + g) ^ rsw)];
#pragma unroll
          for (int tp = 0; tp < TPW; ++tp) {
            const int pix = pp + tp * PW;
            fb[tp] = sR[pix * SPP + ((2 * kc + g) ^ ((pix / PPW) % SPP))];
          }
#pragma unroll
          for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int tp = 0; tp < TPW; ++tp) acc[i][tp] = E::mfma(fa[i], fb[tp], acc[i][tp]);
        }
      }
    }
#undef OCTO_P3_WEIGHTS

    // epilogue, 64 channels at a time: the waves that own them stage their part of the tile in LDS (over the patch),
    // then all lanes write it out with 16-byte stores
#pragma unroll 1
    for (int half = 0; half < WC; ++half) {
      __syncthreads();                   // everyone is done with the patch / the previous half has been written out
      if (wc == half) {
        with_epilogue_mode(a.res ? a.res_mode : OCTO_RES_NONE, is_silu, [&](auto res_c, auto silu_c) __attribute__((always_inline)) {
        constexpr int RES = decltype(res_c)::value;
        constexpr bool SILU = decltype(silu_c)::value;
#pragma unroll
        for (int tp = 0; tp < TPW; ++tp) {
          const int py = wp * TPW + tp;
          const int pl = py * TW + l32;
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            const int cblk = i * 32 + g * 4;                 // within the 64 channels of this half
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const floatx4 b4 = *(const floatx4*)&sBias[half * 64 + cblk + q * 8];
              floatx4 v;
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] = acc[i][tp][q * 4 + e];
              typedef T t4 __attribute__((ext_vector_type(4)));
              const t4 r4 = __builtin_bit_cast(t4, rraw[tp][i][q]);
              v = finish4<RES, SILU>(v, b4, floatx4{(float)r4[0], (float)r4[1], (float)r4[2], (float)r4[3]}, act_lo);
              store4<T>((T*)((char*)sR + (size_t)pl * OPITCH) + cblk + q * 8, v);
            }
          }
        }
              });
      }
      __syncthreads();
      constexpr int VPR = 8, PPP = THREADS / VPR;            // 8 vectors = 64 channels per pixel
      const int v = tid % VPR, pr = tid / VPR;
      const int c = c0 + half * 64 + v * 8;
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
  }
}

int conv3x3_kernel_id(int cs, int bc) { return 1800000000 + bc * 1000 + cs; }

template <typename T, int CS, int BC>
static hipError_t launch_p3_cfg(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm) {
  if (kernel_id) *kernel_id = conv3x3_kernel_id(CS, BC);
  const long long tiles = (long long)a.n * ((a.Wo + P3_TW - 1) / P3_TW) * ((a.Ho + P3_TH - 1) / P3_TH) * ((a.Cout + BC - 1) / BC);
  if (tiles <= 0) return hipSuccess;
  long long grid = (tiles + 7) / 8 * 8;
  const long long cap = (long long)num_cu * 2;
  if (grid > cap) grid = cap;
  if (tm.start && tm.stop)
    hipExtLaunchKernelGGL((conv3x3_patch_kernel<T, CS, BC>), dim3((unsigned)grid), dim3(THREADS), 0, s, tm.start, tm.stop, 0, a);
  else
    hipLaunchKernelGGL((conv3x3_patch_kernel<T, CS, BC>), dim3((unsigned)grid), dim3(THREADS), 0, s, a);
  return hipGetLastError();
}

// 3x3 / stride 1 / pad 1 layers in the 16-bit types whose input channels come in whole slices of 64 (or 32) and whose
// tensors allow 16-byte accesses; anything else is left to the general kernel (hipErrorNotSupported).
hipError_t launch_conv3x3_patch(int dtype, const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, ConvTiming tm) {
  if ((dtype != OCTO_F16 && dtype != OCTO_BF16) || a.pair_view || a.kh != 3 || a.kw != 3 || a.stride_h != 1 || a.stride_w != 1 || a.pad_h != 1 || a.pad_w != 1 || a.out_f32)
    return hipErrorNotSupported;
  if (a.Ho != a.H || a.Wo != a.W || a.K != 9 * a.Cin || a.w_rows < (a.Cout + 127) / 128 * 128) return hipErrorNotSupported;
  if (((a.x_ld | a.x_coff | a.y_ld | a.y_coff) & 7) || ((uintptr_t)a.x & 15) || ((uintptr_t)a.y & 15)) return hipErrorNotSupported;
  if (a.res && (((a.res_ld | a.res_coff) & 3) || ((uintptr_t)a.res & 7))) return hipErrorNotSupported;
  if ((long long)a.H * a.W * a.x_ld * 2 > BUF_MAX) return hipErrorNotSupported;
  // 128-channel tiles (BC = 128) compile, but measured slower than the general kernel's 128x128 tile: not dispatched
  if (a.Cout > 64) return hipErrorNotSupported;
  const bool h16 = dtype == OCTO_F16;
  if (a.Cin % 64 == 0) return h16 ? launch_p3_cfg<_Float16, 64, 64>(a, num_cu, s, kernel_id, tm) : launch_p3_cfg<__bf16, 64, 64>(a, num_cu, s, kernel_id, tm);
  if (a.Cin % 32 == 0) return h16 ? launch_p3_cfg<_Float16, 32, 64>(a, num_cu, s, kernel_id, tm) : launch_p3_cfg<__bf16, 32, 64>(a, num_cu, s, kernel_id, tm);
  return hipErrorNotSupported;
}

}  // namespace octo
