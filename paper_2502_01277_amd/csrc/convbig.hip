// 3x3 / stride-1 convolution for wide layers (about 96 and more output channels) on the matrix cores, with the input
// patch of a tile resident in LDS.
//
// What paces the general implicit-GEMM kernel (conv.hip) on such layers is the vector-memory path: measured on
// MI355X, global -> LDS loads of scattered 64..128-byte pieces run at 23..30 bytes per clock and compute unit however
// deep they are queued, while a 128 x 128 tile needs 64 bytes per clock at the full MFMA rate (a 256 x 256 tile 32).
// A 3x3 layer fetches every input pixel nine times there, once per kernel tap.  Here
//   * a tile is TH x TW output pixels (up to 256, or 512 with the narrow channel tile) of the image stack - the images
//     of the batch stacked vertically, so a tile may span several small images - times BC = 96 / 192 / 256 output channels;
//   * the K loop runs slice-major: for every slice of 32 input channels, the nine taps in turn.  The input patch of a
//     slice (the tile's rows and columns plus a one-pixel border, 64 bytes per pixel, zero outside the images) is
//     loaded once into one of two LDS buffers and the MFMA pixel operand of every tap is read from it with a shifted
//     index; only the weights of a (slice, tap) step, BC x 64 bytes, stream through a ring of NST LDS stages.  Per
//     step a 256 x 256 tile then fetches 16 KB + 1/9 of a patch (about 3 KB) instead of 32 KB;
//   * loads run NST steps ahead of the arithmetic and continuously across tiles (while the last steps of a tile are
//     multiplied the ring already receives the next tile's weights and patch), the one barrier per step sits in the
//     middle of the step's MFMAs, and the epilogue writes from registers, so LDS never has to drain between tiles;
//   * four wavefronts per workgroup, each on (BC / 2) x 128 outputs (96 x 128 with the 96-channel tile): up to 16
//     accumulator blocks of 32 x 32 in the AGPR half of the register file, 7 or 8 operand fragments per 12 or 16 MFMAs;
//   * the bias of a tile arrives in LDS through the same load stream (one 4-byte load per lane and step).
// LDS rows (weights: one output channel; patch: one pixel) are 64 bytes = four 16-byte vectors; vector v of row r sits
// in slot v ^ ((r / 4) % 4), which makes both the 1 KB-contiguous fills and the fragment reads (32 consecutive rows,
// one vector each) bank-conflict free.
// vmcnt bookkeeping: every wavefront issues the same, compile-time known number of loads per step (the nine taps of a
// slice are unrolled), in program order, and loads complete in order;
// stores (epilogue) may complete out of order with respect to loads, but "at most N operations outstanding" still
// implies that all but the N youngest loads have landed.
#include "octo_internal.h"
#include "mfma_common.h"
#include <hip/hip_ext.h>
#include <type_traits>

namespace octo {

// Tile geometry of one layer, built on the host (launch_conv3x3_big).
struct BigGeom {
  int TW, TH;            // output tile: TH rows of the image stack x TW columns; TW divides the image width
  int PW;                // patch width TW + 2
  int tiles_x;           // tiles per image row
  int PL;                // 4 KB passes of the 256 loader lanes that cover the largest patch (<= 8)
  int patch_bytes;       // PL * 4096
  FastDiv div_tw, div_pw, div_h, div_hp2, div_tc, div_tx;   // divisions by TW, PW, H, H + 2, tiles_c, tiles_x
};

namespace {
template <typename T> struct Mfma16;
template <> struct Mfma16<_Float16> {
  static __device__ __forceinline__ floatx16 run(u32x4 a, u32x4 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
  }
};
template <> struct Mfma16<__bf16> {
  static __device__ __forceinline__ floatx16 run(u32x4 a, u32x4 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};
}  // namespace

// A wavefront computes TC x TP blocks of 32 channels x 32 pixels; the four wavefronts of a workgroup are laid out WC along
// the channels and 4 / WC along the pixels, so a tile has BC = 32 * TC * WC channels and BP = 32 * TP * 4 / WC pixels
// (256 or 512).  NST: stages of the weight ring.
template <typename T, int TC, int TP, int WC, int NST>
__global__ __launch_bounds__(THREADS, 1) void conv3x3_big_kernel(const ConvArgs a, const BigGeom gm) {
  static_assert(sizeof(T) == 2, "16-bit storage types");
  constexpr int VN = 8, ES = 2, KV = 4, BK = KV * VN, WP = 4 / WC;
  constexpr int BC = TC * WC * 32, BP = TP * WP * 32;
  static_assert(BP == 256 || BP == 512, "tile of 256 or 512 pixels");
  constexpr int RP = THREADS / KV;         // 64 rows per 4 KB pass of the 256 loader lanes
  constexpr int LA = (BC + RP - 1) / RP;
  // patch passes per step (PPT) at the four loader taps NST .. NST + 3: 8 passes (32 KB) cover the largest patch of a
  // 256-pixel tile, 16 that of a 512-pixel tile
  constexpr int PPT = BP / 128, MAXP = 4 * PPT;
  // loads per wavefront in the step whose loader tap is t: LA of weights; at taps NST .. NST + 3 PPT passes of the next
  // slice's patch; at the last tap the tile's bias
  constexpr auto nlt = [](int t) constexpr { return LA + ((t >= NST && t < NST + 4) ? PPT : 0) + (t == 8 ? 1 : 0); };
  constexpr unsigned ROW_BYTES = KV * 16, STAGE_BYTES = LA * RP * ROW_BYTES, PASS_BYTES = RP * ROW_BYTES;
  constexpr int N_TAPS = 9;
  static_assert(NST >= 3 && NST <= 4 && (NST - 1) * (LA + PPT) + MAXP <= 63, "patch passes at taps NST .. NST + 3; vmcnt has six bits");
  static_assert(TC * TP >= TC + TP + 1, "a half step has room for its operand reads");

  extern __shared__ __attribute__((aligned(1024))) unsigned char dyn_lds[];
  unsigned char* ring = dyn_lds;                                   // NST stages of BC x 64 bytes
  unsigned char* patch = dyn_lds + NST * STAGE_BYTES;              // 2 buffers of gm.patch_bytes
  float* sBias = (float*)(patch + 2 * gm.patch_bytes);             // 2 x 256 floats
  int* sPoff = (int*)(sBias + 2 * THREADS);                        // [MAXP][256]: every lane's patch offsets (own column only)
  unsigned char* dump = (unsigned char*)(sPoff + MAXP * THREADS);  // 4 KB that the placeholder loads (zeros) land in

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wc = wave % WC, wp = wave / WC;
  const int l32 = lane & 31, g = lane >> 5;

  int n_items = a.n;
  if (a.n_dyn) { const int d = *a.n_dyn; n_items = d < a.n ? d : a.n; }
  const int H = a.H, W = a.W;              // stride 1, pad 1: output size == input size
  const int n_rows = n_items * H;          // rows of the image stack
  const int tiles_c = (a.Cout + BC - 1) / BC;
  const int tiles_v = (n_rows + gm.TH - 1) / gm.TH;
  const long long n_tiles = (long long)tiles_v * gm.tiles_x * tiles_c;     // < 2^31 (host)
  const int n_slices = a.Cin / BK;
  const int nk = n_slices * N_TAPS;
  const T* __restrict__ xg = (const T*)a.x + a.x_coff;
  const long long img_elems = (long long)H * W * a.x_ld;

  const int ld_row = tid / KV;
  const int lkv = (tid % KV) ^ ((ld_row >> 2) & 3);      // logical vector that belongs into this lane's LDS slot
  const unsigned rsw = (unsigned)((l32 >> 2) & 3);

  const long long w_bytes = (long long)a.w_rows * a.Kp * ES;
  const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, (int)(w_bytes < BUF_MAX ? w_bytes : BUF_MAX), BUF_FLAGS);
  const __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc((void*)a.bias, 0, a.w_rows * 4, BUF_FLAGS);

  const unsigned lds_wave = (unsigned)__builtin_amdgcn_readfirstlane((int)((unsigned)(uintptr_t)ring + (unsigned)wave * 1024u));
  const unsigned lds_patch = (unsigned)__builtin_amdgcn_readfirstlane((int)((unsigned)(uintptr_t)patch + (unsigned)wave * 1024u));
  const unsigned lds_dump = (unsigned)__builtin_amdgcn_readfirstlane((int)((unsigned)(uintptr_t)dump + (unsigned)wave * 1024u));
  const unsigned lds_bias = (unsigned)__builtin_amdgcn_readfirstlane((int)((unsigned)(uintptr_t)sBias + (unsigned)wave * 256u));

  // tile list of this workgroup: positions blockIdx.x, + gridDim.x, ...; workgroup b runs on die b % 8 and the grid is a
  // multiple of 8, so die d owns the contiguous chunk [d * per_die, (d + 1) * per_die) of the tile list (tiles that
  // share a patch - the channel tiles of the same pixels - and neighbouring patches meet in one L2)
  const int per_die = (int)((n_tiles + 7) >> 3);
  const long long t_end = (long long)per_die * 8;
  auto tile_of = [&](long long t) -> long long { return (long long)((int)t & 7) * per_die + (t >> 3); };
  auto next_valid = [&](long long t) -> long long {
    while (t < t_end && tile_of(t) >= n_tiles) t += gridDim.x;
    return t;
  };
  // tile -> (first channel, first column, first stack row)
  auto tile_origin = [&](long long t, int& c0, int& x0, int& v0) {
    const unsigned tile = (unsigned)tile_of(t);
    const unsigned tpx = fast_div(tile, gm.div_tc);
    c0 = (int)(tile - tpx * (unsigned)tiles_c) * BC;
    const unsigned tv = fast_div(tpx, gm.div_tx);
    x0 = (int)(tpx - tv * (unsigned)gm.tiles_x) * gm.TW;
    v0 = (int)tv * gm.TH;
  };
  // stack row -> row of the padded stack (every image with a zero row above and below)
  auto padded_row = [&](int v) -> int { const int img = (int)fast_div((unsigned)v, gm.div_h); return img * (H + 2) + (v - img * H) + 1; };

  // ---- weight loader: (tile, slice, tap), NST steps ahead of the arithmetic ----
  const long long t_first = next_valid(blockIdx.x);
  if (t_first >= t_end) return;
  long long lt = t_first;
  int lkb = 0, lslice = 0, lpar = 0;       // the loader's tap is lkb % 9: a compile-time constant where the steps are unrolled
  int woff[LA];
  int boff = OOB;
  auto wloader_setup = [&]() {
    lkb = 0; lslice = 0;
    if (lt >= t_end) {
#pragma unroll
      for (int i = 0; i < LA; ++i) woff[i] = OOB;
      boff = OOB;
      return;
    }
    int c0, x0, v0;
    tile_origin(lt, c0, x0, v0);
#pragma unroll
    for (int i = 0; i < LA; ++i)             // rows past the tile or the matrix: out of range, zeros
      woff[i] = ld_row + RP * i < BC ? ((c0 + ld_row + RP * i) * a.Kp + lkv * VN) * ES : OOB;
    boff = tid < BC ? (c0 + tid) * 4 : OOB;
  };

  // ---- patch loader: the patch of the slice AFTER the weight loader's slice (possibly slice 0 of the next tile) ----
  long long pt = lt;                       // tile whose patch is loaded next
  int pslice = 0, ppar = 0;                // its slice, and the patch buffer it goes to
  // sPoff[i][tid]: byte offset of this lane's vector of pass i from the tile's first image (or OOB); kept in LDS, every
  // lane reads only what it wrote itself, so no barrier is involved
  // the patch's buffer descriptor (base: the first image the patch touches) is rebuilt from these three uniform words
  // where a load is issued, which keeps them in scalar registers whatever the register pressure
  int p_lo = 0, p_hi = 0, p_len = 0;
  auto ploader_setup = [&]() {
    if (pt >= t_end) {
#pragma unroll
      for (int i = 0; i < MAXP; ++i) sPoff[i * THREADS + tid] = OOB;
      return;
    }
    int c0, x0, v0;
    tile_origin(pt, c0, x0, v0);
    const int vlast = v0 + gm.TH - 1 < n_rows - 1 ? v0 + gm.TH - 1 : n_rows - 1;
    const int P0 = padded_row(v0) - 1, P1 = padded_row(vlast) + 1;
    const int patch_px = (P1 - P0 + 1) * gm.PW;
    const int img0 = (int)fast_div((unsigned)P0, gm.div_hp2);
    const long long rem_bytes = ((long long)(a.n - img0) * img_elems - a.x_coff) * ES;
    const uintptr_t pbase = (uintptr_t)(xg + (long long)img0 * img_elems);
    p_lo = (int)(unsigned)pbase; p_hi = (int)(unsigned)(pbase >> 32); p_len = (int)(rem_bytes < BUF_MAX ? rem_bytes : BUF_MAX);
#pragma unroll 1
    for (int i = 0; i < MAXP; ++i) {
      const int j = i * THREADS + tid;     // vector of the patch buffer this lane fills in pass i
      const int pp = j >> 2;               // patch pixel; its slot j & 3 holds logical vector slot ^ ((pp / 4) % 4)
      const int vec = (j & 3) ^ ((pp >> 2) & 3);
      const int pr = (int)fast_div((unsigned)pp, gm.div_pw), pc = pp - pr * gm.PW;
      const int P = P0 + pr;
      const int img = (int)fast_div((unsigned)P, gm.div_hp2);
      const int yy = P - img * (H + 2) - 1, xx = x0 - 1 + pc;
      const bool ok = pp < patch_px && (unsigned)yy < (unsigned)H && (unsigned)xx < (unsigned)W && img < n_items;
      sPoff[i * THREADS + tid] = ok ? (int)((((long long)(img - img0) * H + yy) * W + xx) * a.x_ld + vec * VN) * ES : OOB;
    }
  };
  auto ploader_next = [&]() {              // successor of (pt, pslice)
    ppar ^= 1;
    if (++pslice == n_slices) { pslice = 0; pt = next_valid(pt + gridDim.x); ploader_setup(); }
  };

  // the pieces of one step's loads
  auto issue_weight = [&](int st, int ltap, int i) {     // pass i (64 rows) of the weights of (lslice, ltap)
    const unsigned sbase = lds_wave + (unsigned)st * STAGE_BYTES;
    const int koff = (ltap * a.Cin + lslice * BK) * ES;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(sbase + i * PASS_BYTES), "v"(woff[i]), "s"(rsrc_w), "s"(koff) : "memory");
  };
  // Patch passes: the lane's offset of a pass is fetched from LDS first (patch_offset) and used later (issue_patch_pass), so
  // that the wait for it does not also wait for the operand fragment reads issued in between.
  auto patch_offset = [&](int pass) -> int {   // uniform `pass`; OOB for a pass beyond the patch (or negative)
    if (pass < 0 || pass >= gm.PL) return OOB;
    const int po = sPoff[pass * THREADS + tid];
    return po == OOB ? OOB : po + pslice * (BK * ES);
  };
  auto issue_patch_pass = [&](int pass, int off) {
    // a load to LDS always writes (zeros when out of range): placeholders go to the dump
    const unsigned dst = pass >= 0 && pass < gm.PL ? lds_patch + (unsigned)ppar * (unsigned)gm.patch_bytes + (unsigned)pass * 4096u : lds_dump;
    const uintptr_t base = (uintptr_t)(unsigned)__builtin_amdgcn_readfirstlane(p_lo) | ((uintptr_t)(unsigned)__builtin_amdgcn_readfirstlane(p_hi) << 32);
    const __amdgpu_buffer_rsrc_t rsrc_p = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, __builtin_amdgcn_readfirstlane(p_len), BUF_FLAGS);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(__builtin_amdgcn_readfirstlane((int)dst)), "v"(off), "s"(rsrc_p) : "memory");
  };
  auto issue_bias = [&]() {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                 :: "s"(lds_bias + (unsigned)lpar * (THREADS * 4u)), "v"(boff), "s"(rsrc_b) : "memory");
  };
  auto loader_advance = [&](int ltap) {    // uniform
    ++lkb;
    if (ltap == N_TAPS - 1) { ++lslice; ploader_next(); }
    if (lkb == nk) {                       // on to the workgroup's next tile
      lt = next_valid(lt + gridDim.x);
      lpar ^= 1;
      wloader_setup();
    }
  };

  wloader_setup();
  // patch of (first tile, slice 0): all passes up front, then the patch loader moves on to slice 1
  ploader_setup();
#pragma unroll 1
  for (int i = 0; i < MAXP; ++i) issue_patch_pass(i, patch_offset(i));
  ploader_next();
#pragma unroll
  for (int d = 0; d < NST; ++d) {          // taps 0 .. NST - 1 of the first tile: weights only (nk >= 9 > NST)
#pragma unroll
    for (int i = 0; i < LA; ++i) issue_weight(d, d, i);
    loader_advance(d);
  }

  // ---- consumer state ----
  long long ct = t_first;                  // consumer's position in the tile list
  int rd = 0, cpar = 0, cbuf = 0;          // ring stage of the current step, bias buffer of the current tile, patch buffer of the current slice
  // byte offset inside a patch buffer of the vector with channels 0..15 of the slice (the one with 16..31 is this ^ 32)
  // for this lane's pixel of block j at kernel tap t
  unsigned baddr[N_TAPS][TP];
  int pix[TP];                             // output pixel index of block j (-1: outside the tile or the stack)
  int c0 = 0;
  auto consumer_setup = [&]() {
    int x0, v0;
    tile_origin(ct, c0, x0, v0);
    const int P0 = padded_row(v0) - 1;
    const int tile_px = gm.TH * gm.TW;
#pragma unroll
    for (int j = 0; j < TP; ++j) {
      const int q = wp * (TP * 32) + j * 32 + l32;
      const int ty = (int)fast_div((unsigned)q, gm.div_tw), tx = q - ty * gm.TW;
      const int v = v0 + ty;
      const bool ok = q < tile_px && v < n_rows;
      const int pb = ok ? (padded_row(v) - 1 - P0) * gm.PW + tx : 0;       // patch pixel under tap (0, 0)
      pix[j] = ok ? v * W + x0 + tx : -1;
#pragma unroll
      for (int t = 0; t < N_TAPS; ++t) {
        const unsigned px = (unsigned)(pb + (t / 3) * gm.PW + (t % 3));
        baddr[t][j] = px * ROW_BYTES + ((((unsigned)g) ^ ((px >> 2) & 3u)) * 16u);
      }
    }
  };
  consumer_setup();

  const unsigned fa_base = (unsigned)((wc * (TC * 32) + l32) * ROW_BYTES);
  const unsigned sl0 = (((unsigned)g) ^ rsw) * 16u, sl1 = ((2u + (unsigned)g) ^ rsw) * 16u;
  floatx16 acc[TC][TP];
  u32x4 fa0[TC], fb0[TP], fa1[TC], fb1[TP];

  asm volatile("s_waitcnt vmcnt(%0)" :: "n"((NST - 1) * LA) : "memory");     // the first patch and the first step have landed
  __builtin_amdgcn_s_barrier();
  {
    const unsigned char* sa = ring + fa_base + sl0;
#pragma unroll
    for (int i = 0; i < TC; ++i) fa0[i] = *(const u32x4*)(sa + i * (32 * ROW_BYTES));
#pragma unroll
    for (int j = 0; j < TP; ++j) fb0[j] = *(const u32x4*)(patch + baddr[0][j]);
  }

  const bool vec_ok = ((a.y_ld | a.y_coff) & 3) == 0 && (((uintptr_t)a.y & 7) == 0) &&
                      (!a.res || (((a.res_ld | a.res_coff) & 3) == 0 && (((uintptr_t)a.res & 7) == 0)));
  const bool is_silu = a.act == OCTO_ACT_SILU;
  const float act_lo = a.act == OCTO_ACT_RELU ? 0.0f : -INFINITY;

  bool more = true;
  // One K step = kernel tap TAP of the current slice.  The step's 2 x TC x TP MFMAs run in two halves (channels 0..15 and
  // 16..31 of the slice); one operand fragment read, or one piece of the loader, is issued after every MFMA, so that
  // the matrix pipe always has its next instruction waiting: the fragments of the second half during the first half,
  // and after the barrier those of the next step's first half (next tap, next slice or next tile) plus the refill of
  // the ring stage everyone has finished reading.
  auto step = [&](auto tapc, const bool last_of_tile) __attribute__((always_inline)) {
    constexpr int TAP = decltype(tapc)::value;
    constexpr int NEXT = (TAP + 1) % N_TAPS;
    constexpr int LTAP = (TAP + NST) % N_TAPS;         // the loader's tap: NST steps ahead
    // loads still allowed in flight when the next step's operands must have landed: those of the NST - 2 steps after it
    constexpr int IN_FLIGHT = nlt((TAP + 2) % N_TAPS) + (NST > 3 ? nlt((TAP + 3) % N_TAPS) : 0);
    constexpr bool PATCH = LTAP >= NST && LTAP < NST + 4;
    constexpr int PASS0 = PATCH ? PPT * (LTAP - NST) : -PPT;
    constexpr int LAST = TC * TP - 1;
    auto slot = [](int i) constexpr { return TC + TP + i < LAST ? TC + TP + i : LAST; };    // MFMA after which load i of the step is issued
    {
      const unsigned char* sa = ring + (unsigned)rd * STAGE_BYTES + fa_base + sl1;
      const unsigned char* sb = patch + (unsigned)cbuf * (unsigned)gm.patch_bytes;
#pragma unroll
      for (int m = 0; m < TC * TP; ++m) {
        acc[m / TP][m % TP] = Mfma16<T>::run(fa0[m / TP], fb0[m % TP], acc[m / TP][m % TP]);
        if (m < TC) fa1[m] = *(const u32x4*)(sa + m * (32 * ROW_BYTES));
        else if (m < TC + TP) fb1[m - TC] = *(const u32x4*)(sb + (baddr[TAP][m - TC] ^ 32u));
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // this wavefront has everything it needs of stage rd (and, at the last tap, of the slice's patch) in registers;
    // the next step's loads (issued NST - 1 steps ago) have landed once at most (NST - 2) steps' loads are outstanding
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_waitcnt vmcnt(%0)" :: "n"(IN_FLIGHT) : "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    const int st_free = rd;
    rd = rd + 1 == NST ? 0 : rd + 1;
    if (TAP == N_TAPS - 1) {
      cbuf ^= 1;                           // next slice: the other patch buffer
      if (last_of_tile) {                  // uniform: the fragments read below belong to the workgroup's next tile
        ct = next_valid(ct + gridDim.x);
        more = ct < t_end;
        if (more) consumer_setup();
      }
    }
    {
      int poff[PPT];
#pragma unroll
      for (int i = 0; i < PPT; ++i) poff[i] = PATCH ? patch_offset(PASS0 + i) : OOB;
      __builtin_amdgcn_sched_barrier(0);
      const unsigned char* sa = ring + (unsigned)rd * STAGE_BYTES + fa_base + sl0;
      const unsigned char* sb = patch + (unsigned)cbuf * (unsigned)gm.patch_bytes;
#pragma unroll
      for (int m = 0; m < TC * TP; ++m) {
        acc[m / TP][m % TP] = Mfma16<T>::run(fa1[m / TP], fb1[m % TP], acc[m / TP][m % TP]);
        if (m < TC) fa0[m] = *(const u32x4*)(sa + m * (32 * ROW_BYTES));
        else if (m < TC + TP) fb0[m - TC] = *(const u32x4*)(sb + baddr[NEXT][m - TC]);
#pragma unroll
        for (int i = 0; i < LA; ++i)
          if (m == slot(i)) issue_weight(st_free, LTAP, i);
#pragma unroll
        for (int i = 0; i < PPT; ++i)
          if (PATCH && m == slot(LA + i)) issue_patch_pass(PASS0 + i, poff[i]);
        if (LTAP == N_TAPS - 1 && m == slot(LA)) issue_bias();
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    loader_advance(LTAP);
  };

  while (more) {
#pragma unroll
    for (int i = 0; i < TC; ++i)
#pragma unroll
      for (int j = 0; j < TP; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    const int ec0 = c0;                    // origin of the tile whose accumulators are being filled (for its epilogue)
    int epix[TP];
#pragma unroll
    for (int j = 0; j < TP; ++j) epix[j] = pix[j];

    for (int sl = 0; sl < n_slices; ++sl) {
      const bool last = sl + 1 == n_slices;
      step(std::integral_constant<int, 0>{}, false); step(std::integral_constant<int, 1>{}, false); step(std::integral_constant<int, 2>{}, false);
      step(std::integral_constant<int, 3>{}, false); step(std::integral_constant<int, 4>{}, false); step(std::integral_constant<int, 5>{}, false);
      step(std::integral_constant<int, 6>{}, false); step(std::integral_constant<int, 7>{}, false); step(std::integral_constant<int, 8>{}, last);
    }

    // ---- epilogue of the finished tile, from registers: a lane holds one pixel of each 32 x 32 block and 4 groups of 4
    // consecutive channels; the tile's bias is in sBias[cpar] (its loads were among those already awaited)
    const float* bias_s = sBias + cpar * THREADS;
    with_epilogue_mode(a.res ? a.res_mode : OCTO_RES_NONE, is_silu, [&](auto res_c, auto silu_c) __attribute__((always_inline)) {
    constexpr int RES = decltype(res_c)::value;
    constexpr bool SILU = decltype(silu_c)::value;
#pragma unroll
    for (int j = 0; j < TP; ++j) {
      if (epix[j] < 0) continue;
      const size_t p = (size_t)epix[j];
#pragma unroll
      for (int i = 0; i < TC; ++i) {
        const int cblk = wc * (TC * 32) + i * 32 + g * 4;
        const T* rp = RES != OCTO_RES_NONE ? (const T*)a.res + p * a.res_ld + a.res_coff + ec0 + cblk : nullptr;
        T* yp = (T*)a.y + p * a.y_ld + a.y_coff + ec0 + cblk;
        if (vec_ok && ec0 + cblk + 28 <= a.Cout) {
          floatx4 rv[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) rv[q] = floatx4{0.f, 0.f, 0.f, 0.f};
          if (rp) {
#pragma unroll
            for (int q = 0; q < 4; ++q) rv[q] = load4<T>(rp + q * 8);
          }
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const floatx4 b4 = *(const floatx4*)&bias_s[cblk + q * 8];
            floatx4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = acc[i][j][q * 4 + e];
            v = finish4<RES, SILU>(v, b4, rv[q], act_lo);
            store4<T>(yp + q * 8, v);
          }
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int cl = cblk + q * 8 + e;
              if (ec0 + cl < a.Cout) {
                const float r = rp ? (float)rp[q * 8 + e] : 0.f;
                const float t = finish1<RES, SILU>(acc[i][j][q * 4 + e], bias_s[cl], r, act_lo);
                yp[q * 8 + e] = (T)t;
              }
            }
          }
        }
        __builtin_amdgcn_sched_barrier(0);   // one block at a time: keeps the epilogue's register demand low
      }
    }
    });
    cpar ^= 1;
  }
  // the loaders ran NST steps past the end (out-of-range offsets: zeros): let them land before the workgroup's LDS is released
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Tile shape for a W-wide image and a tile of BP pixels: a divisor TW of W (at most 64) with TH = BP / TW; among the
// shapes that fill the tile to within 10 % of the best one, the one with the smallest patch.  False if no shape fills
// at least 3/4 of the tile or the patch needs more than BP / 32 passes of 4 KB.
inline bool big_geometry(int H, int W, int tiles_c, int BP, BigGeom* gm) {
  int best_px = 0;
  for (int tw = W < 64 ? W : 64; tw >= 4; --tw)
    if (W % tw == 0 && (BP / tw) * tw > best_px) best_px = (BP / tw) * tw;
  if (best_px * 4 < BP * 3) return false;
  int best_tw = 0, best_patch = 1 << 30;
  for (int tw = W < 64 ? W : 64; tw >= 4; --tw) {
    if (W % tw) continue;
    const int th = BP / tw;
    if (th * tw * 10 < best_px * 9) continue;
    const int patch = (th + 2 + 2 * ((th - 1 + H - 1) / H)) * (tw + 2);
    if (patch < best_patch) { best_patch = patch; best_tw = tw; }
  }
  gm->TW = best_tw; gm->TH = BP / best_tw; gm->PW = best_tw + 2; gm->tiles_x = W / best_tw;
  // most patch rows a tile can need: its TH rows, one above and below, and two more per image boundary inside it
  const int crossings = (gm->TH - 1 + H - 1) / H;
  const int rows = gm->TH + 2 + 2 * crossings;
  const int vecs = rows * gm->PW * 4;
  gm->PL = (vecs + THREADS - 1) / THREADS;
  if (gm->PL > BP / 32) return false;
  gm->patch_bytes = gm->PL * 4096;
  gm->div_tw = make_fastdiv((unsigned)gm->TW); gm->div_pw = make_fastdiv((unsigned)gm->PW);
  gm->div_h = make_fastdiv((unsigned)H); gm->div_hp2 = make_fastdiv((unsigned)(H + 2));
  gm->div_tc = make_fastdiv((unsigned)tiles_c); gm->div_tx = make_fastdiv((unsigned)gm->tiles_x);
  return true;
}

// dynamic LDS of a configuration: weight ring, two patch buffers, two bias buffers, the lanes' patch offsets, the dump
inline size_t big_lds_bytes(int BC, int BP, int NST, const BigGeom& gm) {
  return (size_t)NST * ((BC + 63) / 64 * 64) * 64 + 2 * (size_t)gm.patch_bytes + 2 * THREADS * sizeof(float) +
         (size_t)(BP / 32) * THREADS * sizeof(int) + 4096;
}

// Compiled once per storage type so that the two build in parallel: convbig_f16.hip and convbig_bf16.hip define
// OCTO_BIG_ONLY_<type> and include this file; compiled as itself it holds only the entry point below.
#ifndef OCTO_CONV_NO_LAUNCHERS
namespace {

template <typename T, int TC, int TP, int WC, int NST>
hipError_t launch_big_cfg(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm) {
  constexpr int BC = TC * WC * 32, BP = TP * (4 / WC) * 32;
  const int tiles_c = (a.Cout + BC - 1) / BC;
  BigGeom gm{};
  if (!big_geometry(a.H, a.W, tiles_c, BP, &gm)) return hipErrorNotSupported;
  const long long n_rows = (long long)a.n * a.H;
  const long long tiles = ((n_rows + gm.TH - 1) / gm.TH) * gm.tiles_x * tiles_c;
  if (tiles <= 0) return hipSuccess;
  if (tiles >= 0x7FFFFFF0LL || n_rows * a.W >= 0x7FFFFFFFLL) return hipErrorNotSupported;
  // a patch is addressed with 32-bit byte offsets from the first image it touches
  if (((long long)(gm.TH + 2) / a.H + 3) * a.H * a.W * a.x_ld * 2 > 0x7FFFFFF0LL) return hipErrorNotSupported;
  const size_t lds = big_lds_bytes(BC, BP, NST, gm);
  if (lds > 160 * 1024) return hipErrorNotSupported;
  static bool attr_set = false;            // more than 64 KB of dynamic LDS needs the attribute (once per instantiation)
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)conv3x3_big_kernel<T, TC, TP, WC, NST>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    (void)hipGetLastError();
    attr_set = true;
  }
  if (kernel_id) *kernel_id = 1700000000 + (BP / 512) * 1000000 + BC * 1000 + gm.TW;
  long long grid = (tiles + 7) / 8 * 8;
  const long long cap = ((long long)num_cu + 7) / 8 * 8;
  if (grid > cap) grid = cap;
  if (tm.start && tm.stop)
    hipExtLaunchKernelGGL((conv3x3_big_kernel<T, TC, TP, WC, NST>), dim3((unsigned)grid), dim3(THREADS), (unsigned)lds, s, tm.start, tm.stop, 0, a, gm);
  else
    hipLaunchKernelGGL((conv3x3_big_kernel<T, TC, TP, WC, NST>), dim3((unsigned)grid), dim3(THREADS), (unsigned)lds, s, a, gm);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_big_typed(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm) {
  // channel tile: the one that pads the channel count least, ties to the larger
  int best_bc = 0, best_pad = 1 << 30;
  for (int bc : {256, 192, 96}) {
    const int pad = (a.Cout + bc - 1) / bc * bc;
    if (pad < best_pad) { best_pad = pad; best_bc = bc; }
  }
  if (best_pad * 4 > a.Cout * 5) return hipErrorNotSupported;     // more than a fifth of the MFMAs would be padding
  // enough tiles to give every compute unit two rounds (below that the general kernel's smaller tiles spread better)
  const long long m_hint = (long long)(a.n_hint > 0 && a.n_hint < a.n ? a.n_hint : a.n) * a.H * a.W;
  const long long tiles_hint = m_hint / (best_bc == 96 ? 512 : 256) * ((a.Cout + best_bc - 1) / best_bc);
  if (tiles_hint < 2LL * num_cu) return hipErrorNotSupported;
  // measured on MI355X: 128 channels x 512 pixels (and 64 x 512) do not beat the general kernel, 96 x 512 does
  switch (best_bc) {
    case 256: return launch_big_cfg<T, 4, 4, 2, 4>(a, num_cu, s, kernel_id, tm);
    case 192: return launch_big_cfg<T, 3, 4, 2, 4>(a, num_cu, s, kernel_id, tm);
    default: return launch_big_cfg<T, 3, 4, 1, 4>(a, num_cu, s, kernel_id, tm);       // 96 channels x 512 pixels
  }
}

}  // namespace

#if defined(OCTO_BIG_ONLY_F16)
hipError_t launch_big_f16(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm) { return launch_big_typed<_Float16>(a, num_cu, s, kernel_id, tm); }
#elif defined(OCTO_BIG_ONLY_BF16)
hipError_t launch_big_bf16(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm) { return launch_big_typed<__bf16>(a, num_cu, s, kernel_id, tm); }
#else
hipError_t launch_big_f16(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm);
hipError_t launch_big_bf16(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm);

// hipErrorNotSupported when the layer does not fit this kernel (the caller then takes the general kernel).
hipError_t launch_conv3x3_big(int dtype, const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, ConvTiming tm) {
  if (dtype != OCTO_F16 && dtype != OCTO_BF16) return hipErrorNotSupported;
  if (a.out_f32 || a.pair_view || a.kh != 3 || a.kw != 3 || a.stride_h != 1 || a.stride_w != 1 || a.pad_h != 1 || a.pad_w != 1) return hipErrorNotSupported;
  if (a.Cin % 32 || a.x_ld % 8 || a.x_coff % 8 || ((uintptr_t)a.x & 15) || a.Cout < 80) return hipErrorNotSupported;
  if (a.Ho != a.H || a.Wo != a.W) return hipErrorNotSupported;
  switch (dtype) {
    case OCTO_F16: return launch_big_f16(a, num_cu, s, kernel_id, tm);
    case OCTO_BF16: return launch_big_bf16(a, num_cu, s, kernel_id, tm);
  }
  return hipErrorNotSupported;
}
#endif   // the main translation unit
#endif   // launchers

}  // namespace octo
