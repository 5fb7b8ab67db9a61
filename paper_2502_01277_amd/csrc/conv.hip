// Convolution as an implicit GEMM on the CDNA4 matrix cores.
//
//   y[n,p,q,k] = act(bias[k] + sum_{r,s,c} x[n, p*stride + r - pad, q*stride + s - pad, c] * w[k,r,s,c]  (+ residual))
// (vertical and horizontal stride / padding are separate arguments: a 3-channel first layer is run on the
// pixel-pair view of a 4-channel-padded input, see pipeline.hip)
//
// GEMM view: rows = output channels (weights, [Cout][K] with K = kh*kw*Cin contiguous),
// columns = output pixels (gathered on the fly from the NHWC input), reduction = K.
// One workgroup = 4 wavefronts (256 lanes) computes a BC x BP tile with
// v_mfma_f32_32x32x16 (fp16 / bf16) or v_mfma_f32_32x32x2 (fp32).  Operands reach LDS in one of two ways: straight
// from global memory (buffer loads with the LDS bit, a ring of stages, one barrier per K step; the path of all layers
// with more than 32 output channels), or through registers (double buffered; 3-channel first layers, whose gather is
// element-wise, and layers with up to 32 output channels).  A tile row is 64 or 128 bytes of K; its 16-byte vectors
// are XOR-swizzled so that both the fills and the MFMA operand reads (16 bytes per lane) are bank-conflict free.
//
// The inner loop is kept nearly free of vector-ALU work, which would otherwise
// starve the matrix cores: operands are fetched with buffer loads whose 32-bit
// offsets are "row offset + tap offset", an out-of-image tap gets an offset beyond
// the buffer range so the hardware returns zeros, and the weight offsets advance
// through the scalar offset operand.
//
// The grid is persistent: workgroups stride over the tile list, whose length may
// depend on an item count that lives in device memory (a variable number of ROIs),
// so no host round trip is needed.
#include "octo_internal.h"
#include "mfma_common.h"
#include <hip/hip_ext.h>

namespace octo {

// BC: output channels per tile, BP: pixels per tile, WC x WP: wavefront grid (WC * WP == 4),
// KV: 16-byte vectors per tile row and K step (one K step = KV*16 bytes of K per row),
// D: K steps whose global loads are in flight in registers (even), MINB: workgroups per CU to fit registers for.
// DMA: operands go global -> LDS directly (buffer loads with the LDS bit), D K-steps ahead, into a ring of D + 1 LDS
// stages; no registers are spent on staging and no LDS store instructions are issued.  The loads are issued from
// inline assembly (the wave's LDS destination is base M0 + lane * 16), and their completion is awaited with explicit
// vmcnt waits whose counts rely on every wave issuing the same number of loads per K step.  M0 is reserved by the
// compiler (it writes M0 immediately before each of its own uses), so setting it inside the asm statement is safe.
template <typename T, int BC, int BP, int WC, int WP, int KV, int D, int MINB, bool VEC, bool DMA = false>
__global__ __launch_bounds__(THREADS, MINB) void conv_mfma_kernel(const ConvArgs a) {
  using E = Elem<T>;
  constexpr int VN = E::N;
  constexpr int ES = (int)sizeof(T);
  constexpr int BK = KV * VN;            // elements per K step
  constexpr int ROWV = KV;               // LDS row pitch in vectors; the vector slot of a row is XOR-swizzled (below)
  constexpr int RPW = 16 / KV;           // tile rows per 256 bytes of LDS (one pass over all banks)
  static_assert(KV == 4 || KV == 8 || KV == 16, "swizzle assumes 64-, 128- or 256-byte rows");
  constexpr int RP = THREADS / KV;       // tile rows covered by one pass of the 256 loader lanes
  constexpr int TC = BC / WC / 32;       // 32x32 blocks per wavefront along channels
  constexpr int TP = BP / WP / 32;
  constexpr int LA = (BC + RP - 1) / RP; // vectors per lane per K step (weights)
  constexpr int LB = BP / RP;            // (pixels)
  static_assert(DMA || D % 2 == 0, "pipeline depth must be even");
  static_assert(WC * WP == 4 && TC >= 1 && TP >= 1 && LB >= 1 && BP % RP == 0 && BC % 32 == 0, "tile shape");
  static_assert(!DMA || (VEC && BC % RP == 0), "direct-to-LDS loads need whole passes of all lanes");
  constexpr int NST = DMA ? D + 1 : 2;   // LDS stages
  constexpr int STAGE_VECS_OP = (BC + BP) * ROWV;
  constexpr int NL = LA + LB;            // load instructions per wave and K step

  // operand tiles; after the K loop the same memory stages the output tile as [pixel][channel] so that it can be
  // written with 16-byte stores that cover whole cache lines
  constexpr int OPITCH = BC * ES + 16;                                    // bytes per staged output row
  constexpr int OPER_VECS = NST * (BC + BP) * ROWV;                       // operand tiles, all stages
  constexpr int STAGE_VECS = BP * OPITCH / 16;                            // output tile
  constexpr bool STAGED = STAGE_VECS <= 4096;                             // stage outputs of up to 64 KB
  constexpr int SMEM_VECS = STAGED && STAGE_VECS > OPER_VECS ? STAGE_VECS : OPER_VECS;
  __shared__ u32x4 smem[SMEM_VECS];
  __shared__ float sBias[BC];
  __shared__ float sScale[ES == 1 ? BC : 1];       // 8-bit storage: factor on the accumulator, per output channel
  u32x4 (*sA)[BC][ROWV] = (u32x4 (*)[BC][ROWV])smem;
  u32x4 (*sB)[BP][ROWV] = (u32x4 (*)[BP][ROWV])(smem + 2 * BC * ROWV);

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
  // register path: a multiple of D (the host pads Kp to a multiple of 128 bytes); direct-to-LDS path: any count, and a
  // last step that runs past Kp multiplies zero-filled pixels
  const int nk = DMA ? (a.Kp + BK - 1) / BK : a.Kp / BK;
  const T* __restrict__ xg = (const T*)a.x + a.x_coff;
  const int HoWo = a.Ho * a.Wo;
  const long long img_elems = (long long)a.H * a.W * a.x_ld;

  const int ld_row = tid / KV;
  const int ld_kv = tid % KV;
  // Row r keeps its 16-byte vector v in slot v ^ ((r / RPW) % KV).  Sixteen lanes that write RPW whole rows, and sixteen
  // lanes that read the same logical vector of sixteen consecutive rows, then each touch a different 16-byte bank group.
  // 32 and THREADS / KV are multiples of RPW * KV, so the swizzle term depends only on the lane.
  const int wsw = ld_kv ^ ((ld_row / RPW) % KV);      // slot this lane writes
  // direct-to-LDS: the lane's slot is fixed by its lane id (ld_kv), so it fetches the vector that belongs there
  const int lkv = DMA ? wsw : ld_kv;                  // logical vector this lane fetches
  const int rsw = (l32 / RPW) % KV;                   // XOR term for this lane's fragment reads
  const bool vec_ok = ((a.y_ld | a.y_coff) & 3) == 0 && (!a.res || ((a.res_ld | a.res_coff) & 3) == 0);
  const bool is_silu = a.act == OCTO_ACT_SILU;
  const float act_lo = a.act == OCTO_ACT_RELU ? 0.0f : -INFINITY;

  // weights: one buffer for the whole packed matrix (padded, so never out of range)
  const long long w_bytes = (long long)a.w_rows * a.Kp * ES;
  const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)a.w, 0, (int)(w_bytes < BUF_MAX ? w_bytes : BUF_MAX), BUF_FLAGS);

  // Workgroups are handed to the eight dies in turn (workgroup b runs on die b % 8) and every die has its own L2.  The
  // tile list is therefore cut into eight contiguous chunks, one per die: tiles that share input rows (neighbouring
  // pixel tiles, and all channel tiles of the same pixels) then meet in one L2 instead of being fetched by every die.
  // The grid is a multiple of 8, so a workgroup stays on its chunk while it strides.
  const long long per_die = (n_tiles + 7) >> 3;
  for (long long t = blockIdx.x; t < per_die * 8; t += gridDim.x) {
    const long long tile = (t & 7) * per_die + (t >> 3);
    if (tile >= n_tiles) continue;
    const int tc = (int)(tile % tiles_c);
    const long long tp = tile / tiles_c;
    const int c0 = tc * BC;
    const long long p0 = tp * BP;

    // activations: a buffer that starts at the first image this tile touches, so that 32-bit offsets suffice
    const int img0 = (int)(p0 / HoWo);
    const long long rem_bytes = ((long long)(a.n - img0) * img_elems - a.x_coff) * ES;
    const __amdgpu_buffer_rsrc_t rsrc_x =
        __builtin_amdgcn_make_buffer_rsrc((void*)(xg + (long long)img0 * img_elems), 0, (int)(rem_bytes < BUF_MAX ? rem_bytes : BUF_MAX), BUF_FLAGS);

    // per-lane pixel rows of the gather: byte offset of the (possibly out-of-image) pixel of tap (0, 0) and the
    // sets of kernel rows / columns that fall inside the image (bit r: row r ok; bit 16+s: column s ok)
    int rowoff[LB];
    unsigned hw_ok[LB];
    int hi0[LB], wi0[LB];   // only used by the element-wise gather
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      const long long m = p0 + ld_row + RP * i;
      rowoff[i] = 0; hw_ok[i] = 0u; hi0[i] = -1000000; wi0[i] = 0;
      if (m < M) {
        // m < 2^31 (checked on the host): pixel -> (image, row, column) with precomputed reciprocals
        const unsigned mu = (unsigned)m;
        const unsigned img = a.HoWo_is_one ? mu : udiv(mu, a.magic_howo, a.shift_howo);
        const unsigned rem = mu - img * (unsigned)HoWo;
        const unsigned ho = a.Wo == 1 ? rem : udiv(rem, a.magic_wo, a.shift_wo);
        const unsigned wo = rem - ho * (unsigned)a.Wo;
        const int h0 = (int)ho * a.stride_h - a.pad_h, w0 = (int)wo * a.stride_w - a.pad_w;
        hi0[i] = h0; wi0[i] = w0;
        rowoff[i] = (int)((((long long)((int)img - img0) * a.H + h0) * a.W + w0) * a.x_ld) * ES;
        // kernel rows r with 0 <= h0 + r < H form the range [max(0, -h0), min(kh, H - h0)); same for columns
        const int rlo = h0 < 0 ? -h0 : 0, rhi = a.H - h0 < a.kh ? a.H - h0 : a.kh;
        const int slo = w0 < 0 ? -w0 : 0, shi = a.W - w0 < a.kw ? a.W - w0 : a.kw;
        const unsigned rm = rhi > rlo ? ((1u << rhi) - 1u) & ~((1u << rlo) - 1u) : 0u;
        const unsigned sm = shi > slo ? ((1u << shi) - 1u) & ~((1u << slo) - 1u) : 0u;
        hw_ok[i] = rm | (sm << 16);
      }
    }
    int woff[LA];
#pragma unroll
    for (int i = 0; i < LA; ++i) woff[i] = ((c0 + ld_row + RP * i) * a.Kp + lkv * VN) * ES;

    floatx16 acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; ++i)
#pragma unroll
      for (int j = 0; j < TP; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // Operands of K step KB.  Element k = KB*BK + lkv*VN of the reduction is channel c of tap (r, s):
    // k = (r*kw + s)*Cin + c; the two divisions use precomputed reciprocals (exact for k < 65536).
    __syncthreads();   // the previous tile's LDS reads are done
    if (tid < BC) sBias[tid] = a.bias[c0 + tid];     // bias is padded to a multiple of 128 channels
    if constexpr (ES == 1) { if (tid < BC) sScale[tid] = a.scale[c0 + tid]; }     // padded alike
    if constexpr (DMA) {
      // LDS byte address of this wave's 1 KB slice of pass 0 of stage 0 (lane l writes at + 16 l)
      const unsigned lds_wave = (unsigned)__builtin_amdgcn_readfirstlane((int)((unsigned)(uintptr_t)smem + (unsigned)wave * 1024u));
      constexpr unsigned STAGE_BYTES = STAGE_VECS_OP * 16, PASS_BYTES = RP * ROWV * 16, A_BYTES = BC * ROWV * 16;
#define OCTO_CONV_DMA(KB, ST)                                                                                       \
      {                                                                                                             \
        const unsigned sbase = lds_wave + (unsigned)(ST) * STAGE_BYTES;                                             \
        const int koff = (KB) * (BK * ES);                                                                          \
        _Pragma("unroll") for (int i = 0; i < LA; ++i)                                                              \
          asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"                  \
                       :: "s"(sbase + i * PASS_BYTES), "v"(woff[i]), "s"(rsrc_w), "s"(koff) : "memory");             \
        const unsigned k = (unsigned)(KB) * BK + lkv * VN;                                                          \
        const unsigned tap = __umulhi(k, a.magic_cin);                                                              \
        const int c = (int)(k - tap * a.Cin);                                                                       \
        const int r = a.kw == 1 ? (int)tap : (int)__umulhi(tap, a.magic_kw);                                        \
        const int s2 = (int)tap - r * a.kw;                                                                         \
        const int delta = ((r * a.W + s2) * a.x_ld + c) * ES;                                                       \
        const unsigned need = k < (unsigned)a.K ? ((1u << r) | (0x10000u << s2)) : 0xFFFFFFFFu;                     \
        _Pragma("unroll") for (int i = 0; i < LB; ++i) {                                                            \
          const int off = (hw_ok[i] & need) == need ? rowoff[i] + delta : OOB;                                      \
          asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"                   \
                       :: "s"(sbase + A_BYTES + i * PASS_BYTES), "v"(off), "s"(rsrc_x) : "memory");                  \
        }                                                                                                           \
      }
      int st_rd = 0, st_wr = D;          // ring positions: stage read in this step, stage filled for step kb + D
#pragma unroll
      for (int d = 0; d < D; ++d) OCTO_CONV_DMA(d, d)
      for (int kb = 0; kb < nk; ++kb) {
        // loads of the D - 1 later steps may stay in flight; those of step kb (issued before them) are complete
        asm volatile("s_waitcnt vmcnt(%0)" :: "n"((D - 1) * NL) : "memory");
        __builtin_amdgcn_s_barrier();    // everyone's part of step kb is in LDS, and everyone is done reading step kb - 1
        OCTO_CONV_DMA(kb + D, st_wr)     // refills the stage that step kb - 1 read; past the last step: zeros, never read
        const u32x4* pa = smem + st_rd * STAGE_VECS_OP;
        const u32x4* pb = pa + BC * ROWV;
        if constexpr (ES == 1) {
          // 8-bit operands: one instruction reduces over 64 values, two vectors per lane and operand
#pragma unroll
          for (int kk = 0; kk < KV / 4; ++kk) {
            u32x4 fa[TC][2], fb[TP][2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
              for (int i = 0; i < TC; ++i) fa[i][h] = pa[(wc * (BC / WC) + i * 32 + l32) * ROWV + ((kk * 4 + h * 2 + g) ^ rsw)];
#pragma unroll
              for (int j = 0; j < TP; ++j) fb[j][h] = pb[(wp * (BP / WP) + j * 32 + l32) * ROWV + ((kk * 4 + h * 2 + g) ^ rsw)];
            }
#pragma unroll
            for (int i = 0; i < TC; ++i)
#pragma unroll
              for (int j = 0; j < TP; ++j) acc[i][j] = E::mfma2(fa[i][0], fa[i][1], fb[j][0], fb[j][1], acc[i][j]);
          }
        } else {
#pragma unroll
        for (int kk = 0; kk < KV / 2; ++kk) {
          u32x4 fa[TC], fb[TP];
#pragma unroll
          for (int i = 0; i < TC; ++i) fa[i] = pa[(wc * (BC / WC) + i * 32 + l32) * ROWV + ((kk * 2 + g) ^ rsw)];
#pragma unroll
          for (int j = 0; j < TP; ++j) fb[j] = pb[(wp * (BP / WP) + j * 32 + l32) * ROWV + ((kk * 2 + g) ^ rsw)];
#pragma unroll
          for (int i = 0; i < TC; ++i)
#pragma unroll
            for (int j = 0; j < TP; ++j) acc[i][j] = E::mfma(fa[i], fb[j], acc[i][j]);
        }
        }
        st_rd = st_rd + 1 == NST ? 0 : st_rd + 1;
        st_wr = st_wr + 1 == NST ? 0 : st_wr + 1;
      }
#undef OCTO_CONV_DMA
      // the loads issued past the last step still write (zeros) into the ring: drain them before the memory is reused
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
    } else {
    u32x4 ra[D][LA], rb[D][LB];
#define OCTO_CONV_LOAD(KB, SL)                                                                                      \
    {                                                                                                               \
      _Pragma("unroll") for (int i = 0; i < LA; ++i)                                                                \
        if (BC % RP == 0 || ld_row + RP * i < BC)                                                                   \
          ra[SL][i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, woff[i], (KB) * (BK * ES), 0);                  \
      if (VEC) {                                                                                                    \
        const unsigned k = (unsigned)(KB) * BK + lkv * VN;                                                          \
        const unsigned tap = __umulhi(k, a.magic_cin);                                                              \
        const int c = (int)(k - tap * a.Cin);                                                                       \
        const int r = a.kw == 1 ? (int)tap : (int)__umulhi(tap, a.magic_kw);                                        \
        const int s2 = (int)tap - r * a.kw;                                                                         \
        const int delta = ((r * a.W + s2) * a.x_ld + c) * ES;                                                       \
        const unsigned need = k < (unsigned)a.K ? ((1u << r) | (0x10000u << s2)) : 0xFFFFFFFFu;                     \
        _Pragma("unroll") for (int i = 0; i < LB; ++i) {                                                            \
          const int off = (hw_ok[i] & need) == need ? rowoff[i] + delta : OOB;                                      \
          rb[SL][i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, off, 0, 0);                                     \
        }                                                                                                           \
      } else {                                                                                                      \
        const int kbase = (KB) * BK + ld_kv * VN;                                                                   \
        _Pragma("unroll") for (int i = 0; i < LB; ++i) {                                                            \
          typedef T tv __attribute__((ext_vector_type(VN)));                                                        \
          tv pk;                                                                                                    \
          const T* rowp = xg + (long long)img0 * img_elems + rowoff[i] / ES;                                        \
          _Pragma("unroll") for (int e = 0; e < VN; ++e) {                                                          \
            const int k = kbase + e;                                                                                \
            T val = (T)0.0f;                                                                                        \
            if (k < a.K) {                                                                                          \
              const int tap = k / a.Cin, c = k - tap * a.Cin;                                                       \
              const int r = tap / a.kw, s2 = tap - r * a.kw;                                                        \
              if ((unsigned)(hi0[i] + r) < (unsigned)a.H && (unsigned)(wi0[i] + s2) < (unsigned)a.W)                \
                val = rowp[(r * a.W + s2) * a.x_ld + c];                                                            \
            }                                                                                                       \
            pk[e] = val;                                                                                            \
          }                                                                                                         \
          rb[SL][i] = __builtin_bit_cast(u32x4, pk);                                                                \
        }                                                                                                           \
      }                                                                                                             \
    }

    // nk is a multiple of D (the packed K extent is padded accordingly); loads past the end return zeros
#pragma unroll
    for (int d = 0; d < D; ++d) OCTO_CONV_LOAD(d, d)
    for (int kb0 = 0; kb0 < nk; kb0 += D) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        const int kb = kb0 + d;
        const int buf = d & 1;           // D is even, so kb & 1 == d & 1
        // operands of step kb: registers -> LDS
#pragma unroll
        for (int i = 0; i < LA; ++i)
          if (BC % RP == 0 || ld_row + RP * i < BC) sA[buf][ld_row + RP * i][wsw] = ra[d][i];
#pragma unroll
        for (int i = 0; i < LB; ++i) sB[buf][ld_row + RP * i][wsw] = rb[d][i];
        __syncthreads();
        OCTO_CONV_LOAD(kb + D, d)
#pragma unroll
        for (int kk = 0; kk < KV / 2; ++kk) {
          u32x4 fa[TC], fb[TP];
#pragma unroll
          for (int i = 0; i < TC; ++i) fa[i] = sA[buf][wc * (BC / WC) + i * 32 + l32][(kk * 2 + g) ^ rsw];
#pragma unroll
          for (int j = 0; j < TP; ++j) fb[j] = sB[buf][wp * (BP / WP) + j * 32 + l32][(kk * 2 + g) ^ rsw];
#pragma unroll
          for (int i = 0; i < TC; ++i)
#pragma unroll
            for (int j = 0; j < TP; ++j) acc[i][j] = E::mfma(fa[i], fb[j], acc[i][j]);
        }
      }
    }
#undef OCTO_CONV_LOAD
    }

    // epilogue: a lane holds pixel column l32 of each 32x32 block and 4 groups of 4 consecutive channels
    // (a launch with a second output tensor always takes the staged path: the host has checked its alignment)
    const bool staged = STAGED && !a.out_f32 && ((a.y_ld | a.y_coff) & (VN - 1)) == 0 && (((uintptr_t)a.y & 15) == 0);
    if (staged) __syncthreads();       // every wavefront is done reading the operand tiles
    // the arithmetic is compiled once per (residual mode, SiLU or not): see finish4
    with_epilogue_mode(a.res ? a.res_mode : OCTO_RES_NONE, is_silu, [&](auto res_c, auto silu_c) __attribute__((always_inline)) {
    constexpr int RES = decltype(res_c)::value;
    constexpr bool SILU = decltype(silu_c)::value;
#pragma unroll
    for (int j = 0; j < TP; ++j) {
      const int pl = wp * (BP / WP) + j * 32 + l32;          // pixel inside the tile
      const long long p = p0 + pl;
      if (p >= M) continue;
#pragma unroll
      for (int i = 0; i < TC; ++i) {
        const int cblk = wc * (BC / WC) + i * 32 + g * 4;     // channel (inside the tile) of this lane's group q = 0
        if (staged || (vec_ok && c0 + cblk + 28 <= a.Cout)) {
          // all four 4-channel groups are inside the tensor and 8/16-byte accesses are aligned (a staged tile may
          // carry channels past Cout; they are dropped when the tile is written out)
          floatx4 rv[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) rv[q] = floatx4{0.f, 0.f, 0.f, 0.f};
          if (RES != OCTO_RES_NONE) {
            const T* rp = (const T*)a.res + (size_t)p * a.res_ld + a.res_coff + c0 + cblk;
            if (vec_ok && c0 + cblk + 28 <= a.Cout) {
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const floatx4 r4 = load4<T>(rp + q * 8);
#pragma unroll
                for (int e = 0; e < 4; ++e) rv[q][e] = ES == 1 ? r4[e] * a.res_scale : r4[e];
              }
            } else {
#pragma unroll
              for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                  if (c0 + cblk + q * 8 + e < a.Cout) rv[q][e] = ES == 1 ? to_f32<T>(rp[q * 8 + e]) * a.res_scale : to_f32<T>(rp[q * 8 + e]);
            }
          }
          const size_t o = (size_t)p * a.y_ld + a.y_coff + c0 + cblk;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const floatx4 b4 = *(const floatx4*)&sBias[cblk + q * 8];
            floatx4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = ES == 1 ? acc[i][j][q * 4 + e] * sScale[cblk + q * 8 + e] : acc[i][j][q * 4 + e];
            v = finish4<RES, SILU>(v, b4, rv[q], act_lo);
            if (a.out_f32) { store4<float>((float*)a.y + o + q * 8, v); continue; }
            if constexpr (ES == 1) {
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] *= a.y_inv_scale;
            }
            if (staged) store4<T>((T*)((char*)smem + (size_t)pl * OPITCH) + cblk + q * 8, v);
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
                float r = 0.f, av = acc[i][j][q * 4 + e];
                if (RES != OCTO_RES_NONE) r = to_f32<T>(((const T*)a.res)[(size_t)p * a.res_ld + a.res_coff + c]);
                if constexpr (ES == 1) { r *= a.res_scale; av *= sScale[cl]; }
                float t = finish1<RES, SILU>(av, sBias[cl], r, act_lo);
                const size_t o = (size_t)p * a.y_ld + a.y_coff + c;
                if (a.out_f32) { ((float*)a.y)[o] = t; continue; }
                if constexpr (ES == 1) t *= a.y_inv_scale;
                ((T*)a.y)[o] = from_f32<T>(t);
              }
            }
          }
        }
      }
    }
    });
    if (staged) {
      // staged tile -> global memory: consecutive lanes write consecutive 16-byte pieces of a pixel's channels
      __syncthreads();
      constexpr int VPR = BC / VN;                 // 16-byte vectors per pixel row of the tile
      constexpr int PPP = THREADS / VPR;           // pixels per pass
      const int v = tid % VPR, pr = tid / VPR;
      const int c = c0 + v * VN;
#pragma unroll
      for (int ps = 0; ps < BP / PPP; ++ps) {
        const int pl = ps * PPP + pr;
        const long long p = p0 + pl;
        if (p < M && c < a.Cout) {
          const u32x4 val = *(const u32x4*)((const char*)smem + (size_t)pl * OPITCH + (size_t)v * 16);
          // two layers in one launch: a vector never straddles the split (a multiple of 8 channels)
          const bool second = a.split > 0 && c >= a.split;
          T* yp = second ? (T*)a.y2 + (size_t)p * a.y2_ld + a.y2_coff + (c - a.split) : (T*)a.y + (size_t)p * a.y_ld + a.y_coff + c;
          if (c + VN <= a.Cout) {
            *(u32x4*)yp = val;
          } else if constexpr (ES == 1) {
            typedef uint8_t bv __attribute__((ext_vector_type(16)));
            const bv b = __builtin_bit_cast(bv, val);
#pragma unroll
            for (int e = 0; e < VN; ++e) if (c + e < a.Cout) yp[e].bits = b[e];
          } else {
            typedef T tv __attribute__((ext_vector_type(VN)));
            const tv tvv = __builtin_bit_cast(tv, val);
#pragma unroll
            for (int e = 0; e < VN; ++e) if (c + e < a.Cout) yp[e] = tvv[e];
          }
        }
      }
    }
  }
}

// This file is compiled once per storage type, so that the types build in parallel: conv_f16.hip, conv_bf16.hip,
// conv_f32.hip and conv_f8.hip define OCTO_CONV_ONLY_<type> and include it; each then holds the kernel instances of
// its type behind one entry point (launch_general_<type>).  Compiled as itself it holds no kernel, only the dispatch
// (launch_conv) and the host helpers.
#ifndef OCTO_CONV_NO_LAUNCHERS
template <typename T, int BC, int BP, int WC, int WP, int KV, int D, int MINB, bool VEC, bool DMA = false>
static hipError_t launch_cfg(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm) {
  if (kernel_id) *kernel_id = conv_kernel_id(BC, BP, KV, MINB, VEC, DMA);
  const long long M = (long long)a.n * a.Ho * a.Wo;
  const long long tiles = ((M + BP - 1) / BP) * ((a.Cout + BC - 1) / BC);
  if (tiles <= 0) return hipSuccess;
  long long grid = (tiles + 7) / 8 * 8;          // a multiple of the die count (see the kernel's tile order)
  const long long cap = ((long long)num_cu * MINB + 7) / 8 * 8;
  if (grid > cap) grid = cap;
  // with timing events the dispatch itself carries them, so their difference is the kernel's own run time
  if (tm.start && tm.stop)
    hipExtLaunchKernelGGL((conv_mfma_kernel<T, BC, BP, WC, WP, KV, D, MINB, VEC, DMA>), dim3((unsigned)grid), dim3(THREADS), 0, s, tm.start, tm.stop, 0, a);
  else
    hipLaunchKernelGGL((conv_mfma_kernel<T, BC, BP, WC, WP, KV, D, MINB, VEC, DMA>), dim3((unsigned)grid), dim3(THREADS), 0, s, a);
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_typed(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm) {
  constexpr int VN = Elem<T>::N;
  const bool vec = (a.Cin % VN == 0) && (a.x_ld % VN == 0) && (a.x_coff % VN == 0) && (((uintptr_t)a.x & 15) == 0) &&
                   a.kh <= 15 && a.kw <= 15;
  // the tile shape is chosen for the expected number of items (any shape is correct for any count: the grid strides
  // over however many tiles the device-side count gives)
  const long long M = (long long)(a.n_hint > 0 && a.n_hint < a.n ? a.n_hint : a.n) * a.Ho * a.Wo;
  auto tiles = [&](int bc, int bp) { return ((M + bp - 1) / bp) * ((a.Cout + bc - 1) / bc); };
  if (!vec) {
    // element-wise gather (first layers with 3 input channels)
    if (a.Cout <= 32) return launch_cfg<T, 32, 128, 1, 4, 4, 2, 2, false>(a, num_cu, s, kernel_id, tm);
    return launch_cfg<T, 64, 128, 2, 2, 4, 2, 2, false>(a, num_cu, s, kernel_id, tm);
  }
  // Tile choice (measured on MI355X).  Up to 32 output channels: register-staged 32x128 tiles.  Otherwise operands
  // go straight into LDS with K steps of 128 bytes: 128x128 tiles where 128 channels per tile pad the channel count
  // no further than 64 do (192 = 3 x 64, but 2 x 128), 64x128 tiles for the middle ground (64x256 with 64-byte K steps
  // for very large, narrow layers), 64x64 tiles for layers with few output pixels.  How many tiles a shape must yield
  // depends on the length of the reduction.  A layer with a short K loop is dominated by start-up and epilogue and runs
  // fastest on the shape that spreads it over all compute units.  A long K loop is paced by the operand fetch from the
  // L2s, so the shape with the most arithmetic per fetched byte wins as soon as a quarter of the compute units get a
  // tile: alone it takes a little longer, but it moves half the bytes, and kernels of other streams use the rest of
  // the chip meanwhile (+4 % on the traffic cascade with four pipeline instances).
  if (a.Cout <= 32) return launch_cfg<T, 32, 128, 1, 4, 4, 2, 4, true>(a, num_cu, s, kernel_id, tm);
  const bool fits128 = a.Cout >= 96 && (a.Cout + 127) / 128 * 128 == (a.Cout + 63) / 64 * 64;
  // Very many pixels: 256-pixel tiles of 64 channels with 64-byte K steps, three workgroups per compute unit.  For
  // layers of at most 64 channels (store-bound first layers, wide early stages), and for short reductions - all
  // epilogue and memory traffic - whose channel count the 128-channel tile would pad (192 = 3 x 64): 192 -> 192 on
  // 32 x 160 x 160 runs 11 % faster than on 64x128 tiles; beyond K = 384 the larger K step wins.
  if (tiles(64, 256) >= 4 * num_cu && (a.Cout <= 64 || (!fits128 && a.Kp <= 384)))
    return launch_cfg<T, 64, 256, 1, 4, 4, 1, 3, true, true>(a, num_cu, s, kernel_id, tm);
  if (fits128 && tiles(128, 128) >= (a.Kp >= 1024 ? num_cu / 4 : 5 * num_cu / 4))
    return launch_cfg<T, 128, 128, 2, 2, 8, 1, 2, true, true>(a, num_cu, s, kernel_id, tm);
  if (tiles(64, 128) >= (a.Kp >= 512 ? num_cu / 4 : 9 * num_cu / 8))
    return launch_cfg<T, 64, 128, 2, 2, 8, 1, 3, true, true>(a, num_cu, s, kernel_id, tm);
  return launch_cfg<T, 64, 64, 2, 2, 8, 1, 4, true, true>(a, num_cu, s, kernel_id, tm);
}

// 8-bit floating point (E4M3) storage: the direct-to-LDS tile shapes only, so the input channels must come in whole
// 16-byte vectors.  Same choice of shape as for the 16-bit types; a K step is 128 (or 64) bytes of K as there, that is
// twice as many values.
#if defined(OCTO_CONV_ONLY_F8)
static hipError_t launch_f8(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm) {
  const bool vec = (a.Cin % 16 == 0) && (a.x_ld % 16 == 0) && (a.x_coff % 16 == 0) && (((uintptr_t)a.x & 15) == 0) && a.kh <= 15 && a.kw <= 15;
  if (!vec || !a.scale || a.pair_view) return hipErrorInvalidValue;
  const long long M = (long long)(a.n_hint > 0 && a.n_hint < a.n ? a.n_hint : a.n) * a.Ho * a.Wo;
  auto tiles = [&](int bc, int bp) { return ((M + bp - 1) / bp) * ((a.Cout + bc - 1) / bc); };
  const bool fits128 = a.Cout >= 96 && (a.Cout + 127) / 128 * 128 == (a.Cout + 63) / 64 * 64;
  if (fits128 && tiles(128, 128) >= (a.Kp >= 2048 ? num_cu / 4 : 5 * num_cu / 4))
    return launch_cfg<f8, 128, 128, 2, 2, 8, 1, 2, true, true>(a, num_cu, s, kernel_id, tm);
  if (a.Cout <= 64 && tiles(64, 256) >= 4 * num_cu) return launch_cfg<f8, 64, 256, 1, 4, 4, 1, 3, true, true>(a, num_cu, s, kernel_id, tm);
  if (tiles(64, 128) >= (a.Kp >= 1024 ? num_cu / 4 : 9 * num_cu / 8))
    return launch_cfg<f8, 64, 128, 2, 2, 8, 1, 3, true, true>(a, num_cu, s, kernel_id, tm);
  return launch_cfg<f8, 64, 64, 2, 2, 8, 1, 4, true, true>(a, num_cu, s, kernel_id, tm);
}
#endif

#if defined(OCTO_CONV_ONLY_F16)
hipError_t launch_general_f16(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm) { return launch_typed<_Float16>(a, num_cu, s, kernel_id, tm); }
#elif defined(OCTO_CONV_ONLY_BF16)
hipError_t launch_general_bf16(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm) { return launch_typed<__bf16>(a, num_cu, s, kernel_id, tm); }
#elif defined(OCTO_CONV_ONLY_F32)
hipError_t launch_general_f32(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm) { return launch_typed<float>(a, num_cu, s, kernel_id, tm); }
#elif defined(OCTO_CONV_ONLY_F8)
hipError_t launch_general_f8(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm) { return launch_f8(a, num_cu, s, kernel_id, tm); }
#else
hipError_t launch_general_f16(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm);
hipError_t launch_general_bf16(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm);
hipError_t launch_general_f32(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm);
hipError_t launch_general_f8(const ConvArgs& a, int num_cu, hipStream_t s, int* kernel_id, const ConvTiming& tm);

// kernel id of a conv tile configuration, decimal digits 1 BBB PPP K M V: channel tile, pixel tile, 16-byte vectors per
// K step, workgroups per CU the registers are sized for, vectorised gather
int conv_kernel_id(int bc, int bp, int kv, int minb, bool vec, bool dma) { return 1000000000 + bc * 1000000 + bp * 1000 + kv * 100 + minb * 10 + (vec ? 1 : 0) + (dma ? 2 : 0); }

size_t conv_packed_weight_elems(int cout, int kh, int kw, int cin, int dtype, int* kp_out, int* cout_pad_out) {
  const int vn = 16 / dtype_size(dtype);
  const int bk = 8 * vn;   // largest K step of any tile configuration
  const int K = kh * kw * cin;
  const int kp = (K + bk - 1) / bk * bk;
  const int cp = (cout + 127) / 128 * 128;
  if (kp_out) *kp_out = kp;
  if (cout_pad_out) *cout_pad_out = cp;
  return (size_t)kp * cp;
}

// Checks the limits the kernel relies on and fills the precomputed reciprocals.
bool conv_prepare(ConvArgs& a, int dtype) {
  if (a.Cin < 1 || a.kw < 1 || a.kh < 1 || a.stride_h < 1 || a.stride_w < 1 || a.Kp >= 65536 || a.w_rows < 1) return false;
  // a tile addresses its pixels with 32-bit byte offsets from the first image it touches: at most two images plus
  // 256 output pixels' worth of further images
  if ((2LL * a.H * a.W + 1024LL * a.stride_h * a.stride_w) * a.x_ld * dtype_size(dtype) > 0x7FFFFFF0LL) return false;
  if ((long long)a.n * a.Ho * a.Wo >= 0x7FFFFFFFLL) return false;
  // floor(n / d) = umulhi(n, magic) >> shift, exact for n < 2^31
  auto magic = [](unsigned d, unsigned* mg, unsigned* sh) {
    unsigned s = 0;
    while ((1ull << s) < d) ++s;
    const unsigned long long m = ((1ull << (32 + s)) + d - 1) / d;
    if (m >> 32) { *mg = (unsigned)(((1ull << (31 + s)) + d - 1) / d); *sh = s - 1; }
    else { *mg = (unsigned)m; *sh = s; }
  };
  a.HoWo_is_one = (a.Ho * a.Wo == 1) ? 1 : 0;
  if (!a.HoWo_is_one) magic((unsigned)(a.Ho * a.Wo), &a.magic_howo, &a.shift_howo);
  if (a.Wo > 1) magic((unsigned)a.Wo, &a.magic_wo, &a.shift_wo);
  a.magic_cin = a.Cin > 1 ? (unsigned)((1ull << 32) / (unsigned)a.Cin) + 1u : 0u;
  a.magic_kw = a.kw > 1 ? (unsigned)((1ull << 32) / (unsigned)a.kw) + 1u : 0u;
  return true;
}

hipError_t launch_conv(int dtype, const ConvArgs& a0, int num_cu, hipStream_t s, int* kernel_id, ConvTiming tm) {
  ConvArgs a = a0;
  if (!conv_prepare(a, dtype)) return hipErrorInvalidValue;
  if (a.split > 0) {
    // two layers in one launch: only the general kernel's staged epilogue knows the second output tensor
    const bool ok = (dtype == OCTO_F16 || dtype == OCTO_BF16) && a.y2 && !a.res && !a.out_f32 && !a.pair_view && !a.pool_y && a.split < a.Cout &&
                    ((a.split | a.Cout | a.y_ld | a.y_coff | a.y2_ld | a.y2_coff) & 7) == 0 && ((((uintptr_t)a.y | (uintptr_t)a.y2) & 15) == 0);
    if (!ok) return hipErrorNotSupported;
    return dtype == OCTO_F16 ? launch_general_f16(a, num_cu, s, kernel_id, tm) : launch_general_bf16(a, num_cu, s, kernel_id, tm);
  }
  const hipError_t es = launch_stem(dtype, a, num_cu, s, kernel_id, tm);
  if (es != hipErrorNotSupported || a.pool_y) return es;      // only the first-layer kernel can pool its own output
  // 3x3 layers with at most 64 output channels on wide images: the input patch of a tile lives in LDS (measured
  // +20% on 56x56x64 layers; the 8x32 pixel tile wastes lanes on narrow feature maps, and with more output channels
  // the general kernel's 128-channel tile re-uses the pixel operand enough)
  {
    const long long m_hint = (long long)(a.n_hint > 0 && a.n_hint < a.n ? a.n_hint : a.n) * a.Ho * a.Wo;
    if (a.Cout <= 64 && a.Wo >= 28 && (a.Wo + 31) / 32 * 32 * 7 <= a.Wo * 8 && m_hint >= 2LL * num_cu * 256) {
      const hipError_t e3 = launch_conv3x3_patch(dtype, a, num_cu, s, kernel_id, tm);
      if (e3 != hipErrorNotSupported) return e3;
    }
  }
  // wide 3x3 / stride-1 layers: large tiles with the input patch resident in LDS (the general kernel is paced by its
  // operand fetch there: every pixel is fetched once per kernel tap)
  {
    const hipError_t eb = launch_conv3x3_big(dtype, a, num_cu, s, kernel_id, tm);
    if (eb != hipErrorNotSupported) return eb;
  }
  switch (dtype) {
    case OCTO_F8: return launch_general_f8(a, num_cu, s, kernel_id, tm);
    case OCTO_F16: return launch_general_f16(a, num_cu, s, kernel_id, tm);
    case OCTO_BF16: return launch_general_bf16(a, num_cu, s, kernel_id, tm);
    case OCTO_F32: return launch_general_f32(a, num_cu, s, kernel_id, tm);
  }
  return hipErrorInvalidValue;
}
#endif   // the main translation unit
#endif   // launchers

}  // namespace octo
