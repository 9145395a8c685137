// 3x3 convolution (zero padding 1, stride 1 or 2) of a channels-last bf16 tensor as an implicit GEMM
// on the MFMA pipeline: out[(b, i, j), o] = sum over (tap, c) of x[b, i * stride + u - 1, j * stride + v - 1, c] *
// w[o, tap * C_in + c], tap = 3u + v.  Rows of the product are output pixels, its contraction runs over the
// nine taps times the input channels; the A operand is never materialised: every thread gathers its 16-byte
// pieces of the input (8 channels of one pixel, which lie inside one tap because C_in is a multiple of 8)
// straight from the tensor, with zeros where the tap falls into the padding.  Tiles are staged through
// registers into padded LDS tiles (double buffered) and multiplied with v_mfma_f32_32x32x16_bf16; the
// epilogue is the GEMM kernels' (bias, optional residual in the storage dtype).  This is the layer class of
// the frozen image encoder (Sec. 2.1, Sec. 2.3: the non-trainable layers that take tens to hundreds of
// milliseconds and are cut into partial batches, Sec. 5).
#include "dp_device.h"
#include "dp_kernels.h"
#include "dp_errors.h"
#include "dp_ktime.h"
#include "dp_gemm_epilogue.h"

#include <algorithm>

namespace dp {

struct ConvParams {
  const bf16* x; const bf16* w;
  int H, W, Cin, Ho, Wo, stride;
  int M, N, K;                   // output pixels, output channels, 9 * C_in
  int tiles_m, tiles_n, group_m;
  int taps_uniform;              // C_in % 64 == 0: a 64-deep k-tile lies inside one filter tap
  float* gn_partial;             // direct-to-LDS kernel: per-(256-pixel block, channel) sum and sum of squares of the output, or nullptr
  EpiParams<bf16> epi;
};

template <int BM, int BN, int WGM, int WGN>
struct ConvSmem {
  static constexpr int BK = 64, LD = BK + 8;
  static constexpr int WN = BN / WGN, C_LD = WN + 4;
  static constexpr size_t TILE_BYTES = 2 * (size_t)(BM + BN) * LD * 2;
  static constexpr size_t EPI_BYTES = (size_t)WGM * WGN * 32 * C_LD * 4;
  static constexpr size_t BYTES = TILE_BYTES > EPI_BYTES ? TILE_BYTES : EPI_BYTES;
};

template <int BM, int BN, int WGM, int WGN>
__global__ void __launch_bounds__(WGM * WGN * 64) conv3x3_bf16_kernel(const ConvParams p) {
  using S = ConvSmem<BM, BN, WGM, WGN>;
  constexpr int BK = S::BK, LD = S::LD, NT = WGM * WGN * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
  constexpr int A_PER = BM * BK / 8 / NT, B_PER = BN * BK / 8 / NT, ROWS_PER_PASS = NT / 8;
  static_assert((BM * BK / 8) % NT == 0 && (BN * BK / 8) % NT == 0 && NT % 8 == 0, "tile/threads mismatch");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16* As = reinterpret_cast<bf16*>(smem_raw);
  bf16* Bs = As + 2 * BM * LD;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, l32 = lane & 31;
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
  int tile_m, tile_n;
  tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, p.group_m, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // A thread stages chunk c8 (8 contraction values) of rows tid / 8 + i * ROWS_PER_PASS of both tiles.  The
  // output pixel behind an A row does not change along the contraction: decode it once.
  const int c8 = tid & 7, r0 = tid >> 3;
  int pix_b[A_PER], pix_h[A_PER], pix_w[A_PER];
  unsigned row_ok = 0;
#pragma unroll
  for (int i = 0; i < A_PER; ++i) {
    const int gm = m0 + r0 + i * ROWS_PER_PASS;
    row_ok |= (unsigned)(gm < p.M) << i;
    const int q = min(gm, p.M - 1);
    const int b = q / (p.Ho * p.Wo), rem = q - b * (p.Ho * p.Wo), ho = rem / p.Wo, wo = rem - ho * p.Wo;
    pix_b[i] = b; pix_h[i] = ho * p.stride - 1; pix_w[i] = wo * p.stride - 1;
  }

  bf16x8 ra[A_PER], rb[B_PER];
  unsigned oka = 0, okb = 0;
  auto load_global = [&](int kt) {
    const int k0 = kt * BK, gk = k0 + c8 * 8;
    int tap, ci;
    if (p.taps_uniform) { tap = k0 / p.Cin; ci = k0 - tap * p.Cin + c8 * 8; }      // tap: one scalar division per k-tile
    else { tap = gk / p.Cin; ci = gk - tap * p.Cin; }
    const bool kok = gk < p.K;
    tap = min(tap, 8); ci = min(ci, p.Cin - 8);
    const int u = tap / 3, v = tap - 3 * u;
    oka = 0; okb = 0;
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
      const int hi = pix_h[i] + u, wi = pix_w[i] + v;
      const bool ok = ((row_ok >> i) & 1) && kok && (unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W;
      const int hc = min(max(hi, 0), p.H - 1), wc = min(max(wi, 0), p.W - 1);      // a valid address in any case
      ra[i] = *reinterpret_cast<const bf16x8*>(p.x + (((size_t)pix_b[i] * p.H + hc) * p.W + wc) * p.Cin + ci);
      oka |= (unsigned)ok << i;
    }
#pragma unroll
    for (int i = 0; i < B_PER; ++i) {
      const int gn = n0 + r0 + i * ROWS_PER_PASS;
      rb[i] = *reinterpret_cast<const bf16x8*>(p.w + (size_t)min(gn, p.N - 1) * p.K + min(gk, p.K - 8));
      okb |= (unsigned)(gn < p.N && kok) << i;
    }
  };
  auto store_lds = [&](int buf) {
    bf16* as = As + buf * BM * LD;
    bf16* bs = Bs + buf * BN * LD;
#pragma unroll
    for (int i = 0; i < A_PER; ++i)
      *reinterpret_cast<bf16x8*>(as + (r0 + i * ROWS_PER_PASS) * LD + c8 * 8) = ((oka >> i) & 1) ? ra[i] : zero8();
#pragma unroll
    for (int i = 0; i < B_PER; ++i)
      *reinterpret_cast<bf16x8*>(bs + (r0 + i * ROWS_PER_PASS) * LD + c8 * 8) = ((okb >> i) & 1) ? rb[i] : zero8();
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nkt = (p.K + BK - 1) / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < nkt; ++kt) {
    const int buf = kt & 1;
    const bool more = kt + 1 < nkt;
    if (more) load_global(kt + 1);
    const bf16* as = As + buf * BM * LD;
    const bf16* bs = Bs + buf * BN * LD;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(as + (wm0 + i * 32 + l32) * LD + ks * 16 + 8 * g);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(bs + (wn0 + j * 32 + l32) * LD + ks * 16 + 8 * g);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(fa[i], fb[j], acc[i][j]);
    }
    if (more) store_lds(buf ^ 1);
    __syncthreads();
  }
  // the operand tiles are dead past the last barrier: each wave reuses its slice of LDS for the epilogue
  float* Cw = reinterpret_cast<float*>(smem_raw) + wave * 32 * S::C_LD;
  wave_epilogue<TM, TN, WN, S::C_LD>(acc, Cw, p.epi, m0 + wm0, n0 + wn0, lane);
}


// ------------------------------------------------------------------ direct-to-LDS pipeline
// The same product with the GEMM kernels' copy pipeline: tiles travel global -> LDS without passing through
// registers (buffer_load ... lds, 16 bytes per lane, every lane with an address of its own, so the gather of
// the input pixels costs nothing extra), three 64-deep k-tiles in flight, fragments fetched one k-step ahead,
// one fence-free barrier per k-tile.  A k-tile lies inside one filter tap (C_in a multiple of 64): its source
// address is the output pixel's base address plus an offset that is the same for the whole wave, and a lane
// whose tap falls into the padding aims its copy past the end of the buffer, which the hardware answers with
// zeros.  256 x 128 output tile, eight waves of 64 x 64 (or 256 x 256, eight waves of 128 x 64).  LDS tiles are unpadded with permuted 16-byte
// chunks, as in the GEMM kernels: chunk c of tile row r sits at position c ^ ((r >> 1) & 7).
template <int BK_, int BN_ = 128>
struct ConvDtlSmem {
  static constexpr int BM = 256, BN = BN_, BK = BK_, STAGES = 3, WGM = BN_ == 256 ? 2 : 4, WGN = BN_ == 256 ? 4 : 2;
  static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  static constexpr int WN = BN / WGN, C_LD = WN + 4;
  static constexpr size_t TILE_BYTES = (size_t)STAGES * STAGE;
  static constexpr size_t EPI_BYTES = (size_t)WGM * WGN * 32 * C_LD * 4;
  static constexpr size_t BYTES = TILE_BYTES > EPI_BYTES ? TILE_BYTES : EPI_BYTES;
};

// Chunk permutation of a tile row (BK / 8 chunks of 16 bytes): BK = 64: key (r >> 1) & 7; BK = 32: (r >> 2) & 3.
template <int BK> __device__ __forceinline__ int conv_key(int r) { return BK == 32 ? ((r >> 2) & 3) : ((r >> 1) & 7); }

// BK = 64: 144 KB of LDS, one workgroup per CU.  BK = 32: 72 KB, two workgroups per CU (MINW = 4 waves per SIMD), which hide
// each other's prologue and epilogue where the contraction is short (C_in = 128 .. 256).
// BN = 256 (BK = 32, 96 KB, eight waves of 128 x 64): half the weight-tile copies and A-fragment reads per FLOP, for layers
// with at least 256 output channels.
template <int BK_, int MINW, int BN_ = 128>
__global__ void __launch_bounds__(512, MINW) conv3x3_dtl_kernel(const ConvParams p, uint32_t x_bytes, uint32_t w_bytes) {
  using S = ConvDtlSmem<BK_, BN_>;
  constexpr int BM = S::BM, BN = S::BN, BK = S::BK, STAGES = S::STAGES, WGN = S::WGN, NW = S::WGM * S::WGN, KS = BK / 16, CPR = BK / 8;
  constexpr int WM = BM / S::WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
  constexpr int A_LOADS = S::A_BYTES / 1024 / NW, B_LOADS = S::B_BYTES / 1024 / NW, LOADS = A_LOADS + B_LOADS, PART_LAST = LOADS / KS;
  static_assert(S::A_BYTES % (1024 * NW) == 0 && S::B_BYTES % (1024 * NW) == 0 && STAGES == 3 && KS % 2 == 0, "pipeline shape");
  constexpr bool INTERLEAVE = BK == 64;
  constexpr uint32_t OUTSIDE = 0xFFFFFFF0u;          // an offset past any buffer this kernel accepts: the copy delivers zeros

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, l32 = lane & 31;
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
  int tile_m, tile_n;
  tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, p.group_m, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int nk = p.K / BK;

  const rsrc_t rx = make_rsrc(p.x, x_bytes), rw = make_rsrc(p.w, w_bytes);
  // per A piece of this wave: byte offset of the output pixel's own input pixel (tap centre) plus this lane's
  // chunk, and the 9-bit set of taps that fall inside the image for that pixel (empty for rows past M)
  int a_base[A_LOADS];
  unsigned a_taps[A_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int r = (wave * A_LOADS + j) * (512 / BK) + lane / CPR, pc = lane % CPR, c = pc ^ conv_key<BK>(r);
    const int gm = m0 + r, q = min(gm, p.M - 1);
    const int b = q / (p.Ho * p.Wo), rem = q - b * (p.Ho * p.Wo), ho = rem / p.Wo, wo = rem - ho * p.Wo;
    const int hc = ho * p.stride, wc = wo * p.stride;
    a_base[j] = (int)(2u * ((uint32_t)((b * p.H + hc) * p.W + wc) * (uint32_t)p.Cin + (uint32_t)c * 8u));
    unsigned m = 0;
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      const int hi = hc + tap / 3 - 1, wi = wc + tap % 3 - 1;
      m |= (unsigned)((unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W) << tap;
    }
    a_taps[j] = gm < p.M ? m : 0u;
  }
  uint32_t vb[B_LOADS];
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j) {
    const int r = (wave * B_LOADS + j) * (512 / BK) + lane / CPR, pc = lane % CPR, c = pc ^ conv_key<BK>(r);
    vb[j] = 2u * ((uint32_t)min(n0 + r, p.N - 1) * (uint32_t)p.K + (uint32_t)c * 8u);
  }
  // the k-tile whose copies are being issued: its tap and its wave-uniform source offset relative to the tap centre
  int it_tap = 0, it_c0 = 0, cur_tap = 0, cur_off = 0;
  auto next_tile = [&]() {
    const int u = (it_tap * 11) >> 5, v = it_tap - 3 * u;          // tap / 3, tap % 3 for tap < 9
    cur_tap = it_tap;
    cur_off = 2 * (((u - 1) * p.W + (v - 1)) * p.Cin + it_c0);
    it_c0 += BK;
    if (it_c0 == p.Cin) { it_c0 = 0; ++it_tap; }
  };
#define DPC_ISSUE_PART(t_, part_, parts_)                                                                             \
  {                                                                                                                   \
    unsigned char* st_ = smem_raw + ((t_) % STAGES) * S::STAGE;                                                       \
    _Pragma("unroll") for (int j = 0; j < A_LOADS; ++j)                                                               \
      if (j % (parts_) == (part_)) {                                                                                  \
        const uint32_t off_ = ((a_taps[j] >> cur_tap) & 1u) ? (uint32_t)(a_base[j] + cur_off) : OUTSIDE;              \
        async_copy_16B_buf(rx, off_, 0u, st_ + (wave * A_LOADS + j) * 1024);                                          \
      }                                                                                                               \
    _Pragma("unroll") for (int j = 0; j < B_LOADS; ++j)                                                               \
      if ((A_LOADS + j) % (parts_) == (part_))                                                                        \
        async_copy_16B_buf(rw, vb[j], (uint32_t)(t_) * (2u * BK), st_ + S::A_BYTES + (wave * B_LOADS + j) * 1024);    \
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  bf16x8 fa[2][TM], fb[2][TN];
#define DPC_FRAGS(st_, ks_, set_)                                                                                     \
  {                                                                                                                   \
    const bf16* as = reinterpret_cast<const bf16*>(smem_raw + (st_) * S::STAGE);                                      \
    const bf16* bs = reinterpret_cast<const bf16*>(smem_raw + (st_) * S::STAGE + S::A_BYTES);                         \
    _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                                                  \
      const int r = wm0 + i * 32 + l32;                                                                               \
      fa[set_][i] = *reinterpret_cast<const bf16x8*>(as + r * BK + (((2 * (ks_) + g) ^ conv_key<BK>(r)) * 8));         \
    }                                                                                                                 \
    _Pragma("unroll") for (int j2 = 0; j2 < TN; ++j2) {                                                               \
      const int r = wn0 + j2 * 32 + l32;                                                                              \
      fb[set_][j2] = *reinterpret_cast<const bf16x8*>(bs + r * BK + (((2 * (ks_) + g) ^ conv_key<BK>(r)) * 8));        \
    }                                                                                                                 \
  }
#define DPC_MFMAS(set_)                                                                                               \
  _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                                      \
    _Pragma("unroll") for (int j2 = 0; j2 < TN; ++j2) acc[i][j2] = mfma32(fa[set_][i], fb[set_][j2], acc[i][j2]);

  // pipeline: as in the GEMM kernels (all three buffers filled up front; k-tile t + 2 is copied, a few pieces per
  // k-step, while k-tile t is multiplied; every wait names exactly the copies it needs)
  for (int t = 0; t < STAGES && t < nk; ++t) { next_tile(); DPC_ISSUE_PART(t, 0, 1); }
  {
    const int y = min(nk, STAGES) - 1;
    if (y == 2) wait_vmcnt<2 * LOADS>();
    else if (y == 1) wait_vmcnt<LOADS>();
    else wait_vmcnt<0>();
  }
  barrier_nofence();
  DPC_FRAGS(0, 0, 0);
  for (int t = 0; t + 1 < nk; ++t) {
    const int st = t % STAGES;
    const bool refill = t >= 1 && t - 1 + STAGES < nk;
    if (refill) next_tile();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks + 1 < KS) {
        DPC_FRAGS(st, ks + 1, (ks + 1) & 1);
      } else {
        wait_lgkmcnt0();
        if (nk - 2 - t >= 1) wait_vmcnt<LOADS - PART_LAST>();
        else wait_vmcnt<0>();
        barrier_nofence();
        DPC_FRAGS((t + 1) % STAGES, 0, 0);
      }
      if (INTERLEAVE && ks + 1 < KS) {
        _Pragma("unroll") for (int q_ = 0; q_ < TM * TN; ++q_) {     // one fragment read behind each MFMA, as in the GEMM kernel
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      } else {
        __builtin_amdgcn_sched_barrier(0);
      }
      DPC_MFMAS(ks & 1);
      __builtin_amdgcn_sched_barrier(0);
      if (refill) DPC_ISSUE_PART(t - 1 + STAGES, ks, KS);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  {
    const int st = (nk - 1) % STAGES;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks + 1 < KS) DPC_FRAGS(st, ks + 1, (ks + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
      DPC_MFMAS(ks & 1);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#undef DPC_FRAGS
#undef DPC_MFMAS
#undef DPC_ISSUE_PART
  __syncthreads();   // every wave is done with the operand tiles before they are reused below
  float* Cw = reinterpret_cast<float*>(smem_raw) + wave * 32 * S::C_LD;
  if (!p.gn_partial) {
    wave_epilogue<TM, TN, WN, S::C_LD>(acc, Cw, p.epi, m0 + wm0, n0 + wn0, lane);
    return;
  }
  // Epilogue with the next GroupNorm's first pass folded in: bias, optional residual, bf16 store, and per channel the sum
  // and the sum of squares of the stored (rounded) values over this tile's 256 pixels.  A lane owns the same 8 columns in
  // every pass over the rows.  The sums are formed per 64-row band (one band per wave in the 256 x 128 tile, two in the
  // 256 x 256 one): the lane's rows in order, the 8 lanes with equal lane % 8 by a butterfly, the four bands of a column in
  // ascending order.  Nothing depends on timing, and both tile shapes associate the additions the same way, so they
  // produce the same bits.
  constexpr int NH = WM / 64;       // 64-row bands per wave
  static_assert(WN == 64 && WM % 64 == 0 && S::BYTES >= S::EPI_BYTES + (size_t)S::WGM * NH * WGN * 2 * 64 * 4, "statistics slab");
  const EpiParams<bf16>& e = p.epi;
  float* stat = reinterpret_cast<float*>(smem_raw + S::EPI_BYTES);      // [band][wave column][sum | sum of squares][64 columns], past the slabs
  float cs[8], cq[8];
  const int lc = (lane & 7) * 8, n = n0 + wn0 + lc;
  bf16x8 bv;
#pragma unroll
  for (int t = 0; t < 8; ++t) bv[t] = (bf16)0.f;
  if (e.bias && n < e.N) bv = *reinterpret_cast<const bf16x8*>(e.bias + n);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    if (i % 2 == 0) {
#pragma unroll
      for (int t = 0; t < 8; ++t) { cs[t] = 0.f; cq[t] = 0.f; }
    }
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) Cw[(8 * (r >> 2) + 4 * g + (r & 3)) * S::C_LD + j * 32 + l32] = acc[i][j][r];
    asm volatile("" ::: "memory");
#pragma unroll 1
    for (int it = 0; it < 4; ++it) {
      const int lr = it * 8 + (lane >> 3), m = m0 + wm0 + i * 32 + lr;
      if (m < e.M && n < e.N) {
        float v[8];
        *reinterpret_cast<f32x4*>(&v[0]) = *reinterpret_cast<const f32x4*>(&Cw[lr * S::C_LD + lc]);
        *reinterpret_cast<f32x4*>(&v[4]) = *reinterpret_cast<const f32x4*>(&Cw[lr * S::C_LD + lc + 4]);
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] += (float)bv[t];
        if (e.residual) {
          const bf16x8 rv = *reinterpret_cast<const bf16x8*>((const bf16*)e.residual + (size_t)m * e.ld_res + n);
#pragma unroll
          for (int t = 0; t < 8; ++t) v[t] += (float)rv[t];
        }
        bf16x8 o;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          o[t] = (bf16)v[t];
          const float f = (float)o[t];
          cs[t] += f; cq[t] = fmaf(f, f, cq[t]);
        }
        *reinterpret_cast<bf16x8*>(e.out + (size_t)m * e.ldo + n) = o;
      }
    }
    asm volatile("" ::: "memory");
    if (i % 2 == 1) {
      // the band is complete: lanes with equal lane % 8 hold the same columns
#pragma unroll
      for (int t = 0; t < 8; ++t) {
#pragma unroll
        for (int o = 8; o < 64; o <<= 1) { cs[t] += __shfl_xor(cs[t], o, 64); cq[t] += __shfl_xor(cq[t], o, 64); }
      }
      const int band = (wave / WGN) * NH + i / 2, wcol = wave % WGN;
      if (lane < 8) {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          stat[((band * WGN + wcol) * 2) * 64 + lane * 8 + t] = cs[t];
          stat[((band * WGN + wcol) * 2 + 1) * 64 + lane * 8 + t] = cq[t];
        }
      }
    }
  }
  __syncthreads();
  if (tid < 2 * BN) {
    const int which = tid / BN, c = tid % BN, wcol = c / 64, cc = c % 64;
    float sum = 0.f;
#pragma unroll
    for (int band = 0; band < S::WGM * NH; ++band) sum += stat[((band * WGN + wcol) * 2 + which) * 64 + cc];
    if (n0 + c < e.N) p.gn_partial[((size_t)tile_m * e.N + n0 + c) * 2 + which] = sum;
  }
}

template <int BK, int MINW, int BN = 128>
static int launch_conv_dtl(ConvParams& p, size_t x_bytes, size_t w_bytes, hipStream_t s) {
  using S = ConvDtlSmem<BK, BN>;
  p.tiles_m = (p.M + S::BM - 1) / S::BM; p.tiles_n = (p.N + S::BN - 1) / S::BN;
  const long n = (long)p.tiles_m * p.tiles_n, ppx = (n + 7) / 8;
  p.group_m = (int)std::max<long>(1, std::min<long>((ppx + p.tiles_n / 2) / p.tiles_n, p.tiles_m));
  auto kern = conv3x3_dtl_kernel<BK, MINW, BN>;
  if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)S::BYTES) != hipSuccess)
    return set_error(DP_EHIP, "hipFuncSetAttribute(conv) failed");
  hipLaunchKernelGGL(kern, dim3((unsigned)n), dim3(512), S::BYTES, s, p, (uint32_t)x_bytes, (uint32_t)w_bytes);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "conv launch failed");
}

template <int BM, int BN, int WGM, int WGN>
static int launch_conv_cfg(ConvParams& p, hipStream_t s) {
  using S = ConvSmem<BM, BN, WGM, WGN>;
  p.tiles_m = (p.M + BM - 1) / BM; p.tiles_n = (p.N + BN - 1) / BN;
  // whole tile-rows per XCD: the tiles that share a band of input pixels run on one L2
  const long n = (long)p.tiles_m * p.tiles_n, ppx = (n + 7) / 8;
  p.group_m = (int)std::max<long>(1, std::min<long>((ppx + p.tiles_n / 2) / p.tiles_n, p.tiles_m));
  auto kern = conv3x3_bf16_kernel<BM, BN, WGM, WGN>;
  if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)S::BYTES) != hipSuccess)
    return set_error(DP_EHIP, "hipFuncSetAttribute(conv) failed");
  hipLaunchKernelGGL(kern, dim3((unsigned)n), dim3(WGM * WGN * 64), S::BYTES, s, p);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "conv launch failed");
}

int launch_conv3x3(const ConvArgs& a, hipStream_t s) {
  if (a.dtype != BF16) return set_error(DP_EUNSUPPORTED, "conv3x3: bf16 storage only");
  if (a.B <= 0 || a.H <= 0 || a.W <= 0 || a.Cin <= 0 || a.Cout <= 0) return set_error(DP_EINVAL, "conv3x3: non-positive size");
  if (a.stride != 1 && a.stride != 2) return set_error(DP_EUNSUPPORTED, "conv3x3: stride must be 1 or 2");
  if (a.Cin % 8 || a.Cout % 8) return set_error(DP_EUNSUPPORTED, "conv3x3: channel counts must be multiples of 8");
  if (!a.x || !a.w || !a.y) return set_error(DP_EINVAL, "conv3x3: null operand");
  const void* ps[] = {a.x, a.w, a.y, a.bias, a.residual};
  for (const void* q : ps) if ((uintptr_t)q % 16) return set_error(DP_EALIGN, "conv3x3: operands must be 16-byte aligned");
  const int Ho = (a.H - 1) / a.stride + 1, Wo = (a.W - 1) / a.stride + 1;
  const long M = (long)a.B * Ho * Wo;
  if (M >= (1L << 31) - 512 || (long)9 * a.Cin >= (1L << 24)) return set_error(DP_EUNSUPPORTED, "conv3x3: too many output pixels or input channels");
  ConvParams p;
  p.x = (const bf16*)a.x; p.w = (const bf16*)a.w;
  p.H = a.H; p.W = a.W; p.Cin = a.Cin; p.Ho = Ho; p.Wo = Wo; p.stride = a.stride;
  p.M = (int)M; p.N = a.Cout; p.K = 9 * a.Cin;
  p.taps_uniform = a.Cin % 64 == 0;
  p.gn_partial = nullptr;
  if (a.gn_applied) *a.gn_applied = 0;
  if (a.gn_partial && !a.gn_applied) return set_error(DP_EINVAL, "conv3x3: gn_partial comes with gn_applied");
  EpiParams<bf16>& e = p.epi;
  e.M = p.M; e.N = p.N; e.out = (bf16*)a.y; e.ldo = a.Cout;
  e.out32 = nullptr; e.ldo32 = 0; e.accumulate = 0; e.partial = nullptr;
  e.bias = (const bf16*)a.bias; e.pre_out = nullptr; e.ld_pre = 0; e.act = 0;
  e.dact_pre = nullptr; e.ld_dact = 0; e.dact_kind = 0; e.gate = nullptr; e.gate_ld = 0; e.rows_per_batch = 1;
  e.residual = a.residual; e.ld_res = a.Cout; e.residual_f32 = 0; e.out_fused_f32 = 0;
  e.geglu = 0; e.geglu_inner = 0; e.geglu_u = nullptr; e.ld_geglu = 0; e.out_scale = 1.0f;
  const double by = 2.0 * ((double)a.B * a.H * a.W * a.Cin + (double)p.N * p.K + (double)M * a.Cout * (a.residual ? 2.0 : 1.0));
  KScope ks(KK_CONV, 2.0 * (double)M * p.N * p.K, by, s, p.M, p.N, p.K);
  // the direct-to-LDS kernel: k-tiles inside one tap, 32-bit byte offsets with room for the "outside" marker
  const size_t x_bytes = 2 * (size_t)a.B * a.H * a.W * a.Cin, w_bytes = 2 * (size_t)p.N * p.K;
  // (whether this kernel is taken depends on one sample's pixel count, not on the number of samples)
  if (a.Cin % 64 == 0 && a.Cout >= 64 && (long)Ho * Wo >= 1024 && x_bytes < (1ull << 31) && w_bytes < (1ull << 31) && !a.force_staged) {
    if (a.gn_partial && (Ho * Wo) % 256 == 0 && ((uintptr_t)a.gn_partial % 16) == 0) { p.gn_partial = a.gn_partial; *a.gn_applied = 1; }
    // measured on the layers of the 512 x 512 encoder: C_in = 128 at stride 1 runs 18 % faster (C_out = 256: 7 %) on the
    // two-workgroups-per-CU variant; from C_in = 256 on, and at stride 2, the deeper k-tile wins
    // 256 x 256 tiles for at least 256 output channels when they load the CUs no worse than the 256 x 128 ones: a CU's time
    // is its number of tiles times the tile's cost, and a 256 x 128 tile costs about 0.6 of a 256 x 256 one.  This choice may
    // depend on the number of samples: the two tile shapes produce the same bits, statistics included.
    if (a.Cout % 256 == 0 && a.Cin >= 128) {
      const long tw = ((M + 255) / 256) * (a.Cout / 256), cus = 256;
      if ((double)((tw + cus - 1) / cus) <= 0.6 * (double)((2 * tw + cus - 1) / cus)) return launch_conv_dtl<32, 2, 256>(p, x_bytes, w_bytes, s);
    }
    return (a.Cin <= 128 && a.stride == 1) ? launch_conv_dtl<32, 4>(p, x_bytes, w_bytes, s) : launch_conv_dtl<64, 2>(p, x_bytes, w_bytes, s);
  }
  if (a.Cout <= 64) return launch_conv_cfg<128, 64, 4, 1>(p, s);
  if ((long)Ho * Wo >= 16384) return launch_conv_cfg<256, 128, 4, 2>(p, s);
  return launch_conv_cfg<128, 128, 2, 2>(p, s);
}

}  // namespace dp
