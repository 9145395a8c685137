// GEMM kernels for the projections and MLPs of a stage (forward y = x W^T, backward
// dx = dy W and dW = dy^T x), fp32 accumulation, with fused epilogues.
//
// bf16 path: MFMA 32x32x16 tiles fed from LDS.  An operand whose contraction index is
// contiguous in memory is staged [rows][BK] and read with 16-byte LDS loads; an operand
// whose contraction index is the slow one (weights in dx, both operands in dW) is staged
// [BK][cols] exactly as it sits in HBM and read with the transposing LDS load, so no
// transposed copy of a weight or activation is ever materialised.  Workgroup ids are
// remapped so that the tiles running on one XCD (one L2) are neighbours in the output.
// fp32 path: plain FMA tiles (used by the small fp32 configuration only).
#include "dp_device.h"
#include "dp_kernels.h"
#include "dp_errors.h"
#include "dp_ktime.h"
#include "dp_gemm_epilogue.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>

namespace dp {

// ------------------------------------------------------------------ bf16 MFMA kernel
struct GemmBf16Params {
  const bf16* A; const bf16* B;
  int M, N, K, lda, ldb;
  int k_tiles_per_split;
  int tiles_m, tiles_n;
  int group_m;                 // tile-rows per group of the workgroup-to-tile map (choose_group_m)
  int split_major;             // register-staged kernel: number of splits of a 1-D grid over (split, tile) pairs, 0 = plain grid of tiles
  // Column sums of the A operand over the contraction (register-staged kernel, contraction-strided A only: the
  // bias gradient next to a weight gradient).  colsum[blockIdx.z * colsum_stride + m]; colsum_acc: add to what is there.
  float* colsum; int colsum_stride; int colsum_acc;
  uint32_t a_bytes, b_bytes;   // extent of each operand in bytes (direct-to-LDS kernels address it with 32-bit offsets)
  EpiParams<bf16> epi;
};

// Bytes from the first to one past the last element of an operand; rows x inner elements, row stride ld.
static inline size_t operand_extent_bytes(int rows, int inner, int ld) { return 2 * ((size_t)(rows - 1) * ld + inner); }
// The direct-to-LDS kernels need both operands below 4 GiB.
static inline bool dtl_addressable(const GemmArgs& a) {
  const size_t ab = a.a_mc ? operand_extent_bytes(a.K, a.M, a.lda) : operand_extent_bytes(a.M, a.K, a.lda);
  const size_t bb = a.b_mc ? operand_extent_bytes(a.K, a.N, a.ldb) : operand_extent_bytes(a.N, a.K, a.ldb);
  return ab < (1ull << 32) && bb < (1ull << 32);
}

template <int BM, int BN, int BK, int WGM, int WGN, bool A_MC, bool B_MC>
struct GemmSmem {
  // [rows][BK + 8] for contraction-contiguous operands; [BK][cols], unpadded with permuted 16-byte
  // chunks (mc_swizzle), for the others
  static constexpr int A_LD = A_MC ? BM : (BK + 8);
  static constexpr int B_LD = B_MC ? BN : (BK + 8);
  static constexpr int A_ELEMS = A_MC ? BK * A_LD : BM * A_LD;
  static constexpr int B_ELEMS = B_MC ? BK * B_LD : BN * B_LD;
  static constexpr int WN = BN / WGN;
  static constexpr int C_LD = WN + 4;                                   // per-wave fp32 staging [32][WN + 4]
  static constexpr size_t TILE_BYTES = 2 * (size_t)(A_ELEMS + B_ELEMS) * 2;
  static constexpr size_t EPI_BYTES = (size_t)WGM * WGN * 32 * C_LD * 4;
  static constexpr size_t BYTES = TILE_BYTES > EPI_BYTES ? TILE_BYTES : EPI_BYTES;
};

template <int BM, int BN, int BK, int WGM, int WGN, bool A_MC, bool B_MC>
__global__ void __launch_bounds__(WGM * WGN * 64)
gemm_bf16_kernel(const GemmBf16Params p) {
  using S = GemmSmem<BM, BN, BK, WGM, WGN, A_MC, B_MC>;
  constexpr int NT = WGM * WGN * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_CHUNKS = BM * BK / 8, B_CHUNKS = BN * BK / 8;
  constexpr int A_PER = A_CHUNKS / NT, B_PER = B_CHUNKS / NT;
  static_assert(A_CHUNKS % NT == 0 && B_CHUNKS % NT == 0, "tile/threads mismatch");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16* As = reinterpret_cast<bf16*>(smem_raw);
  bf16* Bs = As + 2 * S::A_ELEMS;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, l32 = lane & 31;
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
  // Split-K launches come as a 1-D grid over (split, tile) pairs in split-major order, of which every XCD takes a
  // contiguous range (the hardware deals consecutive workgroups round-robin to the 8 XCDs): the tiles of one split,
  // which read the same slice of both operands, run on one or two XCDs instead of all eight.
  int split = 0, tile_m, tile_n;
  if (p.split_major) {
    const int T = p.tiles_m * p.tiles_n;
    const int id = xcd_contiguous_id(blockIdx.x, T * p.split_major);
    split = id / T;
    tile_of_id(id % T, p.tiles_m, p.tiles_n, p.group_m, tile_m, tile_n);
  } else {
    tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, p.group_m, tile_m, tile_n);
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  EpiParams<bf16> epi = p.epi;
  if (p.split_major && epi.partial) epi.partial += (size_t)split * p.M * p.N;   // blockIdx.z is 0 in the 1-D grid

  const int total_kt = (p.K + BK - 1) / BK;
  const int kt_begin = split * p.k_tiles_per_split;
  const int kt_end = min(total_kt, kt_begin + p.k_tiles_per_split);

  // staged tile chunks; out-of-range chunks are loaded from a clamped (valid) address and
  // zeroed only when they are written to LDS, so nothing waits on the loads before the MFMAs
  bf16x8 ra[A_PER], rb[B_PER];
  unsigned oka = 0, okb = 0;
  // bias gradient: every thread always stages the same 8 columns of A (NT is a multiple of BM / 8), so it keeps
  // their running sums; only the workgroups of the first tile column do
  const bool do_colsum = A_MC && p.colsum != nullptr && tile_n == 0;
  float csum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#define DP_GEMM_LOAD_GLOBAL(kt_)                                                              \
  {                                                                                           \
    const int k0_ = (kt_) * BK;                                                               \
    oka = 0; okb = 0;                                                                         \
    _Pragma("unroll") for (int i = 0; i < A_PER; ++i) {                                       \
      const int id = tid + i * NT;                                                            \
      if (A_MC) {                                                                             \
        const int kk = id / (BM / 8), c = id % (BM / 8);                                      \
        const int gk = k0_ + kk, gm = m0 + c * 8;                                             \
        ra[i] = *reinterpret_cast<const bf16x8*>(p.A + (size_t)min(gk, p.K - 1) * p.lda + min(gm, p.M - 8)); \
        oka |= (unsigned)(gk < p.K && gm < p.M) << i;                                         \
      } else {                                                                                \
        const int r = id / (BK / 8), c = id % (BK / 8);                                       \
        const int gm = m0 + r, gk = k0_ + c * 8;                                              \
        ra[i] = *reinterpret_cast<const bf16x8*>(p.A + (size_t)min(gm, p.M - 1) * p.lda + min(gk, p.K - 8)); \
        oka |= (unsigned)(gm < p.M && gk < p.K) << i;                                         \
      }                                                                                       \
    }                                                                                         \
    _Pragma("unroll") for (int i = 0; i < B_PER; ++i) {                                       \
      const int id = tid + i * NT;                                                            \
      if (B_MC) {                                                                             \
        const int kk = id / (BN / 8), c = id % (BN / 8);                                      \
        const int gk = k0_ + kk, gn = n0 + c * 8;                                             \
        rb[i] = *reinterpret_cast<const bf16x8*>(p.B + (size_t)min(gk, p.K - 1) * p.ldb + min(gn, p.N - 8)); \
        okb |= (unsigned)(gk < p.K && gn < p.N) << i;                                         \
      } else {                                                                                \
        const int r = id / (BK / 8), c = id % (BK / 8);                                       \
        const int gn = n0 + r, gk = k0_ + c * 8;                                              \
        rb[i] = *reinterpret_cast<const bf16x8*>(p.B + (size_t)min(gn, p.N - 1) * p.ldb + min(gk, p.K - 8)); \
        okb |= (unsigned)(gn < p.N && gk < p.K) << i;                                         \
      }                                                                                       \
    }                                                                                         \
  }
#define DP_GEMM_STORE_LDS(buf_)                                                               \
  {                                                                                           \
    bf16* as_ = As + (buf_) * S::A_ELEMS;                                                     \
    bf16* bs_ = Bs + (buf_) * S::B_ELEMS;                                                     \
    _Pragma("unroll") for (int i = 0; i < A_PER; ++i) {                                       \
      const int id = tid + i * NT;                                                            \
      if (A_MC) { const int kk = id / (BM / 8), c = id % (BM / 8); const bf16x8 v_ = ((oka >> i) & 1) ? ra[i] : zero8(); \
                  *reinterpret_cast<bf16x8*>(as_ + kk * S::A_LD + mc_swizzle(c, kk) * 8) = v_;                \
                  if (do_colsum) { _Pragma("unroll") for (int t_ = 0; t_ < 8; ++t_) csum[t_] += (float)v_[t_]; } } \
      else      { const int r = id / (BK / 8), c = id % (BK / 8);  *reinterpret_cast<bf16x8*>(as_ + r * S::A_LD + c * 8) = ((oka >> i) & 1) ? ra[i] : zero8(); }  \
    }                                                                                         \
    _Pragma("unroll") for (int i = 0; i < B_PER; ++i) {                                       \
      const int id = tid + i * NT;                                                            \
      if (B_MC) { const int kk = id / (BN / 8), c = id % (BN / 8); *reinterpret_cast<bf16x8*>(bs_ + kk * S::B_LD + mc_swizzle(c, kk) * 8) = ((okb >> i) & 1) ? rb[i] : zero8(); } \
      else      { const int r = id / (BK / 8), c = id % (BK / 8);  *reinterpret_cast<bf16x8*>(bs_ + r * S::B_LD + c * 8) = ((okb >> i) & 1) ? rb[i] : zero8(); }  \
    }                                                                                         \
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  if (kt_begin < kt_end) {
    DP_GEMM_LOAD_GLOBAL(kt_begin);
    DP_GEMM_STORE_LDS(0);
  }
  __syncthreads();

  for (int kt = kt_begin; kt < kt_end; ++kt) {
    const int buf = (kt - kt_begin) & 1;
    const bool more = kt + 1 < kt_end;
    if (more) DP_GEMM_LOAD_GLOBAL(kt + 1);
    const bf16* as = As + buf * S::A_ELEMS;
    const bf16* bs = Bs + buf * S::B_ELEMS;
    // fragments of k-step ks + 1 are fetched from LDS before the MFMAs of k-step ks are issued
    bf16x8 fa[2][TM], fb[2][TN];
#define DP_GEMM_LOAD_FRAGS(ks_, set_)                                                                                   \
    {                                                                                                                     \
      _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                                                   \
        if (A_MC) fa[set_][i] = frag_from_mc_swz(as, S::A_LD, (ks_) * 16, wm0 + i * 32, lane);                 \
        else      fa[set_][i] = *reinterpret_cast<const bf16x8*>(as + (wm0 + i * 32 + l32) * S::A_LD + (ks_) * 16 + 8 * g); \
      }                                                                                                                   \
      _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                                                   \
        if (B_MC) fb[set_][j] = frag_from_mc_swz(bs, S::B_LD, (ks_) * 16, wn0 + j * 32, lane);                 \
        else      fb[set_][j] = *reinterpret_cast<const bf16x8*>(bs + (wn0 + j * 32 + l32) * S::B_LD + (ks_) * 16 + 8 * g); \
      }                                                                                                                   \
    }
    DP_GEMM_LOAD_FRAGS(0, 0);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      if (ks + 1 < BK / 16) DP_GEMM_LOAD_FRAGS(ks + 1, (ks + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(fa[ks & 1][i], fb[ks & 1][j], acc[i][j]);
    }
#undef DP_GEMM_LOAD_FRAGS
    if (more) DP_GEMM_STORE_LDS(buf ^ 1);
    __syncthreads();
  }

  if (A_MC && do_colsum) {      // workgroup-uniform
    // fixed order: a thread's rows in k order (above), then the NT / (BM / 8) row groups in ascending order
    constexpr int GROUPS = NT / (BM / 8);
    float* red = reinterpret_cast<float*>(smem_raw);
    const int c = tid % (BM / 8), grp = tid / (BM / 8);
#pragma unroll
    for (int t = 0; t < 8; ++t) red[grp * BM + c * 8 + t] = csum[t];
    __syncthreads();
    if (tid < BM && m0 + tid < p.M) {
      float sum = 0.f;
      for (int g2 = 0; g2 < GROUPS; ++g2) sum += red[g2 * BM + tid];
      float* o = p.colsum + (size_t)split * p.colsum_stride + m0 + tid;
      *o = p.colsum_acc ? *o + sum : sum;
    }
    __syncthreads();
  }
  float* Cw = reinterpret_cast<float*>(smem_raw) + wave * 32 * S::C_LD;
  wave_epilogue<TM, TN, WN, S::C_LD>(acc, Cw, epi, m0 + wm0, n0 + wn0, lane);
}

#undef DP_GEMM_LOAD_GLOBAL
#undef DP_GEMM_STORE_LDS

// ------------------------------------------------------------------ bf16 MFMA kernel, direct-to-LDS pipeline
// Same tiling and epilogue, but the operand tiles travel global -> LDS without passing through
// registers (buffer_load_dwordx4 ... lds: every lane fetches 16 bytes, the wave's 1 KB lands
// contiguously in LDS) in a ring of three or four buffers, two or three k-tiles ahead of the
// MFMAs.  What bounds this loop on MI355X is not one pipe but three at once: per k-tile a
// 256x128 workgroup needs about as many LDS cycles (fragment reads plus the incoming copies) and
// three quarters as many L1 address cycles as MFMA cycles, so copies, fragment reads and MFMAs
// are interleaved finely and every wait names exactly the data it needs.  The copies use the
// buffer-descriptor form because a flat-address LDS copy in flight makes the compiler treat the
// LDS counter as unordered (every wait for one fragment becomes a wait for all).  LDS tiles are unpadded; bank conflicts
// are avoided by permuting 16-byte chunks inside a row (the permutation is applied through
// the per-lane global address, and undone when fragments are read).
//   K-contiguous operand:  tile [rows][32], chunk c of row r stored at c ^ ((r >> 2) & 3).
//   K-strided operand:     tile [BK][cols], chunk c of k-row k stored at c ^ (4 * (k & 3)).
// Requires K % 32 == 0.  Rows / columns beyond M / N are fetched from a clamped address; they
// only feed accumulators whose outputs are never stored.

template <int BM, int BN, int BK, int STAGES, int WGM, int WGN>
struct DtlSmem {
  static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  static constexpr int WN = BN / WGN;
  static constexpr int C_LD = WN + 4;
  static constexpr size_t TILE_BYTES = (size_t)STAGES * STAGE;
  static constexpr size_t EPI_BYTES = (size_t)WGM * WGN * 32 * C_LD * 4;
  static constexpr size_t BYTES = TILE_BYTES > EPI_BYTES ? TILE_BYTES : EPI_BYTES;
};

// Chunk permutation of a K-contiguous tile row r (BK / 8 chunks per row): conflict-free 16-byte
// reads by 16 consecutive rows.  BK = 32: 4 chunks, key (r >> 2) & 3; BK = 64: 8 chunks, key (r >> 1) & 7.
template <int BK> __device__ __forceinline__ int kc_key(int r) { return BK == 32 ? ((r >> 2) & 3) : ((r >> 1) & 7); }

// FP8: the operands are OCP E4M3 bytes.  The copy pipeline only moves bytes, so an fp8 row of K bytes is handled as a
// row of K / 2 two-byte elements (all sizes and strides in the parameters are given in those units); what changes is the
// k-step (64 bytes instead of 32: two 16-byte chunks per lane) and the instruction, v_mfma_f32_32x32x64_f8f6f4 with both
// block scales at 2^0.  Any assignment of the 64 bytes of a k-step to lanes and byte slots gives the right product as
// long as it is the same for both operands, which it is by symmetry.
typedef __attribute__((ext_vector_type(8))) int i32x8;

template <int BM, int BN, int BK, int STAGES, int WGM, int WGN, bool A_MC, bool B_MC, bool FP8 = false>
__global__ void __launch_bounds__(WGM * WGN * 64)
gemm_bf16_dtl_kernel(const GemmBf16Params p) {
  using S = DtlSmem<BM, BN, BK, STAGES, WGM, WGN>;
  constexpr int NW = WGM * WGN, KS = FP8 ? BK / 32 : BK / 16, CPR = BK / 8;      // k-steps per tile, chunks per K-contiguous row
  static_assert(!FP8 || (!A_MC && !B_MC && BK == 64), "the fp8 variant takes contraction-contiguous operands and 128-byte k-tiles");
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_LOADS = S::A_BYTES / 1024 / NW, B_LOADS = S::B_BYTES / 1024 / NW, LOADS = A_LOADS + B_LOADS;
  static_assert(S::A_BYTES % (1024 * NW) == 0 && S::B_BYTES % (1024 * NW) == 0, "tile/waves mismatch");
  static_assert(KS % 2 == 0 && STAGES >= 2, "pipeline shape");
  constexpr bool INTERLEAVE = BK == 64 && !FP8 && !A_MC && !B_MC;

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, l32 = lane & 31;
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
  int tile_m, tile_n;
  tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, p.group_m, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int kt_begin = blockIdx.z * p.k_tiles_per_split;
  const int kt_end = min(p.K / BK, kt_begin + p.k_tiles_per_split);
  const int nk = kt_end - kt_begin;

  // per-lane byte offset (inside the operand) of each of this wave's 1 KB pieces at k-tile 0;
  // advancing by one k-tile adds a wave-uniform constant.  Rows / column chunks past the matrix edge
  // are clamped to the last valid one (they only feed outputs that are never stored).
  const rsrc_t ra = make_rsrc(p.A, p.a_bytes), rb = make_rsrc(p.B, p.b_bytes);
  uint32_t va[A_LOADS], vb[B_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int blk = wave * A_LOADS + j;
    if (A_MC) {
      const int k = blk * (1024 / (BM * 2)) + lane / (BM / 8), pc = lane % (BM / 8), c = mc_swizzle(pc, k);
      va[j] = 2u * ((uint32_t)(kt_begin * BK + k) * p.lda + min(m0 + c * 8, p.M - 8));
    } else {
      const int r = blk * (512 / BK) + lane / CPR, pc = lane % CPR, c = pc ^ kc_key<BK>(r);
      va[j] = 2u * ((uint32_t)min(m0 + r, p.M - 1) * p.lda + kt_begin * BK + c * 8);
    }
  }
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j) {
    const int blk = wave * B_LOADS + j;
    if (B_MC) {
      const int k = blk * (1024 / (BN * 2)) + lane / (BN / 8), pc = lane % (BN / 8), c = mc_swizzle(pc, k);
      vb[j] = 2u * ((uint32_t)(kt_begin * BK + k) * p.ldb + min(n0 + c * 8, p.N - 8));
    } else {
      const int r = blk * (512 / BK) + lane / CPR, pc = lane % CPR, c = pc ^ kc_key<BK>(r);
      int brow = min(n0 + r, p.N - 1);
      if (p.epi.geglu == 1)   // tile row r: 32-row blocks alternate value / gate rows of the same outputs
        brow = ((r >> 5) & 1) * p.epi.geglu_inner + min(n0 / 2 + (r >> 6) * 32 + (r & 31), p.epi.geglu_inner - 1);
      vb[j] = 2u * ((uint32_t)brow * p.ldb + kt_begin * BK + c * 8);
    }
  }
  const uint32_t a_step = 2u * (A_MC ? (uint32_t)BK * p.lda : BK), b_step = 2u * (B_MC ? (uint32_t)BK * p.ldb : BK);

  // Copies of k-tile t_ whose index j (A pieces first, then B) satisfies j % parts_ == part_.
#define DP_DTL_ISSUE_PART(t_, part_, parts_)                                                                          \
  {                                                                                                                   \
    unsigned char* st_ = smem_raw + ((t_) % STAGES) * S::STAGE;                                                       \
    _Pragma("unroll") for (int j = 0; j < A_LOADS; ++j)                                                               \
      if (j % (parts_) == (part_))                                                                                    \
        async_copy_16B_buf(ra, va[j], (uint32_t)(t_) * a_step, st_ + (wave * A_LOADS + j) * 1024);                    \
    _Pragma("unroll") for (int j = 0; j < B_LOADS; ++j)                                                               \
      if ((A_LOADS + j) % (parts_) == (part_))                                                                        \
        async_copy_16B_buf(rb, vb[j], (uint32_t)(t_) * b_step, st_ + S::A_BYTES + (wave * B_LOADS + j) * 1024);       \
  }
#define DP_DTL_ISSUE(t_) DP_DTL_ISSUE_PART(t_, 0, 1)

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Fragment fetch of k-step ks_ of the k-tile in stage st_ into register set set_.
  bf16x8 fa[2][TM], fb[2][TN];
  i32x8 qa[2][FP8 ? TM : 1], qb[2][FP8 ? TN : 1];     // fp8: 32 bytes per lane and fragment
#define DP_DTL_FRAGS(st_, ks_, set_)                                                                                  \
  { if (FP8) {                                                                                                        \
    const unsigned char* as = smem_raw + (st_) * S::STAGE;                                                            \
    const unsigned char* bs = smem_raw + (st_) * S::STAGE + S::A_BYTES;                                               \
    _Pragma("unroll") for (int i = 0; i < (FP8 ? TM : 0); ++i) {                                                      \
      const int r = wm0 + i * 32 + l32, c0 = 4 * (ks_) + 2 * g, key = kc_key<BK>(r);                                  \
      const u32x4 lo = *reinterpret_cast<const u32x4*>(as + r * (2 * BK) + ((c0 ^ key) * 16));                        \
      const u32x4 hi = *reinterpret_cast<const u32x4*>(as + r * (2 * BK) + (((c0 + 1) ^ key) * 16));                  \
      qa[set_][i] = __builtin_bit_cast(i32x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));              \
    }                                                                                                                 \
    _Pragma("unroll") for (int j2 = 0; j2 < (FP8 ? TN : 0); ++j2) {                                                   \
      const int r = wn0 + j2 * 32 + l32, c0 = 4 * (ks_) + 2 * g, key = kc_key<BK>(r);                                 \
      const u32x4 lo = *reinterpret_cast<const u32x4*>(bs + r * (2 * BK) + ((c0 ^ key) * 16));                        \
      const u32x4 hi = *reinterpret_cast<const u32x4*>(bs + r * (2 * BK) + (((c0 + 1) ^ key) * 16));                  \
      qb[set_][j2] = __builtin_bit_cast(i32x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));             \
    }                                                                                                                 \
  } else {                                                                                                            \
    const bf16* as = reinterpret_cast<const bf16*>(smem_raw + (st_) * S::STAGE);                                      \
    const bf16* bs = reinterpret_cast<const bf16*>(smem_raw + (st_) * S::STAGE + S::A_BYTES);                         \
    _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                                                  \
      if (A_MC) {                                                                                                     \
        fa[set_][i] = frag_from_mc_swz(as, BM, (ks_) * 16, wm0 + i * 32, lane);                                       \
      } else {                                                                                                        \
        const int r = wm0 + i * 32 + l32;                                                                             \
        fa[set_][i] = *reinterpret_cast<const bf16x8*>(as + r * BK + (((2 * (ks_) + g) ^ kc_key<BK>(r)) * 8));        \
      }                                                                                                               \
    }                                                                                                                 \
    _Pragma("unroll") for (int j2 = 0; j2 < TN; ++j2) {                                                               \
      if (B_MC) {                                                                                                     \
        fb[set_][j2] = frag_from_mc_swz(bs, BN, (ks_) * 16, wn0 + j2 * 32, lane);                                     \
      } else {                                                                                                        \
        const int r = wn0 + j2 * 32 + l32;                                                                            \
        fb[set_][j2] = *reinterpret_cast<const bf16x8*>(bs + r * BK + (((2 * (ks_) + g) ^ kc_key<BK>(r)) * 8));       \
      }                                                                                                               \
    }                                                                                                                 \
  } }
#define DP_DTL_MFMAS(set_)                                                                                            \
  _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                                      \
    _Pragma("unroll") for (int j2 = 0; j2 < TN; ++j2) {                                                               \
      if (FP8) acc[i][j2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(qa[set_][FP8 ? i : 0], qb[set_][FP8 ? j2 : 0], acc[i][j2], 0, 0, 0, 127, 0, 127); \
      else acc[i][j2] = mfma32(fa[set_][i], fb[set_][j2], acc[i][j2]);                                                \
    }

  // Software pipeline.  All STAGES buffers are filled up front.  Fragments are fetched one k-step
  // ahead of the MFMAs that use them, also across the k-tile boundary: before the last MFMA group
  // of k-tile t every wave waits for its own fragment reads of that tile and for its share of
  // k-tile t + 1 to land, then meets the others at a barrier.  Past it, k-tile t + 1 is visible to
  // all and nobody reads k-tile t from LDS any more, so its buffer is free for k-tile t + STAGES.
  // Those copies are not issued in one burst behind the barrier (all waves would queue up at the
  // texture addresser together while the MFMA pipes drain) but spread over the k-steps of
  // k-tile t + 1, a few per MFMA group; they still run STAGES - 2 k-tiles ahead of their use.
  constexpr int PART_LAST = LOADS / KS;   // number of copies with index % KS == KS - 1
  static_assert(STAGES >= 3 && STAGES <= 4 && 3 * LOADS < 64, "pipeline shape");
  for (int t = 0; t < STAGES && t < nk; ++t) DP_DTL_ISSUE(t);
  {
    const int y = min(nk, STAGES) - 1;
    if (y >= 3) wait_vmcnt<3 * LOADS>();
    else if (y == 2) wait_vmcnt<2 * LOADS>();
    else if (y == 1) wait_vmcnt<LOADS>();
    else wait_vmcnt<0>();
  }
  barrier_nofence();
  DP_DTL_FRAGS(0, 0, 0);
  // all k-tiles but the last: no branch between the fragment reads and the MFMAs, so the waits for
  // LDS data stay exact (a merge of paths with different numbers of reads in flight would make the
  // compiler wait for all of them)
  for (int t = 0; t + 1 < nk; ++t) {
    const int st = t % STAGES;
    const bool refill = t >= 1 && t - 1 + STAGES < nk;   // k-tile t - 1 + STAGES goes into the buffer k-tile t - 1 left
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks + 1 < KS) {
        DP_DTL_FRAGS(st, ks + 1, (ks + 1) & 1);
      } else {
        wait_lgkmcnt0();
        // copies younger than k-tile t + 1 that may stay in flight: whole k-tiles t + 2 .. t - 2 + STAGES
        // and the parts of k-tile t - 1 + STAGES issued so far (never more than are really there)
        const int avail = nk - 2 - t;
        if (STAGES == 4 && avail >= 2) wait_vmcnt<2 * LOADS - PART_LAST>();
        else if (STAGES == 4 && avail == 1) wait_vmcnt<LOADS>();
        else if (STAGES == 3 && avail >= 1) wait_vmcnt<LOADS - PART_LAST>();
        else wait_vmcnt<0>();
        barrier_nofence();
        DP_DTL_FRAGS((t + 1) % STAGES, 0, 0);
      }
      if (INTERLEAVE && ks + 1 < KS) {
        // 64-deep k-tiles: the scheduler may place one fragment read behind each MFMA instead of issuing the whole
        // batch first (6-10 % on the N = 640 projections; the 32-deep tiles lose 4 % with it and keep the batch)
        _Pragma("unroll") for (int q_ = 0; q_ < TM * TN; ++q_) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      } else {
        __builtin_amdgcn_sched_barrier(0);
      }
      DP_DTL_MFMAS(ks & 1);
      __builtin_amdgcn_sched_barrier(0);
      if (refill) DP_DTL_ISSUE_PART(t - 1 + STAGES, ks, KS);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  {
    const int st = (nk - 1) % STAGES;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks + 1 < KS) DP_DTL_FRAGS(st, ks + 1, (ks + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
      DP_DTL_MFMAS(ks & 1);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#undef DP_DTL_FRAGS
#undef DP_DTL_MFMAS
#undef DP_DTL_ISSUE
#undef DP_DTL_ISSUE_PART
  __syncthreads();   // every wave is done with the operand tiles before they are reused below

  float* Cw = reinterpret_cast<float*>(smem_raw) + wave * 32 * S::C_LD;
  wave_epilogue<TM, TN, WN, S::C_LD>(acc, Cw, p.epi, m0 + wm0, n0 + wn0, lane);
}

// ------------------------------------------------------------------ bf16 MFMA kernel, 16x16x32 tiles (flexible tile shapes)
// The same direct-to-LDS pipeline with v_mfma_f32_16x16x32_bf16, whose 16-row / 16-column granularity
// allows workgroup tiles such as 256x160 (wave tile 64x80: 9 fragment reads per 20 MFMAs).  It exists
// for output widths that leave 256x128 / 256x256 tiles with padded columns or a badly filled last round
// (N = 320: 256 tiles of 256x160 instead of 256 half-empty 256x256 tiles; N = 1152: 256 tiles, 10 % padding).
// Contraction-contiguous operands only (y = x W^T), 64-deep k-tiles, 8 waves.
// Register layout of the instruction (lane l): A row l % 16, B column l % 16, both k = 8 * (l / 16) .. + 7 of
// the 32-deep step; D column l % 16, rows 4 * (l / 16) + r.
typedef __attribute__((ext_vector_type(4))) float f32x4_acc;

template <int BM, int BN, int STAGES, int WGM, int WGN>
struct Dtl16Smem {
  static constexpr int BK = 64;
  static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  static constexpr int WN = BN / WGN;
  static constexpr int C_LD = WN + 4;
  static constexpr size_t TILE_BYTES = (size_t)STAGES * STAGE;
  static constexpr size_t EPI_BYTES = (size_t)WGM * WGN * 16 * C_LD * 4;
  static constexpr size_t BYTES = TILE_BYTES > EPI_BYTES ? TILE_BYTES : EPI_BYTES;
};

template <int BM, int BN, int STAGES, int WGM, int WGN>
__global__ void __launch_bounds__(WGM * WGN * 64)
gemm_bf16_dtl16_kernel(const GemmBf16Params p) {
  using S = Dtl16Smem<BM, BN, STAGES, WGM, WGN>;
  constexpr int BK = 64, NW = WGM * WGN, KS = 2, CPR = 8;        // two 32-deep k-steps per k-tile, 8 chunks per tile row
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 16, TN = WN / 16;
  constexpr int PIECES = (S::A_BYTES + S::B_BYTES) / 1024, A_PIECES = S::A_BYTES / 1024;
  constexpr int LOADS = (PIECES + NW - 1) / NW;                   // copies per wave and k-tile; surplus slots repeat the last piece
  static_assert(WM % 16 == 0 && WN % 16 == 0 && S::A_BYTES % 1024 == 0 && S::B_BYTES % 1024 == 0, "tile shape");
  static_assert(STAGES == 3 && 2 * LOADS < 64, "pipeline shape");

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, q = lane >> 4;
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
  int tile_m, tile_n;
  tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, p.group_m, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int nk = p.K / BK;

  // Piece j of this wave: 8 tile rows x 128 bytes of A (pieces 0 .. A_PIECES - 1) or B.  A wave-uniform
  // choice of descriptor per slot is made with two issue paths below; the per-lane byte offset is fixed.
  const rsrc_t ra = make_rsrc(p.A, p.a_bytes), rb = make_rsrc(p.B, p.b_bytes);
  uint32_t vo[LOADS];
  int ldsoff[LOADS];
  bool isa[LOADS];
#pragma unroll
  for (int j = 0; j < LOADS; ++j) {
    const int piece = min(wave * LOADS + j, PIECES - 1);
    isa[j] = piece < A_PIECES;
    const int blk = isa[j] ? piece : piece - A_PIECES;
    const int r = blk * 8 + lane / CPR, pc = lane % CPR, c = pc ^ kc_key<BK>(r);
    if (isa[j]) vo[j] = 2u * ((uint32_t)min(m0 + r, p.M - 1) * p.lda + c * 8);
    else vo[j] = 2u * ((uint32_t)min(n0 + r, p.N - 1) * p.ldb + c * 8);
    ldsoff[j] = (isa[j] ? 0 : S::A_BYTES) + blk * 1024;
  }
#define DP16_ISSUE_PART(t_, part_, parts_)                                                                            \
  {                                                                                                                   \
    unsigned char* st_ = smem_raw + ((t_) % STAGES) * S::STAGE;                                                       \
    _Pragma("unroll") for (int j = 0; j < LOADS; ++j)                                                                 \
      if (j % (parts_) == (part_)) {                                                                                  \
        if (isa[j]) async_copy_16B_buf(ra, vo[j], (uint32_t)(t_) * (2u * BK), st_ + ldsoff[j]);                       \
        else async_copy_16B_buf(rb, vo[j], (uint32_t)(t_) * (2u * BK), st_ + ldsoff[j]);                              \
      }                                                                                                               \
  }

  f32x4_acc acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;

  bf16x8 fa[2][TM], fb[2][TN];
#define DP16_FRAGS(st_, ks_, set_)                                                                                    \
  {                                                                                                                   \
    const bf16* as = reinterpret_cast<const bf16*>(smem_raw + (st_) * S::STAGE);                                      \
    const bf16* bs = reinterpret_cast<const bf16*>(smem_raw + (st_) * S::STAGE + S::A_BYTES);                         \
    _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                                                  \
      const int r = wm0 + i * 16 + l16;                                                                               \
      fa[set_][i] = *reinterpret_cast<const bf16x8*>(as + r * BK + (((4 * (ks_) + q) ^ kc_key<BK>(r)) * 8));          \
    }                                                                                                                 \
    _Pragma("unroll") for (int j2 = 0; j2 < TN; ++j2) {                                                               \
      const int r = wn0 + j2 * 16 + l16;                                                                              \
      fb[set_][j2] = *reinterpret_cast<const bf16x8*>(bs + r * BK + (((4 * (ks_) + q) ^ kc_key<BK>(r)) * 8));         \
    }                                                                                                                 \
  }
#define DP16_MFMAS(set_)                                                                                              \
  _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                                      \
    _Pragma("unroll") for (int j2 = 0; j2 < TN; ++j2)                                                                 \
      acc[i][j2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[set_][i], fb[set_][j2], acc[i][j2], 0, 0, 0);

  // pipeline: identical in structure to gemm_bf16_dtl_kernel (three buffers, copies two k-tiles ahead,
  // spread over the k-steps; exact waits)
  constexpr int PART_LAST = LOADS / KS;
#pragma unroll
  for (int t = 0; t < STAGES; ++t)
    if (t < nk) DP16_ISSUE_PART(t, 0, 1);
  {
    const int y = min(nk, STAGES) - 1;
    if (y == 2) wait_vmcnt<2 * LOADS>();
    else if (y == 1) wait_vmcnt<LOADS>();
    else wait_vmcnt<0>();
  }
  barrier_nofence();
  DP16_FRAGS(0, 0, 0);
  for (int t = 0; t + 1 < nk; ++t) {
    const int st = t % STAGES;
    const bool refill = t >= 1 && t - 1 + STAGES < nk;
    // k-step 0: fetch the fragments of k-step 1, MFMAs of k-step 0
    DP16_FRAGS(st, 1, 1);
    __builtin_amdgcn_sched_barrier(0);
    DP16_MFMAS(0);
    __builtin_amdgcn_sched_barrier(0);
    if (refill) DP16_ISSUE_PART(t - 1 + STAGES, 0, KS);
    __builtin_amdgcn_sched_barrier(0);
    // k-step 1: publish k-tile t + 1, fetch its first fragments, MFMAs of k-step 1
    wait_lgkmcnt0();
    if (nk - 2 - t >= 1) wait_vmcnt<LOADS - PART_LAST>();
    else wait_vmcnt<0>();
    barrier_nofence();
    DP16_FRAGS((t + 1) % STAGES, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    DP16_MFMAS(1);
    __builtin_amdgcn_sched_barrier(0);
    if (refill) DP16_ISSUE_PART(t - 1 + STAGES, 1, KS);
    __builtin_amdgcn_sched_barrier(0);
  }
  {
    const int st = (nk - 1) % STAGES;
    DP16_FRAGS(st, 1, 1);
    __builtin_amdgcn_sched_barrier(0);
    DP16_MFMAS(0);
    __builtin_amdgcn_sched_barrier(0);
    DP16_MFMAS(1);
  }
#undef DP16_FRAGS
#undef DP16_MFMAS
#undef DP16_ISSUE_PART
  __syncthreads();   // every wave is done with the operand tiles before they are reused below

  // Epilogue: 16-row slabs through the wave's own fp32 LDS region, then 8 consecutive columns per lane.
  float* Cw = reinterpret_cast<float*>(smem_raw) + wave * 16 * S::C_LD;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) Cw[(4 * q + r) * S::C_LD + j * 16 + l16] = acc[i][j][r];
    asm volatile("" ::: "memory");
    constexpr int CHUNKS = 16 * WN / 8;
#pragma unroll 1
    for (int it = 0; it < (CHUNKS + 63) / 64; ++it) {
      const int id = it * 64 + lane;
      const int lr = id / (WN / 8), lc = (id % (WN / 8)) * 8;
      const int m = m0 + wm0 + i * 16 + lr, n = n0 + wn0 + lc;
      if (id < CHUNKS && m < p.M && n < p.N) {
        float v[8];
        *reinterpret_cast<f32x4*>(&v[0]) = *reinterpret_cast<const f32x4*>(&Cw[lr * S::C_LD + lc]);
        *reinterpret_cast<f32x4*>(&v[4]) = *reinterpret_cast<const f32x4*>(&Cw[lr * S::C_LD + lc + 4]);
        epi_vec8(p.epi, m, n, v);
      }
    }
    asm volatile("" ::: "memory");
  }
}

// ------------------------------------------------------------------ fp32 FMA kernel
struct GemmF32Params {
  const float* A; const float* B;
  int M, N, K, lda, ldb, a_mc, b_mc;
  EpiParams<float> epi;
};

// 64x64 output tile, 16-deep k slices, 256 threads each owning a 4x4 micro-tile.
__global__ void __launch_bounds__(256) gemm_f32_kernel(const GemmF32Params p) {
  __shared__ float As[16][65];
  __shared__ float Bs[16][65];
  const int tid = threadIdx.x;
  const int tm = (tid / 16) * 4, tn = (tid % 16) * 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < p.K; k0 += 16) {
    for (int i = tid; i < 64 * 16; i += 256) {
      const int kk = i % 16, r = i / 16;
      const int gm = m0 + r, gn = n0 + r, gk = k0 + kk;
      float a = 0.f, b = 0.f;
      if (gk < p.K) {
        if (gm < p.M) a = p.a_mc ? p.A[(size_t)gk * p.lda + gm] : p.A[(size_t)gm * p.lda + gk];
        if (gn < p.N) b = p.b_mc ? p.B[(size_t)gk * p.ldb + gn] : p.B[(size_t)gn * p.ldb + gk];
      }
      As[kk][r] = a;
      Bs[kk][r] = b;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][tm + i]; b[i] = Bs[kk][tn + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) epi_store<float>(p.epi, m0 + tm + i, n0 + tn + j, acc[i][j]);
}

// Second pass of a split-K GEMM with a storage-dtype output: sums the fp32 partial tiles in ascending
// split order (fixed order, run-to-run identical) and applies the GEMM's epilogue to the sums.  One thread
// per 8 consecutive columns of a row.
__global__ void __launch_bounds__(256) reduce_epilogue_kernel(EpiParams<bf16> e, const float* __restrict__ partial, int splits) {
  const int per_row = e.N / 8;
  const size_t idx = blockIdx.x * (size_t)256 + threadIdx.x;
  if (idx >= (size_t)e.M * per_row) return;
  const int m = (int)(idx / per_row), n = (int)(idx % per_row) * 8;
  const float* p = partial + (size_t)m * e.N + n;
  const size_t plane = (size_t)e.M * e.N;
  float v[8];
  *reinterpret_cast<f32x4*>(&v[0]) = *reinterpret_cast<const f32x4*>(p);
  *reinterpret_cast<f32x4*>(&v[4]) = *reinterpret_cast<const f32x4*>(p + 4);
  for (int z = 1; z < splits; ++z) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(p + z * plane), b = *reinterpret_cast<const f32x4*>(p + z * plane + 4);
#pragma unroll
    for (int t = 0; t < 4; ++t) { v[t] += a[t]; v[4 + t] += b[t]; }
  }
  epi_vec8(e, m, n, v);
}

// ------------------------------------------------------------------ host side
template <typename T>
static EpiParams<T> make_epi(const GemmArgs& a) {
  EpiParams<T> e;
  e.M = a.M; e.N = a.N;
  e.out = (T*)a.out; e.ldo = a.ldo;
  e.out32 = a.out_f32; e.ldo32 = a.ldo32; e.accumulate = a.accumulate;
  e.partial = nullptr;
  e.bias = (const T*)a.bias;
  e.pre_out = (T*)a.pre_out; e.ld_pre = a.ld_pre;
  e.act = a.act;
  e.dact_pre = (const T*)a.dact_pre; e.ld_dact = a.ld_dact; e.dact_kind = a.dact_kind;
  e.gate = (const T*)a.gate; e.gate_ld = a.gate_ld; e.rows_per_batch = a.rows_per_batch > 0 ? a.rows_per_batch : 1;
  e.residual = a.residual; e.ld_res = a.ld_res; e.residual_f32 = a.residual_f32; e.out_fused_f32 = a.out_fused_f32;
  e.geglu = a.geglu; e.geglu_inner = a.geglu_inner; e.geglu_u = (const T*)a.geglu_u; e.ld_geglu = a.ld_geglu;
  e.out_scale = 1.0f;
  return e;
}

// Bytes a bf16 GEMM launch has to move once: both operands, the result in its output type, and every
// tensor its fused epilogue reads or writes beside it (fp32 residual in and out, the saved projection next
// to a GeGLU output, the saved pre-activation of a backward).  Split-K partial sums are not counted.
static double gemm_tensor_bytes(const GemmArgs& a) {
  const double mn = (double)a.M * a.N;
  double b = 2.0 * ((double)a.M * a.K + (double)a.N * a.K);
  if (a.out_f32) return b + 4.0 * mn * (a.accumulate ? 2.0 : 1.0);
  if (a.geglu == 1) return b + 2.0 * (double)a.M * a.geglu_inner + (a.pre_out ? 2.0 * mn : 0.0);
  if (a.geglu == 2) return b + 2.0 * 2.0 * (double)a.M * 2.0 * a.geglu_inner;      // u read, du written: [M, 2 inner] each
  b += mn * (a.out_fused_f32 ? 4.0 : 2.0);
  if (a.pre_out) b += 2.0 * mn;
  if (a.dact_pre) b += 2.0 * mn;
  if (a.residual) b += mn * (a.residual_f32 ? 4.0 : 2.0);
  return b;
}

// Group height of the workgroup-to-tile map.  An XCD's contiguous share of the tiles spans 1 / k of a group
// when k XCDs share one: the row operand's panels of that group are then fetched by k L2s and each L2 fetches
// 1 / k of the column operand, k * (row operand bytes) + (8 / k) * (column operand bytes) in total, least at
// k = sqrt(8 * cols / rows).  Narrow outputs (N <= ~0.25 M: the N = 640 and 1152 projections) want k = 1, whole
// tile-rows per XCD, which halves the fetches of their large row operand against the fixed 8 tile-rows used
// before; wide ones (N = 5120) keep two XCDs per group.  Measured on cfg2 (L2 fetch bytes per launch, rocprofv3
// FETCH_SIZE): 256x128x64 projections 65 -> 47 MB, weight-gradient GEMMs 119 -> 94 MB; step time -0.3 to -1 %.
static int choose_group_m(const GemmArgs& a, int tiles_m, int tiles_n) {
  const double rows = a.M, cols = a.N;
  const double ks = std::sqrt(8.0 * cols / rows);
  const int k = ks < 1.41 ? 1 : (ks < 2.83 ? 2 : (ks < 5.66 ? 4 : 8));
  const long n = (long)tiles_m * tiles_n, ppx = (n + 7) / 8;
  const long g = (k * ppx + tiles_n / 2) / tiles_n;
  return (int)std::max<long>(1, std::min<long>(g, tiles_m));
}

// Tile configurations of the bf16 kernel.
struct TileCfg { int bm, bn, bk, waves; };
static const TileCfg kCfgs[] = {
    {128, 128, 64, 4},   // 0: two workgroups per CU; small or ragged problems
    {256, 128, 64, 8},   // 1
    {256, 256, 64, 8},   // 2: least LDS and L2 traffic per FLOP; large problems
    {128, 256, 64, 8},   // 3
    {256, 128, 32, 8},   // 4: shallower k-tile, two workgroups per CU
    {128, 128, 32, 4},   // 5
};
constexpr int kNumCfgs = sizeof(kCfgs) / sizeof(kCfgs[0]);
constexpr int kCUs = 256;

// Split-K factor of the fp32-output (weight-gradient) GEMMs: the largest power of two that keeps every
// workgroup of the launch resident at once (`slots` = CUs x workgroups per CU of the configuration), with
// at least 8 64-deep k-tiles per split and at most 32 partial sums to reduce.  A launch that spills into a
// second round loses what the extra splits gained (90 tiles of 256x256, one per CU: 2 splits run 10 %
// faster than 4 on the bare GEMM).  Inside the stage these GEMMs run on the side stream under the main
// stream's kernels and every policy tried, a split count that is not a power of two included, stays
// within 0.5 % of the step time.
static int choose_splits(long tiles, int kt, int slots) {
  const long cap = std::min<long>(std::min<long>(slots / std::max<long>(tiles, 1), kt / 8), 32);
  int s = 1;
  while (2 * s <= cap) s *= 2;
  return s;
}

// Split-K factor of a GEMM with a storage-dtype output (second pass: reduce_epilogue_kernel).  It pays
// where a few tiles would each walk the contraction alone while most CUs idle: the frozen encoder's
// projections on a partial batch (6 to 72 tiles of 128x128, K = 768 or 3072).  Measured on MI355X, encoder
// forward in samples/s without and with it: 1074 -> 1450 (slices of 1 sample), 4118 -> 5224 (4), 15881 ->
// 18057 (16).  The second pass costs a launch and the partial sums' traffic, so a short contraction
// (K < 2048) is split only up to 48 tiles (at 54 and 72 tiles it lost 9 %), a long one up to 96 (at 120
// tiles, 64 samples, the gain is cancelled).  At least 6 64-deep k-tiles per split; 3 or 12 measured no better.
static int choose_splits_epi(long tiles, int kt) {
  if (kt < 12 || tiles > (kt >= 32 ? 96 : 48)) return 1;
  const long cap = std::min<long>(std::min<long>(kCUs / std::max<long>(tiles, 1), kt / 6), 16);
  int s = 1;
  while (2 * s <= cap) s *= 2;
  return s;
}

// The same when the choice is made for `choice_rows` rows (GemmArgs::choice_rows) but M rows are computed.
size_t gemm_epi_splitk_ws_bytes_for(int M, int N, int K, int choice_rows) {
  size_t worst = 0;
  const int shapes[][2] = {{64, 64}, {128, 128}, {256, 128}, {256, 256}};
  for (const auto& t : shapes) {
    const long tiles = (long)((choice_rows + t[0] - 1) / t[0]) * ((N + t[1] - 1) / t[1]);
    const int sp = choose_splits_epi(tiles, K / 64);
    if (sp > 1) worst = std::max(worst, (size_t)sp * M * N * sizeof(float));
  }
  return worst;
}

size_t gemm_epi_splitk_ws_bytes(int M, int N, int K) {
  size_t worst = 0;
  const int shapes[][2] = {{64, 64}, {128, 128}, {256, 128}, {256, 256}};
  for (const auto& t : shapes) {
    const long tiles = (long)((M + t[0] - 1) / t[0]) * ((N + t[1] - 1) / t[1]);
    const int sp = choose_splits_epi(tiles, K / 64);
    if (sp > 1) worst = std::max(worst, (size_t)sp * M * N * sizeof(float));
  }
  return worst;
}

// Picks the tile configuration (indices as in launch_gemm's switch), from sweeps of all GEMM shapes of
// the five workloads on MI355X:
//  - y = x W^T (both operands K-contiguous; also dx = dy W on transposed weight copies): the
//    direct-to-LDS kernels, tile chosen by the cost model below;
//  - dx = dy W with W as stored (fp32-free fallback when no transposed copy exists): 256x256
//    direct-to-LDS tiles when they fill the CUs, else the register-staged kernel;
//  - dW = dy^T x (both operands read through the transposing LDS load): register-staged 128x128 tiles,
//    two workgroups per CU; 256x256 direct-to-LDS tiles for large M and N.
static int choose_cfg(int M, int N, int K, bool a_mc, bool b_mc, bool dtl_ok, bool allow16 = true) {
  const long t256x256 = (long)((M + 255) / 256) * ((N + 255) / 256);
  const long t256x128 = (long)((M + 255) / 256) * ((N + 127) / 128);
  const bool dtl32 = dtl_ok && K % 32 == 0, dtl64 = dtl_ok && K % 64 == 0;
  if (a_mc) return (dtl32 && b_mc && t256x256 >= 80) ? 6 : 0;
  if (!b_mc) {
    // y = x W^T on contraction-contiguous operands: pick the direct-to-LDS tile with the least
    // (rounds over the 256 CUs) x (tile area / measured relative efficiency).  The efficiencies were
    // fitted on MI355X over the GEMM shapes of the five workloads: 256x256 tiles move the fewest LDS
    // and L1 bytes per FLOP; 256x160 (16x16x32 MFMA tiles) exists for widths that leave the others
    // with padded columns or a badly filled last round (N = 320, 1152, 2560).  A 192x128 tile for
    // N = 640 (215 instead of 160 workgroups) won 5 % on bare GEMMs and lost 2 % inside the stage.
    // A few hundred rows and a short contraction (the frozen encoder's projections on a partial batch): 64x64 tiles give
    // 4x the workgroups of 128x128 ones, each with a quarter of the work per k-tile, and no split-K pass is needed.
    // Measured on the text encoder (samples/s at slices of 1 / 4 / 16): 1538 / 5617 / 19148 -> 1733 / 6490 / 20040; with more
    // 128x128 tiles than the limits below the larger tiles win again (16 samples, K = 3072: -6 % with 64x64 tiles).
    if (dtl64 && (long)((M + 127) / 128) * ((N + 127) / 128) <= (K <= 1024 ? 100 : 24)) return 15;
    struct Cand { int idx, bm, bn; float eff; bool need64; };
    // Two 256x128 workgroups per CU (configuration 12, three 32-deep buffers) hide each other's prologue,
    // epilogue and barrier stalls: the shorter the contraction and the more tiles per CU, the more it pays.
    const float eff12 = t256x128 <= kCUs ? 0.95f : (K <= 384 ? 1.6f : (K <= 768 ? 1.25f : (K <= 1536 ? 1.15f : 0.9f)));
    const Cand cands[] = {{6, 256, 256, 1.27f, false}, {11, 256, 160, 1.01f, true}, {12, 256, 128, eff12, false},
                          {9, 256, 128, 1.00f, true}, {13, 128, 128, 0.98f, true}, {8, 128, 128, 0.85f, false}};
    int best = -1;
    float best_cost = 0.f;
    for (const Cand& c : cands) {
      if (c.need64 ? !dtl64 : !dtl32) continue;
      if (c.idx == 11 && !allow16) continue;       // the 16x16x32 instruction sums a k-step of 32 at once: other bits than the 32x32x16 tiles
      const long tiles = (long)((M + c.bm - 1) / c.bm) * ((N + c.bn - 1) / c.bn);
      const float cost = (float)((tiles + kCUs - 1) / kCUs) * (float)(c.bm * c.bn) / c.eff;
      if (best < 0 || cost < best_cost) { best = c.idx; best_cost = cost; }
    }
    if (best >= 0) return best;
    return t256x128 >= 128 ? 1 : 0;
  }
  if (dtl32 && t256x256 >= 128) return 6;
  if (dtl32 && K <= 1024) return 8;
  if (K >= 2 * N && t256x256 >= 128) return 2;
  return t256x128 >= 128 ? 1 : 0;
}

size_t gemm_splitk_ws_bytes(int M, int N, int K) {
  size_t worst = 0;
  for (int c = 0; c < kNumCfgs; ++c) {
    const long tiles = (long)((M + kCfgs[c].bm - 1) / kCfgs[c].bm) * ((N + kCfgs[c].bn - 1) / kCfgs[c].bn);
    const int s = choose_splits(tiles, (K + kCfgs[c].bk - 1) / kCfgs[c].bk, 2 * kCUs);
    if (s > 1) worst = std::max(worst, (size_t)s * ((size_t)M * N + M) * sizeof(float));   // + the column sums of A per split
  }
  return worst;
}

template <int BM, int BN, int BK, int WGM, int WGN, bool A_MC, bool B_MC>
static int launch_bf16_cfg(const GemmArgs& a, hipStream_t s) {
  using S = GemmSmem<BM, BN, BK, WGM, WGN, A_MC, B_MC>;
  GemmBf16Params p;
  p.A = (const bf16*)a.A; p.B = (const bf16*)a.B;
  p.M = a.M; p.N = a.N; p.K = a.K; p.lda = a.lda; p.ldb = a.ldb; p.split_major = 0;
  p.epi = make_epi<bf16>(a);
  p.tiles_m = (a.M + BM - 1) / BM; p.tiles_n = (a.N + BN - 1) / BN;
  p.group_m = choose_group_m(a, p.tiles_m, p.tiles_n);
  const int kt = (a.K + BK - 1) / BK;
  int splits = 1;
  if (a.out_f32) {
    splits = choose_splits((long)p.tiles_m * p.tiles_n, kt, S::BYTES <= 80 * 1024 ? 2 * kCUs : kCUs);
    if (splits > 1) {
      const size_t need = (size_t)splits * ((size_t)a.M * a.N + (a.colsum_out ? a.M : 0)) * sizeof(float);
      if (!a.splitk_ws || a.splitk_ws_bytes < need) splits = 1;
    }
  }
  p.k_tiles_per_split = (kt + splits - 1) / splits;
  splits = (kt + p.k_tiles_per_split - 1) / p.k_tiles_per_split;
  if (splits > 1) p.epi.partial = a.splitk_ws;
  float* colsum_ws = nullptr;
  p.colsum = nullptr; p.colsum_stride = 0; p.colsum_acc = 0;
  if (A_MC && a.colsum_out) {
    if (!a.out_f32) return set_error(DP_EUNSUPPORTED, "gemm: column sums come with an fp32 output only");
    if (splits > 1) { colsum_ws = a.splitk_ws + (size_t)splits * a.M * a.N; p.colsum = colsum_ws; p.colsum_stride = a.M; }
    else { p.colsum = a.colsum_out; p.colsum_acc = a.accumulate; }
  }
  dim3 grid(p.tiles_m * p.tiles_n, 1, splits);
  p.split_major = 0;
  if (splits > 1) { p.split_major = splits; grid = dim3(p.tiles_m * p.tiles_n * splits, 1, 1); }
  const size_t smem = S::BYTES;
  auto kern = gemm_bf16_kernel<BM, BN, BK, WGM, WGN, A_MC, B_MC>;
  static std::atomic<bool> attr_set{false};   // setting it twice is harmless; the flag only saves the call
  if (!attr_set.load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
      return set_error(DP_EHIP, "hipFuncSetAttribute(gemm) failed");
    attr_set.store(true, std::memory_order_release);
  }
  {
    // the timing scope brackets the GEMM kernel alone (the split-K reduction is its own class)
    KScope ks(a.a_mc ? KK_GEMM_TN : (a.b_mc ? KK_GEMM_NN : KK_GEMM_NT), 2.0 * a.M * a.N * a.K,
              gemm_tensor_bytes(a), s, a.M, a.N, a.K);
    hipLaunchKernelGGL(kern, grid, dim3(WGM * WGN * 64), smem, s, p);
  }
  if (hipGetLastError() != hipSuccess) return set_error(DP_EHIP, "gemm launch failed");
  if (splits > 1) {
    KScope ks(KK_REDUCE, 0.0, 4.0 * (splits + 1.0) * a.M * a.N, s, a.M, a.N, splits);
    return launch_reduce_partials2(a.splitk_ws, splits, (size_t)a.M * a.N, a.out_f32, colsum_ws, colsum_ws ? (size_t)a.M : 0,
                                   a.colsum_out, a.accumulate, s);
  }
  return DP_OK;
}

template <int BM, int BN, int BK, int STAGES, int WGM, int WGN, bool A_MC, bool B_MC>
static int launch_dtl_cfg(const GemmArgs& a, hipStream_t s) {
  using S = DtlSmem<BM, BN, BK, STAGES, WGM, WGN>;
  GemmBf16Params p;
  p.A = (const bf16*)a.A; p.B = (const bf16*)a.B;
  p.M = a.M; p.N = a.N; p.K = a.K; p.lda = a.lda; p.ldb = a.ldb; p.split_major = 0;
  p.epi = make_epi<bf16>(a);
  p.tiles_m = (a.M + BM - 1) / BM; p.tiles_n = (a.N + BN - 1) / BN;
  p.group_m = choose_group_m(a, p.tiles_m, p.tiles_n);
  if (!dtl_addressable(a)) return set_error(DP_EUNSUPPORTED, "gemm: operand too large for the forced direct-to-LDS configuration");
  p.a_bytes = (uint32_t)(A_MC ? operand_extent_bytes(a.K, a.M, a.lda) : operand_extent_bytes(a.M, a.K, a.lda));
  p.b_bytes = (uint32_t)(B_MC ? operand_extent_bytes(a.K, a.N, a.ldb) : operand_extent_bytes(a.N, a.K, a.ldb));
  const int kt = a.K / BK;
  int splits = 1;
  if (a.out_f32) {
    splits = choose_splits((long)p.tiles_m * p.tiles_n, kt * BK / 64, S::BYTES <= 80 * 1024 ? 2 * kCUs : kCUs);
  } else if (a.splitk_ws && a.geglu != 1) {
    const long rows_for_choice = a.choice_rows > 0 ? a.choice_rows : a.M;
    splits = a.choice_rows < 0 ? 1 : choose_splits_epi(((rows_for_choice + BM - 1) / BM) * p.tiles_n, kt * BK / 64);
  }
  if (splits > 1) {
    const size_t need = (size_t)splits * a.M * a.N * sizeof(float);
    if (!a.splitk_ws || a.splitk_ws_bytes < need) {
      // with choice_rows the split is part of what the caller asked for: running unsplit would silently change the sums
      if (a.choice_rows > 0) return set_error(DP_EWORKSPACE, "gemm: split-K workspace too small for the split chosen from choice_rows");
      splits = 1;
    }
  }
  p.k_tiles_per_split = (kt + splits - 1) / splits;
  splits = (kt + p.k_tiles_per_split - 1) / p.k_tiles_per_split;
  if (splits > 1) p.epi.partial = a.splitk_ws;
  dim3 grid(p.tiles_m * p.tiles_n, 1, splits);
  const size_t smem = S::BYTES;
  auto kern = gemm_bf16_dtl_kernel<BM, BN, BK, STAGES, WGM, WGN, A_MC, B_MC>;
  static std::atomic<bool> attr_set{false};   // setting it twice is harmless; the flag only saves the call
  if (!attr_set.load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
      return set_error(DP_EHIP, "hipFuncSetAttribute(gemm) failed");
    attr_set.store(true, std::memory_order_release);
  }
  {
    // the timing scope brackets the GEMM kernel alone (the split-K reduction is its own class)
    KScope ks(a.a_mc ? KK_GEMM_TN : (a.b_mc ? KK_GEMM_NN : KK_GEMM_NT), 2.0 * a.M * a.N * a.K,
              gemm_tensor_bytes(a), s, a.M, a.N, a.K);
    hipLaunchKernelGGL(kern, grid, dim3(WGM * WGN * 64), smem, s, p);
  }
  if (hipGetLastError() != hipSuccess) return set_error(DP_EHIP, "gemm launch failed");
  if (a.ln_applied) *a.ln_applied = 0;
  if (splits > 1 && !a.out_f32 && a.ln_out && a.ln_applied && a.ln_gamma && a.ln_beta && a.residual && a.residual_f32 && a.out_fused_f32 &&
      a.out == a.residual && a.ldo == a.N && a.ld_res == a.N && !a.act && !a.dact_pre && !a.gate && !a.pre_out && !a.geglu && a.N <= 2048) {
    // the reduction pass also normalises the rows it completes (one launch less per projection onto the residual stream)
    *a.ln_applied = 1;
    return launch_reduce_residual_ln(a.splitk_ws, splits, a.M, a.N, a.bias, (float*)a.out, a.ln_out, a.ln_gamma, a.ln_beta, a.ln_eps, s);
  }
  if (splits > 1 && !a.out_f32) {
    KScope ks(KK_REDUCE, 0.0, 4.0 * splits * a.M * a.N + 2.0 * a.M * a.N, s, a.M, a.N, splits);
    const size_t groups = (size_t)a.M * (a.N / 8);
    hipLaunchKernelGGL(reduce_epilogue_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, s, make_epi<bf16>(a), a.splitk_ws, splits);
    return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "gemm split-K epilogue launch failed");
  }
  if (splits > 1) {
    KScope ks(KK_REDUCE, 0.0, 4.0 * (splits + 1.0) * a.M * a.N, s, a.M, a.N, splits);
    return launch_reduce_partials(a.splitk_ws, splits, (size_t)a.M * a.N, a.out_f32, a.accumulate, s);
  }
  return DP_OK;
}

// C = out_scale * (A_q B_q^T) (+ bias) for OCP E4M3 operands A_q [M, K], B_q [N, K] (bytes, contraction contiguous), storage-dtype
// (bf16) output.  The kernel sees the operands as two-byte elements: K / 2 of them per row.
template <int BM, int BN, int WGM, int WGN>
static int launch_fp8_cfg(const Fp8GemmArgs& a, hipStream_t s) {
  constexpr int BK = 64, STAGES = 3;
  using S = DtlSmem<BM, BN, BK, STAGES, WGM, WGN>;
  GemmBf16Params p;
  memset(&p, 0, sizeof(p));
  p.A = (const bf16*)a.A; p.B = (const bf16*)a.B;
  p.M = a.M; p.N = a.N; p.K = a.K / 2; p.lda = a.lda / 2; p.ldb = a.ldb / 2;
  EpiParams<bf16>& e = p.epi;
  e.M = a.M; e.N = a.N; e.out = (bf16*)a.out; e.ldo = a.ldo; e.bias = (const bf16*)a.bias; e.rows_per_batch = 1; e.out_scale = a.out_scale;
  p.tiles_m = (a.M + BM - 1) / BM; p.tiles_n = (a.N + BN - 1) / BN;
  GemmArgs shape; memset(&shape, 0, sizeof(shape)); shape.M = a.M; shape.N = a.N;
  p.group_m = choose_group_m(shape, p.tiles_m, p.tiles_n);
  p.a_bytes = (uint32_t)((size_t)(a.M - 1) * a.lda + a.K);
  p.b_bytes = (uint32_t)((size_t)(a.N - 1) * a.ldb + a.K);
  p.k_tiles_per_split = p.K / BK;
  auto kern = gemm_bf16_dtl_kernel<BM, BN, BK, STAGES, WGM, WGN, false, false, true>;
  if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)S::BYTES) != hipSuccess)
    return set_error(DP_EHIP, "hipFuncSetAttribute(gemm fp8) failed");
  KScope ks(KK_GEMM_FP8, 2.0 * a.M * a.N * a.K, (double)a.M * a.K + (double)a.N * a.K + 2.0 * a.M * a.N, s, a.M, a.N, a.K);
  hipLaunchKernelGGL(kern, dim3(p.tiles_m * p.tiles_n, 1, 1), dim3(WGM * WGN * 64), S::BYTES, s, p);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "gemm fp8 launch failed");
}

int launch_gemm_fp8(const Fp8GemmArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return set_error(DP_EINVAL, "gemm fp8: non-positive size");
  if (!a.A || !a.B || !a.out) return set_error(DP_EINVAL, "gemm fp8: null operand");
  if (a.K % 128) return set_error(DP_EUNSUPPORTED, "gemm fp8: K must be a multiple of 128");
  if (a.lda % 16 || a.ldb % 16 || a.lda < a.K || a.ldb < a.K) return set_error(DP_EUNSUPPORTED, "gemm fp8: leading dims must be multiples of 16 bytes and at least K");
  if (a.N % 8 || a.ldo % 8 || a.ldo < a.N) return set_error(DP_EUNSUPPORTED, "gemm fp8: N and ldc must be multiples of 8, ldc >= N");
  if (!(a.out_scale > 0.f)) return set_error(DP_EINVAL, "gemm fp8: the output scale must be positive");
  const void* ps[] = {a.A, a.B, a.out, a.bias};
  for (const void* q : ps) if ((uintptr_t)q % 16) return set_error(DP_EALIGN, "gemm fp8: operands must be 16-byte aligned");
  if ((size_t)(a.M - 1) * a.lda + a.K >= (1ull << 32) || (size_t)(a.N - 1) * a.ldb + a.K >= (1ull << 32))
    return set_error(DP_EUNSUPPORTED, "gemm fp8: operand larger than 4 GiB");
  const long t256 = (long)((a.M + 255) / 256) * ((a.N + 127) / 128);
  if (t256 >= kCUs / 2) return launch_fp8_cfg<256, 128, 4, 2>(a, s);
  return launch_fp8_cfg<128, 128, 4, 2>(a, s);
}

template <int BM, int BN, int WGM, int WGN>
static int launch_dtl16(const GemmArgs& a, hipStream_t s) {
  using S = Dtl16Smem<BM, BN, 3, WGM, WGN>;
  if (a.a_mc || a.b_mc || a.out_f32 || a.K % 64) return set_error(DP_EUNSUPPORTED, "gemm: forced 16x16-tile configuration needs contraction-contiguous operands, a storage-dtype output and K % 64 == 0");
  if (!dtl_addressable(a)) return set_error(DP_EUNSUPPORTED, "gemm: operand too large for the forced direct-to-LDS configuration");
  GemmBf16Params p;
  p.A = (const bf16*)a.A; p.B = (const bf16*)a.B;
  p.M = a.M; p.N = a.N; p.K = a.K; p.lda = a.lda; p.ldb = a.ldb; p.split_major = 0;
  p.epi = make_epi<bf16>(a);
  p.tiles_m = (a.M + BM - 1) / BM; p.tiles_n = (a.N + BN - 1) / BN;
  p.group_m = choose_group_m(a, p.tiles_m, p.tiles_n);
  p.a_bytes = (uint32_t)operand_extent_bytes(a.M, a.K, a.lda);
  p.b_bytes = (uint32_t)operand_extent_bytes(a.N, a.K, a.ldb);
  p.k_tiles_per_split = a.K / 64;
  auto kern = gemm_bf16_dtl16_kernel<BM, BN, 3, WGM, WGN>;
  static std::atomic<bool> attr_set{false};   // setting it twice is harmless; the flag only saves the call
  if (!attr_set.load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)S::BYTES) != hipSuccess)
      return set_error(DP_EHIP, "hipFuncSetAttribute(gemm) failed");
    attr_set.store(true, std::memory_order_release);
  }
  KScope ks(KK_GEMM_NT, 2.0 * a.M * a.N * a.K, gemm_tensor_bytes(a), s, a.M, a.N, a.K);
  hipLaunchKernelGGL(kern, dim3(p.tiles_m * p.tiles_n), dim3(WGM * WGN * 64), S::BYTES, s, p);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "gemm launch failed");
}

template <int BM, int BN, int BK, int STAGES, int WGM, int WGN>
static int launch_dtl_layout(const GemmArgs& a, hipStream_t s) {
  if (a.K % BK) return set_error(DP_EUNSUPPORTED, "gemm: K is not a multiple of the k-tile of the forced configuration");
  if (!a.a_mc && !a.b_mc) return launch_dtl_cfg<BM, BN, BK, STAGES, WGM, WGN, false, false>(a, s);
  if (!a.a_mc && a.b_mc) return launch_dtl_cfg<BM, BN, BK, STAGES, WGM, WGN, false, true>(a, s);
  if (a.a_mc && a.b_mc) return launch_dtl_cfg<BM, BN, BK, STAGES, WGM, WGN, true, true>(a, s);
  return launch_dtl_cfg<BM, BN, BK, STAGES, WGM, WGN, true, false>(a, s);
}

template <int BM, int BN, int BK, int WGM, int WGN>
static int launch_bf16_layout(const GemmArgs& a, hipStream_t s) {
  if (!a.a_mc && !a.b_mc) return launch_bf16_cfg<BM, BN, BK, WGM, WGN, false, false>(a, s);
  if (!a.a_mc && a.b_mc) return launch_bf16_cfg<BM, BN, BK, WGM, WGN, false, true>(a, s);
  if (a.a_mc && a.b_mc) return launch_bf16_cfg<BM, BN, BK, WGM, WGN, true, true>(a, s);
  return launch_bf16_cfg<BM, BN, BK, WGM, WGN, true, false>(a, s);
}

// The bias gradient can ride in a weight-gradient GEMM when that GEMM runs on the register-staged kernel.
bool gemm_colsum_supported(const GemmArgs& a) {
  if (a.dtype != BF16 || !a.a_mc || !a.b_mc || !a.out_f32 || a.M % 8) return false;
  const int cfg = (a.force_cfg > 0) ? a.force_cfg - 1 : choose_cfg(a.M, a.N, a.K, true, true, dtl_addressable(a));
  return cfg >= 0 && cfg <= 5;
}

bool gemm_geglu_fwd_supported(const GemmArgs& a) {
  return a.dtype == BF16 && !a.a_mc && !a.b_mc && a.K % 32 == 0 && a.geglu_inner > 0 && a.geglu_inner % 32 == 0 &&
         a.N == 2 * a.geglu_inner && a.ldo >= a.geglu_inner && (!a.pre_out || a.ld_pre >= a.N) && dtl_addressable(a);
}

int gemm_choose_cfg(int M, int N, int K) { return choose_cfg(M, N, K, false, false, true); }

int launch_gemm(const GemmArgs& a, hipStream_t s) {
  if (a.ln_applied) *a.ln_applied = 0;
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return set_error(DP_EINVAL, "gemm: non-positive size");
  if (!a.A || !a.B || (!a.out && !a.out_f32)) return set_error(DP_EINVAL, "gemm: null operand");
  if (a.out_f32 && a.ldo32 < a.N) return set_error(DP_EINVAL, "gemm: ldo32 < N");
  if (a.out_f32 && a.ldo32 != a.N) return set_error(DP_EUNSUPPORTED, "gemm: fp32 output must be dense");
  if (a.colsum_out && !gemm_colsum_supported(a)) return set_error(DP_EUNSUPPORTED, "gemm: column sums are not available for this problem");
  if (a.dtype == BF16) {
    // 16-byte vector loads: every row start and the contiguous extent must be multiples of 8 elements
    const int a_inner = a.a_mc ? a.M : a.K, b_inner = a.b_mc ? a.N : a.K;
    if ((a.lda % 8) || (a.ldb % 8) || (a_inner % 8) || (b_inner % 8))
      return set_error(DP_EUNSUPPORTED, "gemm(bf16): leading dims and contiguous extents must be multiples of 8");
    if (((uintptr_t)a.A % 16) || ((uintptr_t)a.B % 16)) return set_error(DP_EALIGN, "gemm(bf16): operands must be 16-byte aligned");
    if (a.lda < a_inner || a.ldb < b_inner) return set_error(DP_EINVAL, "gemm: leading dim too small");
    if (a.N % 8) return set_error(DP_EUNSUPPORTED, "gemm(bf16): N must be a multiple of 8");
    if (a_inner < 8 || b_inner < 8) return set_error(DP_EUNSUPPORTED, "gemm(bf16): contiguous extents must be at least 8");
    const int elds[] = {a.out ? a.ldo : 8, a.pre_out ? a.ld_pre : 8, a.dact_pre ? a.ld_dact : 8, a.gate ? a.gate_ld : 8, a.residual ? a.ld_res : 8};
    for (int x : elds) if (x % 8 || x < 8) return set_error(DP_EUNSUPPORTED, "gemm(bf16): epilogue leading dims must be multiples of 8");
    const void* eps[] = {a.out, a.out_f32, a.bias, a.pre_out, a.dact_pre, a.gate, a.residual, a.splitk_ws};
    for (const void* x : eps) if ((uintptr_t)x % 16) return set_error(DP_EALIGN, "gemm(bf16): epilogue operands must be 16-byte aligned");
    if (a.geglu) {
      if (a.geglu != 1 && a.geglu != 2) return set_error(DP_EINVAL, "gemm: bad geglu mode");
      if (!a.out || a.out_f32 || a.act || a.dact_pre || a.gate || a.residual || a.out_fused_f32)
        return set_error(DP_EUNSUPPORTED, "gemm: a GeGLU epilogue combines with a bias only");
      if (a.geglu == 1 && !gemm_geglu_fwd_supported(a)) return set_error(DP_EUNSUPPORTED, "gemm: fused GeGLU forward not available for this problem");
      if (a.geglu == 2) {
        if (a.N != a.geglu_inner || a.geglu_inner % 8 || !a.geglu_u || a.ld_geglu % 8 || a.ld_geglu < 2 * a.geglu_inner ||
            a.ldo < 2 * a.geglu_inner || a.pre_out || ((uintptr_t)a.geglu_u % 16))
          return set_error(DP_EINVAL, "gemm: bad fused GeGLU backward arguments");
      }
    }
    int cfg = (a.force_cfg > 0 && a.force_cfg <= kNumCfgs + 11) ? a.force_cfg - 1 : choose_cfg(a.choice_rows > 0 ? a.choice_rows : a.M, a.N, a.K, a.a_mc != 0, a.b_mc != 0, dtl_addressable(a), a.choice_rows >= 0);
    if (a.geglu == 1 && (cfg < 6 || cfg > 14 || cfg == 11)) {   // cfg 11 has no column permutation in its loader either
      // the column permutation lives in the direct-to-LDS loader
      const long t256x256 = (long)((a.M + 255) / 256) * ((a.N + 255) / 256);
      cfg = t256x256 >= 128 ? 6 : 8;
    }
    switch (cfg) {
      case 1: return launch_bf16_layout<256, 128, 64, 4, 2>(a, s);
      case 2: return launch_bf16_layout<256, 256, 64, 2, 4>(a, s);
      case 3: return launch_bf16_layout<128, 256, 64, 2, 4>(a, s);
      case 4: return launch_bf16_layout<256, 128, 32, 4, 2>(a, s);
      case 5: return launch_bf16_layout<128, 128, 32, 2, 2>(a, s);
      case 6: return launch_dtl_layout<256, 256, 32, 4, 2, 4>(a, s);
      case 7: return launch_dtl_layout<256, 128, 32, 4, 4, 2>(a, s);
      case 8: return launch_dtl_layout<128, 128, 32, 4, 2, 2>(a, s);
      case 9: return launch_dtl_layout<256, 128, 64, 3, 4, 2>(a, s);
      case 10: return launch_dtl_layout<128, 128, 64, 3, 2, 2>(a, s);
      case 11: return launch_dtl16<256, 160, 4, 2>(a, s);
      case 12: return launch_dtl_layout<256, 128, 32, 3, 4, 2>(a, s);   // 72 KB of LDS: two workgroups per CU
      case 13: return launch_dtl_layout<128, 128, 64, 3, 4, 2>(a, s);   // eight waves on a 128x128 tile
      case 14: return launch_dtl_layout<128, 128, 32, 4, 4, 2>(a, s);
      // small tiles: many workgroups for problems of a few hundred rows (contraction-contiguous operands only: the chunk
      // permutation of a contraction-strided tile needs at least 128 columns)
      case 15:
      case 16:
        if (a.a_mc || a.b_mc || a.K % 64) return set_error(DP_EUNSUPPORTED, "gemm: the forced 64-row configurations need contraction-contiguous operands and K % 64 == 0");
        return cfg == 15 ? launch_dtl_cfg<64, 64, 64, 3, 2, 2, false, false>(a, s) : launch_dtl_cfg<64, 128, 64, 3, 2, 2, false, false>(a, s);
      default: break;
    }
    return launch_bf16_layout<128, 128, 64, 2, 2>(a, s);
  }
  GemmF32Params p;
  p.A = (const float*)a.A; p.B = (const float*)a.B;
  p.M = a.M; p.N = a.N; p.K = a.K; p.lda = a.lda; p.ldb = a.ldb; p.a_mc = a.a_mc; p.b_mc = a.b_mc;
  p.epi = make_epi<float>(a);
  dim3 grid((a.N + 63) / 64, (a.M + 63) / 64, 1);
  KScope ks(KK_GEMM_F32, 2.0 * a.M * a.N * a.K, 4.0 * ((double)a.M * a.K + (double)a.N * a.K + (double)a.M * a.N), s, a.M, a.N, a.K);
  hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, s, p);
  if (hipGetLastError() != hipSuccess) return set_error(DP_EHIP, "gemm(f32) launch failed");
  return DP_OK;
}

}  // namespace dp
