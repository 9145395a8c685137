// Fused softmax attention, forward and backward, for self-attention (N keys),
// cross-attention to the text context (77 keys) and the text encoder's causal attention.
//
// bf16 path (MFMA 32x32x16, wave64).  A wave owns 32 queries (forward, dQ) or 32 keys
// (dK/dV) and keeps them in registers as the MFMA B operand; the other side streams
// through LDS in 64-row tiles.  Scores are produced transposed (S^T = K Q^T) so that a
// lane holds one query column: the online-softmax statistics are lane-local, and the
// probability block, once rounded to bf16, already has the register layout of the B
// operand of the second product (O^T = V^T P^T).  The operand that needs its
// contraction index moved (V, and K/Q/dO in the backward) is read from its row-major
// LDS tile with the transposing LDS load.  The backward is split into a dQ kernel and
// a dK/dV kernel so that no floating-point atomics are needed (run-to-run identical).
// The streamed tiles are copied global -> LDS directly (`buffer_load ... lds`) into unpadded tiles whose
// 16-byte chunks are permuted per row, so that both ways of reading a tile stay free of bank conflicts.
//
// fp32 path: one wave per query (or key) row, plain FMA; used by the small fp32
// configuration only.
#include "dp_device.h"
#include "dp_kernels.h"
#include "dp_errors.h"
#include "dp_ktime.h"
#include <math.h>
#include <algorithm>

namespace dp {

struct AttnK {
  int B, H, Nq, Nk, dh;
  float scale_log2;   // scale * log2(e)
  float scale;
  const void* q; int ldq;
  const void* k; int ldk;
  const void* v; int ldv;
  void* o; int ldo;
  float* lse;
  const void* dout; int lddo;
  float* delta;
  void* dq; int lddq;
  void* dk; int lddk;
  void* dv; int lddv;
  int qsplits; float* dkv_partial;   // dK/dV kernel: query range split + fp32 partial outputs [2][qsplits][B * Nk][H * dh]
};

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// Layout of a streamed [64 x DHP] bf16 tile in LDS: 64 rows of DHP / 8 16-byte chunks, no padding; the chunk
// at position pos of a row is chunk pos ^ key(row).  A tile is read two ways -- by rows as an MFMA A operand
// (16 consecutive rows, one chunk each, per 256 bytes of LDS bandwidth) and through the transposing load (4
// consecutive rows x 64 bytes) -- and the key keeps both conflict-free:
//   DHP = 64 (128-byte rows): key = row bits (0, 2, 1): a bijection of row & 7 whose bit 2 is row bit 1, so
//     8 consecutive rows land in 8 different positions and the 4 rows of a transposing read in 4 different
//     64-byte bank groups;
//   DHP = 96 (192-byte rows): consecutive rows already start 192 bytes apart, i.e. in different 64-byte groups;
//     rows r and r + 4 share one, so key = (row >> 2) & 3 moves them apart inside the group.
template <int DHP> struct AttnTile;
template <> struct AttnTile<64> {
  static constexpr int PIECES = 2;     // 1 KB copy instructions per wave and tile (16 rows)
  static __device__ __forceinline__ int key(int row) { return (row & 1) | ((row & 4) >> 1) | ((row & 2) << 1); }
};
template <> struct AttnTile<96> {
  static constexpr int PIECES = 3;
  static __device__ __forceinline__ int key(int row) { return (row >> 2) & 3; }
};

// Global -> LDS copy of one tile (`buffer_load ... lds`: the wave's 64 x 16 bytes land contiguously in LDS).
// A wave owns rows 16 * wave .. + 15; each lane keeps the byte offset, inside the (batch, head) slice, of the
// chunk that belongs at its LDS position.  Chunks past d_head get an offset of 2^31, which stays outside the
// buffer descriptor's range whatever tile offset is added: they, like rows past the end of the slice, arrive
// as zeros without touching memory.
template <int DHP>
struct AttnTileCopy {
  using T = AttnTile<DHP>;
  uint32_t off[T::PIECES];
  __device__ __forceinline__ void init(int wave, int lane, int ld, int dh) {
#pragma unroll
    for (int j = 0; j < T::PIECES; ++j) {
      const int o = 1024 * j + 16 * lane;                     // byte inside the wave's 16-row block
      const int row = 16 * wave + o / (2 * DHP), pos = (o % (2 * DHP)) / 16;
      const int chunk = pos ^ T::key(row);
      off[j] = 8 * chunk < dh ? (uint32_t)(row * ld + 8 * chunk) * 2u : 0x80000000u;
    }
  }
  // rows row0 .. row0 + 63 of the slice behind r (the tile offset goes into the per-lane offset: only that
  // one is range-checked)
  __device__ __forceinline__ void issue(rsrc_t r, int row0, int ld, bf16* stage, int wave) const {
#pragma unroll
    for (int j = 0; j < T::PIECES; ++j)
      async_copy_16B_buf(r, off[j] + (uint32_t)row0 * (uint32_t)ld * 2u, 0, stage + 16 * wave * DHP + 512 * j);
  }
};

// Per-lane element offsets of the fragment reads, computed once.  A row fragment (rows 32 * t + l32, k-chunk
// c) is at row[c] + 32 * DHP * t.  A transposed fragment in the slot order of frag_from_mc_accorder (rows
// r0 .. r0 + 15 with r0 a multiple of 16, which leaves the keys alone; columns 32 * i .. + 31) is read as two
// halves at tr_lo[i] + DHP * r0 and tr_hi[i] + DHP * r0 (8 rows apart).
template <int DHP>
struct AttnFragOff {
  using T = AttnTile<DHP>;
  int row[DHP / 16], tr_lo[DHP / 32], tr_hi[DHP / 32];
  __device__ __forceinline__ void init(int lane) {
    const int g = lane >> 5, l32 = lane & 31, b = lane >> 4, j = lane & 15;
#pragma unroll
    for (int c = 0; c < DHP / 16; ++c) row[c] = l32 * DHP + 8 * ((2 * c + g) ^ T::key(l32));
    const int r = 4 * (b >> 1) + (j >> 2);
#pragma unroll
    for (int i = 0; i < DHP / 32; ++i) {
      const int chunk = 4 * i + 2 * (b & 1) + ((j & 3) >> 1);
      tr_lo[i] = r * DHP + 8 * (chunk ^ T::key(r)) + 4 * (j & 1);
      tr_hi[i] = (r + 8) * DHP + 8 * (chunk ^ T::key(r + 8)) + 4 * (j & 1);
    }
  }
  __device__ __forceinline__ bf16x8 row_frag(const bf16* tile, int t, int c) const {
    return *reinterpret_cast<const bf16x8*>(tile + row[c] + 32 * DHP * t);
  }
  __device__ __forceinline__ bf16x8 tr_frag(const bf16* tile, int r0, int i) const {
    const bf16x4 lo = lds_read_tr(tile + tr_lo[i] + DHP * r0);
    const bf16x4 hi = lds_read_tr(tile + tr_hi[i] + DHP * r0);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  }
};
// byte extent of a (batch, head) slice of n rows with leading dimension ld (elements), d_head columns
__device__ __forceinline__ uint32_t attn_slice_bytes(int n, int ld, int dh) { return (uint32_t)(((size_t)(n - 1) * ld + dh) * 2); }

__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int off) {
  bf16x8 o;
#pragma unroll
  for (int u = 0; u < 8; ++u) o[u] = (bf16)v[off + u];
  return o;
}

// Maps a linear workgroup id to (tile along the sequence, batch * head).  Hardware deals
// consecutive ids round-robin to the 8 XCDs; with this map all tiles of one (batch, head) run
// on the same XCD, so its K/V (or Q/dO) stream is fetched into one L2 only.
__device__ __forceinline__ void attn_block_map(int id, int ntiles, int BH, int& tile, int& bh) {
  const int full = (BH / 8) * 8;
  if (id < full * ntiles) {
    const int grp = id / (8 * ntiles), r = id % (8 * ntiles);
    bh = grp * 8 + (r & 7);
    tile = r >> 3;
  } else {
    const int r = id - full * ntiles;
    bh = full + r / ntiles;
    tile = r % ntiles;
  }
}

// ------------------------------------------------------------------ forward (bf16)
// A workgroup covers 128 queries (32 per wave) and walks the keys in 64-row tiles, two LDS stages.
template <int DHP, bool CAUSAL>
__global__ void __launch_bounds__(256, DHP == 64 ? 4 : 3) attn_fwd_bf16_kernel(const AttnK p) {
  constexpr int KC = DHP / 16, DT = DHP / 32, BQ = 128, TILE = 64 * DHP;
  __shared__ __attribute__((aligned(1024))) bf16 Ks[2][TILE];
  __shared__ __attribute__((aligned(1024))) bf16 Vs[2][TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, l32 = lane & 31;
  int qtile, bh;
  attn_block_map(blockIdx.x, (p.Nq + BQ - 1) / BQ, p.B * p.H, qtile, bh);
  const int b = bh / p.H, h = bh % p.H;
  const int q0 = qtile * BQ + wave * 32;               // first query of this wave
  const int qi = q0 + l32;
  const bf16* qb = (const bf16*)p.q + (size_t)b * p.Nq * p.ldq + h * p.dh;
  const bf16* kb = (const bf16*)p.k + (size_t)b * p.Nk * p.ldk + h * p.dh;
  const bf16* vb = (const bf16*)p.v + (size_t)b * p.Nk * p.ldv + h * p.dh;
  const rsrc_t kr = make_rsrc(kb, attn_slice_bytes(p.Nk, p.ldk, p.dh));
  const rsrc_t vr = make_rsrc(vb, attn_slice_bytes(p.Nk, p.ldv, p.dh));

  AttnFragOff<DHP> fo;
  fo.init(lane);
  AttnTileCopy<DHP> ck, cv;
  ck.init(wave, lane, p.ldk, p.dh);
  cv.init(wave, lane, p.ldv, p.dh);
  ck.issue(kr, 0, p.ldk, Ks[0], wave);
  cv.issue(vr, 0, p.ldv, Vs[0], wave);

  bf16x8 qf[KC];
#pragma unroll
  for (int c = 0; c < KC; ++c) qf[c] = ld8(qb + (size_t)qi * p.ldq + 16 * c + 8 * g, qi < p.Nq && 16 * c + 8 * g < p.dh);
  f32x16 oacc[DT];
  float m = -INFINITY, lsum = 0.f;
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;

  int nkt = (p.Nk + 63) / 64;
  if (CAUSAL) nkt = min(nkt, (min(p.Nq, qtile * BQ + BQ) + 63) / 64);
  wait_vmcnt<0>();
  __syncthreads();

  for (int kt = 0; kt < nkt; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nkt) {      // every wave left stage buf ^ 1 at the barrier that ended the previous iteration
      ck.issue(kr, (kt + 1) * 64, p.ldk, Ks[buf ^ 1], wave);
      cv.issue(vr, (kt + 1) * 64, p.ldv, Vs[buf ^ 1], wave);
    }
    // S^T = K Q^T
    f32x16 s[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[t][r] = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int c = 0; c < KC; ++c) s[t] = mfma32(fo.row_frag(Ks[buf], t, c), qf[c], s[t]);
    // online softmax, one query column per lane (shared with lane ^ 32).  Masking only in tiles that cross the
    // end of the keys or the causal diagonal (one wave-uniform branch around a block of selects; a test per
    // element would be compiled into a branch per element)
    const bool edge = kt * 64 + 64 > p.Nk || (CAUSAL && kt * 64 + 63 > q0);
    if (edge) {
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kt * 64 + 32 * t + acc_row(r, g);
          const bool dead = key >= p.Nk || (CAUSAL && key > qi);
          s[t][r] = dead ? -INFINITY : s[t][r];
        }
    }
    // running maximum over raw scores (the scale is positive, so it commutes with max)
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[t][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    mx = fmaxf(m, mx * p.scale_log2);                    // m is kept in the scaled (log2) domain
    // The reference point only has to bound the exponents, not equal the maximum: it is moved (and the
    // accumulators rescaled) when some query of the wave has outgrown it by 2^8; until then the
    // probabilities of this tile are taken relative to the old one (at most 256, exact in the final
    // O = acc / sum and LSE = ref + log sum).  Wave-uniform, so the rescale is skipped for most tiles.
    const bool bump = __any(mx > m + 8.0f);
    mx = bump ? mx : m;
    const float mref = (mx == -INFINITY) ? 0.f : mx;
    float rs = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float e = __builtin_amdgcn_exp2f(fmaf(s[t][r], p.scale_log2, -mref));
        s[t][r] = e;
        rs += e;
      }
    rs += __shfl_xor(rs, 32, 64);
    if (bump) {
      const float alpha = __builtin_amdgcn_exp2f(m - mref);
      lsum *= alpha;
#pragma unroll
      for (int i = 0; i < DT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
    }
    lsum += rs;
    m = mx;
    // O^T += V^T P^T
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int cc = 0; cc < 2; ++cc) {
        const bf16x8 pf = pack8(s[t], 8 * cc);
#pragma unroll
        for (int i = 0; i < DT; ++i) oacc[i] = mfma32(fo.tr_frag(Vs[buf], 32 * t + 16 * cc, i), pf, oacc[i]);
      }
    wait_vmcnt<0>();      // this wave's pieces of the next tile have landed
    __syncthreads();      // ... and everybody's; all reads of stage buf are done
  }

  if (qi < p.Nq) {
    const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
    bf16* ob = (bf16*)p.o + ((size_t)b * p.Nq + qi) * p.ldo + h * p.dh;
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int col = 32 * i + 8 * r4 + 4 * g;
        if (col < p.dh) {
          bf16x4 o;
#pragma unroll
          for (int u = 0; u < 4; ++u) o[u] = (bf16)(oacc[i][4 * r4 + u] * inv);
          *reinterpret_cast<bf16x4*>(ob + col) = o;
        }
      }
    if (p.lse && g == 0) p.lse[((size_t)b * p.H + h) * p.Nq + qi] = m * LN2 + logf(lsum);
  }
}

// ------------------------------------------------------------------ delta = rowsum(dO * O)
// 8 lanes per (token, head) pair.
template <typename T>
__global__ void attn_delta_kernel(const T* __restrict__ o, int ldo, const T* __restrict__ dout, int lddo, float* __restrict__ delta,
                                  int B, int H, int Nq, int dh) {
  const size_t gid = (blockIdx.x * (size_t)blockDim.x + threadIdx.x) / 8;
  const int sub = threadIdx.x & 7;
  const size_t total = (size_t)B * Nq * H;
  float s = 0.f;
  if (gid < total) {
    const int h = gid % H; const size_t row = gid / H;   // row = b * Nq + n
    const T* po = o + row * ldo + h * dh;
    const T* pd = dout + row * lddo + h * dh;
    for (int t = sub; t < dh; t += 8) s += to_f<T>(po[t]) * to_f<T>(pd[t]);
  }
  s += __shfl_xor(s, 1, 64); s += __shfl_xor(s, 2, 64); s += __shfl_xor(s, 4, 64);
  if (gid < total && sub == 0) {
    const int h = gid % H; const size_t row = gid / H;
    const size_t b = row / Nq, n = row % Nq;
    delta[(b * H + h) * Nq + n] = s;
  }
}

// ------------------------------------------------------------------ dQ (bf16)
template <int DHP>
__global__ void __launch_bounds__(256, DHP == 64 ? 4 : 2) attn_bwd_dq_bf16_kernel(const AttnK p) {
  constexpr int KC = DHP / 16, DT = DHP / 32, TILE = 64 * DHP;
  __shared__ __attribute__((aligned(1024))) bf16 Ks[2][TILE];
  __shared__ __attribute__((aligned(1024))) bf16 Vs[2][TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, l32 = lane & 31;
  int qtile, bh;
  attn_block_map(blockIdx.x, (p.Nq + 127) / 128, p.B * p.H, qtile, bh);
  const int b = bh / p.H, h = bh % p.H;
  const int qi = qtile * 128 + wave * 32 + l32;
  const bool qok = qi < p.Nq;
  const bf16* kb = (const bf16*)p.k + (size_t)b * p.Nk * p.ldk + h * p.dh;
  const bf16* vb = (const bf16*)p.v + (size_t)b * p.Nk * p.ldv + h * p.dh;
  const rsrc_t kr = make_rsrc(kb, attn_slice_bytes(p.Nk, p.ldk, p.dh));
  const rsrc_t vr = make_rsrc(vb, attn_slice_bytes(p.Nk, p.ldv, p.dh));
  const bf16* qrow = (const bf16*)p.q + ((size_t)b * p.Nq + qi) * p.ldq + h * p.dh;
  const bf16* dorow = (const bf16*)p.dout + ((size_t)b * p.Nq + qi) * p.lddo + h * p.dh;

  AttnFragOff<DHP> fo;
  fo.init(lane);
  AttnTileCopy<DHP> ck, cv;
  ck.init(wave, lane, p.ldk, p.dh);
  cv.init(wave, lane, p.ldv, p.dh);
  ck.issue(kr, 0, p.ldk, Ks[0], wave);
  cv.issue(vr, 0, p.ldv, Vs[0], wave);

  bf16x8 qf[KC], dof[KC];
#pragma unroll
  for (int c = 0; c < KC; ++c) {
    const bool ok = qok && 16 * c + 8 * g < p.dh;
    qf[c] = ld8(qrow + 16 * c + 8 * g, ok);
    dof[c] = ld8(dorow + 16 * c + 8 * g, ok);
  }
  const size_t sidx = ((size_t)b * p.H + h) * p.Nq + qi;
  const float lse2 = qok ? p.lse[sidx] * LOG2E : INFINITY;
  // delta = rowsum(dO * O), computed here from the dO fragments the lane already holds (its half of
  // the head dimension; lane ^ 32 holds the other half) and stored for the dK/dV kernel, which runs
  // after this one on the same stream
  float dlt = 0.f;
  {
    const bf16* orow = (const bf16*)p.o + ((size_t)b * p.Nq + qi) * p.ldo + h * p.dh;
#pragma unroll
    for (int c = 0; c < KC; ++c) {
      const bf16x8 of = ld8(orow + 16 * c + 8 * g, qok && 16 * c + 8 * g < p.dh);
#pragma unroll
      for (int u = 0; u < 8; ++u) dlt = fmaf((float)of[u], (float)dof[c][u], dlt);
    }
    dlt += __shfl_xor(dlt, 32, 64);
    if (qok && g == 0) p.delta[sidx] = dlt;
  }

  f32x16 acc[DT];
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  const int nkt = (p.Nk + 63) / 64;
  wait_vmcnt<0>();
  __syncthreads();
  for (int kt = 0; kt < nkt; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nkt) {      // every wave left stage buf ^ 1 at the barrier that ended the previous iteration
      ck.issue(kr, (kt + 1) * 64, p.ldk, Ks[buf ^ 1], wave);
      cv.issue(vr, (kt + 1) * 64, p.ldv, Vs[buf ^ 1], wave);
    }
    // Keys past Nk need no masking here: their K and V rows are zero in LDS, so dP = 0 and the
    // finite dS they get multiplies a zero K row in the dQ product.
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int c = 0; c < KC; ++c) {
        s = mfma32(fo.row_frag(Ks[buf], t, c), qf[c], s);
        dp = mfma32(fo.row_frag(Vs[buf], t, c), dof[c], dp);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pr = __builtin_amdgcn_exp2f(fmaf(s[r], p.scale_log2, -lse2));
        s[r] = pr * (dp[r] - dlt);
      }
#pragma unroll
      for (int cc = 0; cc < 2; ++cc) {
        const bf16x8 dsf = pack8(s, 8 * cc);
#pragma unroll
        for (int i = 0; i < DT; ++i) acc[i] = mfma32(fo.tr_frag(Ks[buf], 32 * t + 16 * cc, i), dsf, acc[i]);
      }
    }
    wait_vmcnt<0>();
    __syncthreads();
  }
  if (qok) {
    bf16* ob = (bf16*)p.dq + ((size_t)b * p.Nq + qi) * p.lddq + h * p.dh;
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int col = 32 * i + 8 * r4 + 4 * g;
        if (col < p.dh) {
          bf16x4 o;
#pragma unroll
          for (int u = 0; u < 4; ++u) o[u] = (bf16)(acc[i][4 * r4 + u] * p.scale);
          *reinterpret_cast<bf16x4*>(ob + col) = o;
        }
      }
  }
}

// ------------------------------------------------------------------ dK, dV (bf16)
// grid.x = ceil(Nk / 128) * qsplits; each wave owns 32 keys and walks its share of the query tiles.
// MINW: waves per SIMD the register allocation aims at (3 costs d_head 64 a few spilled address registers).
template <int DHP, int MINW>
__global__ void __launch_bounds__(256, MINW) attn_bwd_dkv_bf16_kernel(const AttnK p) {
  constexpr int KC = DHP / 16, DT = DHP / 32, TILE = 64 * DHP;
  __shared__ __attribute__((aligned(1024))) bf16 Qs[2][TILE];
  __shared__ __attribute__((aligned(1024))) bf16 Ds[2][TILE];
  __shared__ __attribute__((aligned(16))) float lse_s[2][64];
  __shared__ __attribute__((aligned(16))) float dlt_s[2][64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, l32 = lane & 31;
  int ktile, bh;
  const int qs = blockIdx.x % p.qsplits;
  attn_block_map(blockIdx.x / p.qsplits, (p.Nk + 127) / 128, p.B * p.H, ktile, bh);
  const int b = bh / p.H, h = bh % p.H;
  const int ki = ktile * 128 + wave * 32 + l32;
  const bool kok = ki < p.Nk;
  const bf16* qb = (const bf16*)p.q + (size_t)b * p.Nq * p.ldq + h * p.dh;
  const bf16* dob = (const bf16*)p.dout + (size_t)b * p.Nq * p.lddo + h * p.dh;
  const rsrc_t qr = make_rsrc(qb, attn_slice_bytes(p.Nq, p.ldq, p.dh));
  const rsrc_t dr = make_rsrc(dob, attn_slice_bytes(p.Nq, p.lddo, p.dh));
  const bf16* krow = (const bf16*)p.k + ((size_t)b * p.Nk + ki) * p.ldk + h * p.dh;
  const bf16* vrow = (const bf16*)p.v + ((size_t)b * p.Nk + ki) * p.ldv + h * p.dh;
  const float* lse_b = p.lse + ((size_t)b * p.H + h) * p.Nq;
  const float* dlt_b = p.delta + ((size_t)b * p.H + h) * p.Nq;

  // this workgroup's share of the 64-query tiles
  const int nqt_all = (p.Nq + 63) / 64, tps = (nqt_all + p.qsplits - 1) / p.qsplits;
  const int qt0 = qs * tps, nqt = min(nqt_all, qt0 + tps);
  AttnFragOff<DHP> fo;
  fo.init(lane);
  AttnTileCopy<DHP> cq, cd;
  cq.init(wave, lane, p.ldq, p.dh);
  cd.init(wave, lane, p.lddo, p.dh);
  if (qt0 < nqt) {
    cq.issue(qr, qt0 * 64, p.ldq, Qs[0], wave);
    cd.issue(dr, qt0 * 64, p.lddo, Ds[0], wave);
  }
  float r_lse = 0.f, r_dlt = 0.f;
  auto load_stats = [&](int qt) {
    if (tid < 64) {
      const int qi = qt * 64 + tid;
      r_lse = qi < p.Nq ? lse_b[qi] * LOG2E : INFINITY;
      r_dlt = qi < p.Nq ? dlt_b[qi] : 0.f;
    }
  };
  auto store_stats = [&](int buf) {
    if (tid < 64) { lse_s[buf][tid] = r_lse; dlt_s[buf][tid] = r_dlt; }
  };
  load_stats(qt0);

  bf16x8 kf[KC], vf[KC];
#pragma unroll
  for (int c = 0; c < KC; ++c) {
    const bool ok = kok && 16 * c + 8 * g < p.dh;
    kf[c] = ld8(krow + 16 * c + 8 * g, ok);
    vf[c] = ld8(vrow + 16 * c + 8 * g, ok);
  }
  f32x16 dkacc[DT], dvacc[DT];
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dkacc[i][r] = 0.f; dvacc[i][r] = 0.f; }

  store_stats(0);
  wait_vmcnt<0>();
  __syncthreads();

  for (int qt = qt0; qt < nqt; ++qt) {
    const int buf = (qt - qt0) & 1;
    const bool more = qt + 1 < nqt;
    if (more) {
      cq.issue(qr, (qt + 1) * 64, p.ldq, Qs[buf ^ 1], wave);
      cd.issue(dr, (qt + 1) * 64, p.lddo, Ds[buf ^ 1], wave);
      load_stats(qt + 1);
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int c = 0; c < KC; ++c) {
        s = mfma32(fo.row_frag(Qs[buf], t, c), kf[c], s);
        dp = mfma32(fo.row_frag(Ds[buf], t, c), vf[c], dp);
      }
      f32x16 ds;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const f32x4 l4 = *reinterpret_cast<const f32x4*>(&lse_s[buf][32 * t + 8 * r4 + 4 * g]);
        const f32x4 d4 = *reinterpret_cast<const f32x4*>(&dlt_s[buf][32 * t + 8 * r4 + 4 * g]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int r = 4 * r4 + u;
          // a lane whose key is past Nk computes garbage that stays in its own accumulator columns,
          // which are never stored; queries past Nq have lse = +inf, hence pr = 0
          const float pr = __builtin_amdgcn_exp2f(fmaf(s[r], p.scale_log2, -l4[u]));
          s[r] = pr;
          ds[r] = pr * (dp[r] - d4[u]);
        }
      }
#pragma unroll
      for (int cc = 0; cc < 2; ++cc) {
        const bf16x8 pf = pack8(s, 8 * cc);
        const bf16x8 dsf = pack8(ds, 8 * cc);
#pragma unroll
        for (int i = 0; i < DT; ++i) {
          dvacc[i] = mfma32(fo.tr_frag(Ds[buf], 32 * t + 16 * cc, i), pf, dvacc[i]);
          dkacc[i] = mfma32(fo.tr_frag(Qs[buf], 32 * t + 16 * cc, i), dsf, dkacc[i]);
        }
      }
    }
    if (more) store_stats(buf ^ 1);
    wait_vmcnt<0>();
    __syncthreads();
  }
  if (kok && p.qsplits > 1) {
    // fp32 partial sums of this query range; reduced in a fixed order by attn_dkv_reduce_kernel
    const size_t hd = (size_t)p.H * p.dh, rows = (size_t)p.B * p.Nk;
    float* pk = p.dkv_partial + ((size_t)qs * rows + (size_t)b * p.Nk + ki) * hd + h * p.dh;
    float* pv = pk + (size_t)p.qsplits * rows * hd;
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int col = 32 * i + 8 * r4 + 4 * g;
        if (col < p.dh) {
          f32x4 ok_, ov;
#pragma unroll
          for (int u = 0; u < 4; ++u) { ok_[u] = dkacc[i][4 * r4 + u] * p.scale; ov[u] = dvacc[i][4 * r4 + u]; }
          *reinterpret_cast<f32x4*>(pk + col) = ok_;
          *reinterpret_cast<f32x4*>(pv + col) = ov;
        }
      }
  } else if (kok) {
    bf16* dkb = (bf16*)p.dk + ((size_t)b * p.Nk + ki) * p.lddk + h * p.dh;
    bf16* dvb = (bf16*)p.dv + ((size_t)b * p.Nk + ki) * p.lddv + h * p.dh;
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int col = 32 * i + 8 * r4 + 4 * g;
        if (col < p.dh) {
          bf16x4 ok_, ov;
#pragma unroll
          for (int u = 0; u < 4; ++u) { ok_[u] = (bf16)(dkacc[i][4 * r4 + u] * p.scale); ov[u] = (bf16)dvacc[i][4 * r4 + u]; }
          *reinterpret_cast<bf16x4*>(dkb + col) = ok_;
          *reinterpret_cast<bf16x4*>(dvb + col) = ov;
        }
      }
  }
}

// dk[row, col] = sum_qs partial_k[qs][row][col] (ascending qs), same for dv; 4 columns per thread.
__global__ void attn_dkv_reduce_kernel(const float* __restrict__ partial, int qsplits, size_t rows, int hd, bf16* __restrict__ dk, int lddk,
                                       bf16* __restrict__ dv, int lddv) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const int per_row = hd / 4;
  if (i >= rows * per_row) return;
  const size_t row = i / per_row; const int col = (int)(i % per_row) * 4;
  f32x4 sk = {0.f, 0.f, 0.f, 0.f}, sv = sk;
  const size_t plane = rows * hd;
  for (int q = 0; q < qsplits; ++q) {
    sk += *reinterpret_cast<const f32x4*>(partial + (size_t)q * plane + row * hd + col);
    sv += *reinterpret_cast<const f32x4*>(partial + ((size_t)qsplits + q) * plane + row * hd + col);
  }
  bf16x4 ok_, ov;
#pragma unroll
  for (int u = 0; u < 4; ++u) { ok_[u] = (bf16)sk[u]; ov[u] = (bf16)sv[u]; }
  *reinterpret_cast<bf16x4*>(dk + row * lddk + col) = ok_;
  *reinterpret_cast<bf16x4*>(dv + row * lddv + col) = ov;
}

// ------------------------------------------------------------------ fp32 path (one wave per row)
constexpr int F32_MAX_DH = 256;

__global__ void __launch_bounds__(64) attn_fwd_f32_kernel(const AttnK p, int causal) {
  extern __shared__ float sc[];        // [Nk]
  __shared__ float qs[F32_MAX_DH];
  const int lane = threadIdx.x, i = blockIdx.x, b = blockIdx.y / p.H, h = blockIdx.y % p.H;
  const float* q = (const float*)p.q + ((size_t)b * p.Nq + i) * p.ldq + h * p.dh;
  const float* kb = (const float*)p.k + (size_t)b * p.Nk * p.ldk + h * p.dh;
  const float* vb = (const float*)p.v + (size_t)b * p.Nk * p.ldv + h * p.dh;
  for (int t = lane; t < p.dh; t += 64) qs[t] = q[t];
  __syncthreads();
  float mx = -INFINITY;
  for (int j = lane; j < p.Nk; j += 64) {
    float s = 0.f;
    for (int t = 0; t < p.dh; ++t) s = fmaf(qs[t], kb[(size_t)j * p.ldk + t], s);
    s *= p.scale;
    if (causal && j > i) s = -INFINITY;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j < p.Nk; j += 64) {
    const float e = expf(sc[j] - mx);
    sc[j] = e;
    sum += e;
  }
  sum = wave_sum(sum);
  __syncthreads();
  float* o = (float*)p.o + ((size_t)b * p.Nq + i) * p.ldo + h * p.dh;
  for (int t = lane; t < p.dh; t += 64) {
    float a = 0.f;
    for (int j = 0; j < p.Nk; ++j) a = fmaf(sc[j], vb[(size_t)j * p.ldv + t], a);
    o[t] = a / sum;
  }
  if (p.lse && lane == 0) p.lse[((size_t)b * p.H + h) * p.Nq + i] = mx + logf(sum);
}

__global__ void __launch_bounds__(64) attn_bwd_dq_f32_kernel(const AttnK p) {
  extern __shared__ float sc[];        // [Nk]
  __shared__ float qs[F32_MAX_DH];
  __shared__ float dos[F32_MAX_DH];
  const int lane = threadIdx.x, i = blockIdx.x, b = blockIdx.y / p.H, h = blockIdx.y % p.H;
  const float* q = (const float*)p.q + ((size_t)b * p.Nq + i) * p.ldq + h * p.dh;
  const float* dor = (const float*)p.dout + ((size_t)b * p.Nq + i) * p.lddo + h * p.dh;
  const float* kb = (const float*)p.k + (size_t)b * p.Nk * p.ldk + h * p.dh;
  const float* vb = (const float*)p.v + (size_t)b * p.Nk * p.ldv + h * p.dh;
  for (int t = lane; t < p.dh; t += 64) { qs[t] = q[t]; dos[t] = dor[t]; }
  __syncthreads();
  const size_t sidx = ((size_t)b * p.H + h) * p.Nq + i;
  const float lse = p.lse[sidx], dlt = p.delta[sidx];
  for (int j = lane; j < p.Nk; j += 64) {
    float s = 0.f, dp = 0.f;
    for (int t = 0; t < p.dh; ++t) {
      s = fmaf(qs[t], kb[(size_t)j * p.ldk + t], s);
      dp = fmaf(dos[t], vb[(size_t)j * p.ldv + t], dp);
    }
    sc[j] = expf(s * p.scale - lse) * (dp - dlt);
  }
  __syncthreads();
  float* dq = (float*)p.dq + ((size_t)b * p.Nq + i) * p.lddq + h * p.dh;
  for (int t = lane; t < p.dh; t += 64) {
    float a = 0.f;
    for (int j = 0; j < p.Nk; ++j) a = fmaf(sc[j], kb[(size_t)j * p.ldk + t], a);
    dq[t] = a * p.scale;
  }
}

__global__ void __launch_bounds__(64) attn_bwd_dkv_f32_kernel(const AttnK p) {
  extern __shared__ float sc[];        // [2][Nq]: p, ds
  __shared__ float ks[F32_MAX_DH];
  __shared__ float vs[F32_MAX_DH];
  const int lane = threadIdx.x, j = blockIdx.x, b = blockIdx.y / p.H, h = blockIdx.y % p.H;
  const float* kr = (const float*)p.k + ((size_t)b * p.Nk + j) * p.ldk + h * p.dh;
  const float* vr = (const float*)p.v + ((size_t)b * p.Nk + j) * p.ldv + h * p.dh;
  const float* qb = (const float*)p.q + (size_t)b * p.Nq * p.ldq + h * p.dh;
  const float* dob = (const float*)p.dout + (size_t)b * p.Nq * p.lddo + h * p.dh;
  const float* lse_b = p.lse + ((size_t)b * p.H + h) * p.Nq;
  const float* dlt_b = p.delta + ((size_t)b * p.H + h) * p.Nq;
  for (int t = lane; t < p.dh; t += 64) { ks[t] = kr[t]; vs[t] = vr[t]; }
  __syncthreads();
  float* pp = sc; float* dsp = sc + p.Nq;
  for (int i = lane; i < p.Nq; i += 64) {
    float s = 0.f, dp = 0.f;
    for (int t = 0; t < p.dh; ++t) {
      s = fmaf(qb[(size_t)i * p.ldq + t], ks[t], s);
      dp = fmaf(dob[(size_t)i * p.lddo + t], vs[t], dp);
    }
    const float pr = expf(s * p.scale - lse_b[i]);
    pp[i] = pr;
    dsp[i] = pr * (dp - dlt_b[i]);
  }
  __syncthreads();
  float* dk = (float*)p.dk + ((size_t)b * p.Nk + j) * p.lddk + h * p.dh;
  float* dv = (float*)p.dv + ((size_t)b * p.Nk + j) * p.lddv + h * p.dh;
  for (int t = lane; t < p.dh; t += 64) {
    float a = 0.f, c = 0.f;
    for (int i = 0; i < p.Nq; ++i) {
      a = fmaf(dsp[i], qb[(size_t)i * p.ldq + t], a);
      c = fmaf(pp[i], dob[(size_t)i * p.lddo + t], c);
    }
    dk[t] = a * p.scale;
    dv[t] = c;
  }
}

// ------------------------------------------------------------------ host side
static AttnK make_k(const AttnArgs& a) {
  AttnK k;
  k.B = a.B; k.H = a.H; k.Nq = a.Nq; k.Nk = a.Nk; k.dh = a.d_head;
  k.scale = a.scale; k.scale_log2 = a.scale * LOG2E;
  k.q = a.q; k.ldq = a.ldq; k.k = a.k; k.ldk = a.ldk; k.v = a.v; k.ldv = a.ldv; k.o = a.o; k.ldo = a.ldo; k.lse = a.lse;
  k.dout = a.dout; k.lddo = a.lddo; k.delta = a.delta; k.dq = a.dq; k.lddq = a.lddq; k.dk = a.dk; k.lddk = a.lddk;
  k.dv = a.dv; k.lddv = a.lddv;
  k.qsplits = 1; k.dkv_partial = nullptr;
  return k;
}

static int check_attn(const AttnArgs& a, bool bwd) {
  if (a.B <= 0 || a.H <= 0 || a.Nq <= 0 || a.Nk <= 0 || a.d_head <= 0) return set_error(DP_EINVAL, "attention: non-positive size");
  if (!a.q || !a.k || !a.v || !a.o) return set_error(DP_EINVAL, "attention: null operand");
  if ((size_t)a.B * a.H > 65535) return set_error(DP_EUNSUPPORTED, "attention: batch * heads exceeds 65535");
  const int span = a.H * a.d_head;
  if (a.ldq < span || a.ldk < span || a.ldv < span || a.ldo < span) return set_error(DP_EINVAL, "attention: leading dim smaller than heads * d_head");
  if (bwd) {
    if (!a.dout || !a.lse || !a.delta || !a.dq || !a.dk || !a.dv) return set_error(DP_EINVAL, "attention backward: null operand");
    if (a.lddo < span || a.lddq < span || a.lddk < span || a.lddv < span) return set_error(DP_EINVAL, "attention backward: leading dim too small");
    if (a.causal) return set_error(DP_EUNSUPPORTED, "attention backward: causal mask not supported (the causal encoder is frozen)");
  }
  if (a.dtype == BF16) {
    if (a.d_head % 8 || a.d_head > 96) return set_error(DP_EUNSUPPORTED, "attention(bf16): d_head must be a multiple of 8, at most 96");
    const int lds[] = {a.ldq, a.ldk, a.ldv, a.ldo, bwd ? a.lddo : 8, bwd ? a.lddq : 8, bwd ? a.lddk : 8, bwd ? a.lddv : 8};
    for (int x : lds) if (x % 8) return set_error(DP_EUNSUPPORTED, "attention(bf16): leading dims must be multiples of 8");
    const void* ps[] = {a.q, a.k, a.v, a.o, bwd ? a.dout : a.q, bwd ? a.dq : a.q, bwd ? a.dk : a.q, bwd ? a.dv : a.q};
    for (const void* x : ps) if ((uintptr_t)x % 16) return set_error(DP_EALIGN, "attention(bf16): operands must be 16-byte aligned");
    // the tile copies address one (batch, head) slice with 32-bit byte offsets and keep bit 31 for "no data"
    const size_t maxld = (size_t)std::max(std::max(a.ldq, a.ldk), std::max(a.ldv, bwd ? a.lddo : 8));
    if ((size_t)std::max(a.Nq, a.Nk) * maxld * 2 >= (1ull << 31)) return set_error(DP_EUNSUPPORTED, "attention(bf16): one batch element's q / k / v rows must span less than 2 GiB");
  } else {
    if (a.d_head > F32_MAX_DH) return set_error(DP_EUNSUPPORTED, "attention(fp32): d_head > 256");
    if ((size_t)a.Nk * 4 > 60000 || (bwd && (size_t)a.Nq * 8 > 60000)) return set_error(DP_EUNSUPPORTED, "attention(fp32): sequence too long for the fp32 path");
  }
  return DP_OK;
}

size_t attn_dkv_ws_bytes(int B, int H, int Nk, int d_head) { return 2 * (size_t)16 * B * Nk * H * d_head * sizeof(float); }

int launch_attn_fwd(const AttnArgs& a, hipStream_t s) {
  if (int e = check_attn(a, false)) return e;
  const AttnK k = make_k(a);
  const double fl = 4.0 * a.B * a.H * (double)a.Nq * a.Nk * a.d_head;
  const double by = dtype_size(a.dtype) * (double)a.B * a.H * a.d_head * (2.0 * a.Nq + 2.0 * a.Nk);
  KScope ks(a.dtype == BF16 ? KK_ATTN_FWD : KK_ATTN_F32, fl, by, s, a.Nq, a.Nk, a.d_head);
  if (a.dtype == BF16) {
    dim3 grid(((a.Nq + 127) / 128) * a.B * a.H);
    if (a.d_head <= 64) {
      if (a.causal) hipLaunchKernelGGL((attn_fwd_bf16_kernel<64, true>), grid, dim3(256), 0, s, k);
      else hipLaunchKernelGGL((attn_fwd_bf16_kernel<64, false>), grid, dim3(256), 0, s, k);
    } else {
      if (a.causal) hipLaunchKernelGGL((attn_fwd_bf16_kernel<96, true>), grid, dim3(256), 0, s, k);
      else hipLaunchKernelGGL((attn_fwd_bf16_kernel<96, false>), grid, dim3(256), 0, s, k);
    }
  } else {
    hipLaunchKernelGGL(attn_fwd_f32_kernel, dim3(a.Nq, a.B * a.H), dim3(64), (size_t)a.Nk * sizeof(float), s, k, a.causal);
  }
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "attention forward launch failed");
}

int launch_attn_bwd(const AttnArgs& a, hipStream_t s) {
  if (int e = check_attn(a, true)) return e;
  const AttnK k = make_k(a);
  const size_t pairs = (size_t)a.B * a.Nq * a.H;
  const dim3 dgrid((pairs * 8 + 255) / 256);
  if (a.dtype == BF16) {
    dim3 gq(((a.Nq + 127) / 128) * a.B * a.H), gk(((a.Nk + 127) / 128) * a.B * a.H);
    // algorithmic backward work = 2x forward, split evenly between the two kernels for accounting
    const double fl = 4.0 * a.B * a.H * (double)a.Nq * a.Nk * a.d_head;
    const double by = 2.0 * (double)a.B * a.H * a.d_head * (3.0 * a.Nq + 2.0 * a.Nk);
    {
      KScope ks(KK_ATTN_BWD_DQ, fl, by, s, a.Nq, a.Nk, a.d_head);
      if (a.d_head <= 64) hipLaunchKernelGGL(attn_bwd_dq_bf16_kernel<64>, gq, dim3(256), 0, s, k);
      else hipLaunchKernelGGL(attn_bwd_dq_bf16_kernel<96>, gq, dim3(256), 0, s, k);
    }
    {
      // few key tiles (cross-attention to 77 keys): split the query range over more workgroups
      AttnK k2 = k;
      const long base_blocks = (long)((a.Nk + 127) / 128) * a.B * a.H;
      const int nqt = (a.Nq + 63) / 64;
      int qsplit = 1;
      if (base_blocks < 256) qsplit = (int)std::min<long>(std::min<long>(16, nqt / 2 > 0 ? nqt / 2 : 1), (512 + base_blocks - 1) / base_blocks);
      const size_t need = 2 * (size_t)qsplit * a.B * a.Nk * a.H * a.d_head * sizeof(float);
      if (qsplit > 1 && (!a.dkv_ws || a.dkv_ws_bytes < need || ((uintptr_t)a.dkv_ws % 16))) qsplit = 1;
      k2.qsplits = qsplit; k2.dkv_partial = a.dkv_ws;
      dim3 gk2(gk.x * qsplit);
      {
        KScope ks(KK_ATTN_BWD_DKV, fl, by, s, a.Nq, a.Nk, a.d_head);
        // Two workgroups per CU hold 512 at a time; a larger grid gains more from a third resident workgroup
        // than the tighter register budget costs (1024 tokens, 640 workgroups: 120 -> 110 us for the whole
        // backward), a smaller one only pays for it (77 keys: 43 -> 46 us)
        if (a.d_head <= 64 && qsplit == 1 && gk.x > 2 * 256) hipLaunchKernelGGL((attn_bwd_dkv_bf16_kernel<64, 3>), gk2, dim3(256), 0, s, k2);
        else if (a.d_head <= 64) hipLaunchKernelGGL((attn_bwd_dkv_bf16_kernel<64, 2>), gk2, dim3(256), 0, s, k2);
        else hipLaunchKernelGGL((attn_bwd_dkv_bf16_kernel<96, 2>), gk2, dim3(256), 0, s, k2);
      }
      if (qsplit > 1) {
        const size_t rows = (size_t)a.B * a.Nk; const int hd = a.H * a.d_head;
        KScope ks(KK_REDUCE, 0.0, (double)need + 4.0 * rows * hd, s, (int)rows, hd, qsplit);
        hipLaunchKernelGGL(attn_dkv_reduce_kernel, dim3((rows * (hd / 4) + 255) / 256), dim3(256), 0, s, a.dkv_ws, qsplit, rows, hd,
                           (bf16*)a.dk, a.lddk, (bf16*)a.dv, a.lddv);
      }
    }
  } else {
    hipLaunchKernelGGL(attn_delta_kernel<float>, dgrid, dim3(256), 0, s, (const float*)a.o, a.ldo, (const float*)a.dout, a.lddo, a.delta, a.B, a.H, a.Nq, a.d_head);
    hipLaunchKernelGGL(attn_bwd_dq_f32_kernel, dim3(a.Nq, a.B * a.H), dim3(64), (size_t)a.Nk * sizeof(float), s, k);
    hipLaunchKernelGGL(attn_bwd_dkv_f32_kernel, dim3(a.Nk, a.B * a.H), dim3(64), (size_t)2 * a.Nq * sizeof(float), s, k);
  }
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "attention backward launch failed");
}

}  // namespace dp
