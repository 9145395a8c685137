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
// For d_head = 64 the streamed tiles are copied global -> LDS directly (the *_dtl_kernel variants);
// other head widths stage them through registers.
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

// Copies a [64 x DHP] tile (rows row0.., zero-filled outside [0,nrows) x [0,dh)) into registers / LDS.
template <int DHP, int NT>
struct TileLoader {
  static constexpr int CHUNKS = 64 * DHP / 8;
  static constexpr int PER = (CHUNKS + NT - 1) / NT;
  bf16x8 r[PER];
  __device__ __forceinline__ void load(const bf16* base, int ld, int row0, int nrows, int dh, int tid) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int id = tid + i * NT;
      const int row = id / (DHP / 8), c = (id % (DHP / 8)) * 8;
      const bool ok = (CHUNKS % NT == 0 || id < CHUNKS) && row0 + row < nrows && c < dh;
      r[i] = ld8(base + (size_t)(row0 + row) * ld + c, ok);
    }
  }
  __device__ __forceinline__ void store(bf16* tile, int tld, int tid) const {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int id = tid + i * NT;
      const int row = id / (DHP / 8), c = (id % (DHP / 8)) * 8;
      if (CHUNKS % NT == 0 || id < CHUNKS) *reinterpret_cast<bf16x8*>(tile + row * tld + c) = r[i];
    }
  }
};

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
// A wave owns QT tiles of 32 queries; every K / V fragment fetched from LDS is used for all of
// them (QT = 2 halves the LDS traffic per FLOP, and the MFMAs of one query tile can overlap the
// softmax arithmetic of the other).  A workgroup covers 128 * QT queries.
template <int DHP, bool CAUSAL, int QT>
__global__ void __launch_bounds__(256, (QT == 1 && DHP == 64) ? 3 : 2) attn_fwd_bf16_kernel(const AttnK p) {
  constexpr int KC = DHP / 16, DT = DHP / 32, BQ = 128 * QT;
  constexpr int K_LD = DHP + 8, V_LD = DHP + 16;
  __shared__ __attribute__((aligned(16))) bf16 Ks[2][64 * K_LD];
  __shared__ __attribute__((aligned(16))) bf16 Vs[2][64 * V_LD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, l32 = lane & 31;
  int qtile, bh;
  attn_block_map(blockIdx.x, (p.Nq + BQ - 1) / BQ, p.B * p.H, qtile, bh);
  const int b = bh / p.H, h = bh % p.H;
  const int q0 = qtile * BQ + wave * 32 * QT;          // first query of this wave
  const bf16* qb = (const bf16*)p.q + (size_t)b * p.Nq * p.ldq + h * p.dh;
  const bf16* kb = (const bf16*)p.k + (size_t)b * p.Nk * p.ldk + h * p.dh;
  const bf16* vb = (const bf16*)p.v + (size_t)b * p.Nk * p.ldv + h * p.dh;

  bf16x8 qf[QT][KC];
#pragma unroll
  for (int j = 0; j < QT; ++j)
#pragma unroll
    for (int c = 0; c < KC; ++c) {
      const int qi = q0 + 32 * j + l32;
      qf[j][c] = ld8(qb + (size_t)qi * p.ldq + 16 * c + 8 * g, qi < p.Nq && 16 * c + 8 * g < p.dh);
    }

  f32x16 oacc[QT][DT];
  float m[QT], lsum[QT];
#pragma unroll
  for (int j = 0; j < QT; ++j) {
    m[j] = -INFINITY; lsum[j] = 0.f;
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[j][i][r] = 0.f;
  }

  int nkt = (p.Nk + 63) / 64;
  if (CAUSAL) nkt = min(nkt, (min(p.Nq, qtile * BQ + BQ) + 63) / 64);

  TileLoader<DHP, 256> lk, lv;
  lk.load(kb, p.ldk, 0, p.Nk, p.dh, tid);
  lv.load(vb, p.ldv, 0, p.Nk, p.dh, tid);
  lk.store(Ks[0], K_LD, tid);
  lv.store(Vs[0], V_LD, tid);
  __syncthreads();

  for (int kt = 0; kt < nkt; ++kt) {
    const int buf = kt & 1;
    const bool more = kt + 1 < nkt;
    if (more) {
      lk.load(kb, p.ldk, (kt + 1) * 64, p.Nk, p.dh, tid);
      lv.load(vb, p.ldv, (kt + 1) * 64, p.Nk, p.dh, tid);
    }
    // S^T = K Q^T for the wave's QT query tiles: K fragments are fetched once
    f32x16 s[QT][2];
#pragma unroll
    for (int j = 0; j < QT; ++j)
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[j][t][r] = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int c = 0; c < KC; ++c) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Ks[buf][(32 * t + l32) * K_LD + 16 * c + 8 * g]);
#pragma unroll
        for (int j = 0; j < QT; ++j) s[j][t] = mfma32(a, qf[j][c], s[j][t]);
      }
    // online softmax, one query column per lane (shared with lane ^ 32)
    const bool key_edge = kt * 64 + 64 > p.Nk;
#pragma unroll
    for (int j = 0; j < QT; ++j) {
      const int qi = q0 + 32 * j + l32;
      const bool edge = key_edge || (CAUSAL && kt * 64 + 63 > q0 + 32 * j);
      // masking only in tiles that cross the end of the keys or the causal diagonal (one wave-uniform
      // branch around a block of selects; a test per element would be compiled into a branch per element)
      if (edge) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kt * 64 + 32 * t + acc_row(r, g);
            const bool dead = key >= p.Nk || (CAUSAL && key > qi);
            s[j][t][r] = dead ? -INFINITY : s[j][t][r];
          }
      }
      // running maximum over raw scores (the scale is positive, so it commutes with max)
      float mx = -INFINITY;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[j][t][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      mx = fmaxf(m[j], mx * p.scale_log2);                 // m[j] is kept in the scaled (log2) domain
      // The reference point only has to bound the exponents, not equal the maximum: it is moved (and the
      // accumulators rescaled) when some query of the wave has outgrown it by 2^8; until then the
      // probabilities of this tile are taken relative to the old one (at most 256, exact in the final
      // O = acc / sum and LSE = ref + log sum).  Wave-uniform, so the rescale is skipped for most tiles.
      const bool bump = __any(mx > m[j] + 8.0f);
      mx = bump ? mx : m[j];
      const float mref = (mx == -INFINITY) ? 0.f : mx;
      float rs = 0.f;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float e = __builtin_amdgcn_exp2f(fmaf(s[j][t][r], p.scale_log2, -mref));
          s[j][t][r] = e;
          rs += e;
        }
      rs += __shfl_xor(rs, 32, 64);
      if (bump) {
        const float alpha = __builtin_amdgcn_exp2f(m[j] - mref);
        lsum[j] *= alpha;
#pragma unroll
        for (int i = 0; i < DT; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[j][i][r] *= alpha;
      }
      lsum[j] += rs;
      m[j] = mx;
    }
    // O^T += V^T P^T: V fragments are fetched once for all query tiles
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int cc = 0; cc < 2; ++cc) {
        bf16x8 pf[QT];
#pragma unroll
        for (int j = 0; j < QT; ++j) pf[j] = pack8(s[j][t], 8 * cc);
#pragma unroll
        for (int i = 0; i < DT; ++i) {
          const bf16x8 a = frag_from_mc_accorder(&Vs[buf][(32 * t + 16 * cc) * V_LD + 32 * i], V_LD, lane);
#pragma unroll
          for (int j = 0; j < QT; ++j) oacc[j][i] = mfma32(a, pf[j], oacc[j][i]);
        }
      }
    if (more) {
      lk.store(Ks[buf ^ 1], K_LD, tid);
      lv.store(Vs[buf ^ 1], V_LD, tid);
    }
    __syncthreads();
  }

#pragma unroll
  for (int j = 0; j < QT; ++j) {
    const int qi = q0 + 32 * j + l32;
    if (qi < p.Nq) {
      const float inv = lsum[j] > 0.f ? 1.0f / lsum[j] : 0.f;
      bf16* ob = (bf16*)p.o + ((size_t)b * p.Nq + qi) * p.ldo + h * p.dh;
#pragma unroll
      for (int i = 0; i < DT; ++i)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int col = 32 * i + 8 * r4 + 4 * g;
          if (col < p.dh) {
            bf16x4 o;
#pragma unroll
            for (int u = 0; u < 4; ++u) o[u] = (bf16)(oacc[j][i][4 * r4 + u] * inv);
            *reinterpret_cast<bf16x4*>(ob + col) = o;
          }
        }
      if (p.lse && g == 0) p.lse[((size_t)b * p.H + h) * p.Nq + qi] = m[j] * LN2 + logf(lsum[j]);
    }
  }
}

// The same forward for d_head = 64 with the K and V tiles copied global -> LDS directly (no register
// staging: 16 fewer registers per lane, no LDS stores in the loop).  A [64 x 64] bf16 tile is 64 rows of
// eight 16-byte chunks with no padding; a wave copies 8 rows per instruction, lane = 8 * row + position,
// and the chunk a position holds is position ^ key(row), so that the fragment reads stay conflict-free:
// K (rows read as MFMA A fragments, lanes vary in the row): key = row & 7;
// V (read by the transposing load, 4 rows x 64 bytes per half-wave): key = 4 * ((row >> 1) & 1).
// Rows past the end of the keys come back as zeros from the buffer descriptor's range check.
__device__ __forceinline__ int attn_kkey(int row) { return row & 7; }
__device__ __forceinline__ int attn_vkey(int row) { return 4 * ((row >> 1) & 1); }

template <bool CAUSAL>
__global__ void __launch_bounds__(256, 4) attn_fwd_dtl_kernel(const AttnK p) {
  constexpr int KC = 4, DT = 2, BQ = 128, TILE = 64 * 64;
  __shared__ __attribute__((aligned(1024))) bf16 Ks[2][TILE];
  __shared__ __attribute__((aligned(1024))) bf16 Vs[2][TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, l32 = lane & 31;
  int qtile, bh;
  attn_block_map(blockIdx.x, (p.Nq + BQ - 1) / BQ, p.B * p.H, qtile, bh);
  const int b = bh / p.H, h = bh % p.H;
  const int q0 = qtile * BQ + wave * 32;
  const bf16* qb = (const bf16*)p.q + (size_t)b * p.Nq * p.ldq + h * 64;
  const bf16* kb = (const bf16*)p.k + (size_t)b * p.Nk * p.ldk + h * 64;
  const bf16* vb = (const bf16*)p.v + (size_t)b * p.Nk * p.ldv + h * 64;
  const rsrc_t kr = make_rsrc(kb, (uint32_t)(((size_t)(p.Nk - 1) * p.ldk + 64) * 2));
  const rsrc_t vr = make_rsrc(vb, (uint32_t)(((size_t)(p.Nk - 1) * p.ldv + 64) * 2));

  bf16x8 qf[KC];
#pragma unroll
  for (int c = 0; c < KC; ++c) {
    const int qi = q0 + l32;
    qf[c] = ld8(qb + (size_t)qi * p.ldq + 16 * c + 8 * g, qi < p.Nq);
  }
  f32x16 oacc[DT];
  float m = -INFINITY, lsum = 0.f;
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;

  int nkt = (p.Nk + 63) / 64;
  if (CAUSAL) nkt = min(nkt, (min(p.Nq, qtile * BQ + BQ) + 63) / 64);

  // this wave's share of a tile: rows 16 * wave .. + 15 of K and of V, two 8-row pieces each
  uint32_t ko[2], vo[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = 16 * wave + 8 * j + (lane >> 3), pc = lane & 7;
    ko[j] = (uint32_t)(row * p.ldk + 8 * (pc ^ attn_kkey(row))) * 2u;
    vo[j] = (uint32_t)(row * p.ldv + 8 * (pc ^ attn_vkey(row))) * 2u;
  }
  auto copy_tile = [&](int kt, int st) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      // the tile's offset goes into the per-lane offset: only that one is range-checked
      async_copy_16B_buf(kr, ko[j] + (uint32_t)kt * 64u * (uint32_t)p.ldk * 2u, 0, &Ks[st][(16 * wave + 8 * j) * 64]);
      async_copy_16B_buf(vr, vo[j] + (uint32_t)kt * 64u * (uint32_t)p.ldv * 2u, 0, &Vs[st][(16 * wave + 8 * j) * 64]);
    }
  };
  copy_tile(0, 0);
  wait_vmcnt<0>();
  __syncthreads();

  for (int kt = 0; kt < nkt; ++kt) {
    const int buf = kt & 1;
    // every wave left stage buf ^ 1 at the barrier that ended the previous iteration
    if (kt + 1 < nkt) copy_tile(kt + 1, buf ^ 1);
    f32x16 s[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[t][r] = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int c = 0; c < KC; ++c) {
        const int row = 32 * t + l32;
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Ks[buf][row * 64 + 8 * ((2 * c + g) ^ attn_kkey(row))]);
        s[t] = mfma32(a, qf[c], s[t]);
      }
    const int qi = q0 + l32;
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
    // online softmax with a lazily moved reference point, as in attn_fwd_bf16_kernel
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[t][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    mx = fmaxf(m, mx * p.scale_log2);
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
    // O^T += V^T P^T; the transposing load takes, per lane, 4 consecutive channels of one key row
    const int vb4 = lane >> 4, vj = lane & 15;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int cc = 0; cc < 2; ++cc) {
        const bf16x8 pf = pack8(s[t], 8 * cc);
#pragma unroll
        for (int i = 0; i < DT; ++i) {
          const int row = 32 * t + 16 * cc + 4 * (vb4 >> 1) + (vj >> 2);       // and row + 8 (same key)
          const int chunk = 4 * i + 2 * (vb4 & 1) + ((vj & 3) >> 1);
          const bf16* a0 = &Vs[buf][row * 64 + 8 * (chunk ^ attn_vkey(row)) + 4 * (vj & 1)];
          const bf16x4 lo = lds_read_tr(a0);
          const bf16x4 hi = lds_read_tr(a0 + 8 * 64);
          oacc[i] = mfma32(__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7), pf, oacc[i]);
        }
      }
    wait_vmcnt<0>();      // this wave's pieces of the next tile have landed
    __syncthreads();      // ... and everybody's; all reads of stage buf are done
  }

  const int qi = q0 + l32;
  if (qi < p.Nq) {
    const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
    bf16* ob = (bf16*)p.o + ((size_t)b * p.Nq + qi) * p.ldo + h * 64;
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 o;
#pragma unroll
        for (int u = 0; u < 4; ++u) o[u] = (bf16)(oacc[i][4 * r4 + u] * inv);
        *reinterpret_cast<bf16x4*>(ob + 32 * i + 8 * r4 + 4 * g) = o;
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
__global__ void __launch_bounds__(256, DHP == 64 ? 3 : 2) attn_bwd_dq_bf16_kernel(const AttnK p) {
  constexpr int KC = DHP / 16, DT = DHP / 32;
  constexpr int LD = DHP + 8;
  __shared__ __attribute__((aligned(16))) bf16 Ks[2][64 * LD];
  __shared__ __attribute__((aligned(16))) bf16 Vs[2][64 * LD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, l32 = lane & 31;
  int qtile, bh;
  attn_block_map(blockIdx.x, (p.Nq + 127) / 128, p.B * p.H, qtile, bh);
  const int b = bh / p.H, h = bh % p.H;
  const int qi = qtile * 128 + wave * 32 + l32;
  const bool qok = qi < p.Nq;
  const bf16* kb = (const bf16*)p.k + (size_t)b * p.Nk * p.ldk + h * p.dh;
  const bf16* vb = (const bf16*)p.v + (size_t)b * p.Nk * p.ldv + h * p.dh;
  const bf16* qrow = (const bf16*)p.q + ((size_t)b * p.Nq + qi) * p.ldq + h * p.dh;
  const bf16* dorow = (const bf16*)p.dout + ((size_t)b * p.Nq + qi) * p.lddo + h * p.dh;

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
  TileLoader<DHP, 256> lk, lv;
  lk.load(kb, p.ldk, 0, p.Nk, p.dh, tid);
  lv.load(vb, p.ldv, 0, p.Nk, p.dh, tid);
  lk.store(Ks[0], LD, tid);
  lv.store(Vs[0], LD, tid);
  __syncthreads();

  for (int kt = 0; kt < nkt; ++kt) {
    const int buf = kt & 1;
    const bool more = kt + 1 < nkt;
    if (more) {
      lk.load(kb, p.ldk, (kt + 1) * 64, p.Nk, p.dh, tid);
      lv.load(vb, p.ldv, (kt + 1) * 64, p.Nk, p.dh, tid);
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
        bf16x8 ka = *reinterpret_cast<const bf16x8*>(&Ks[buf][(32 * t + l32) * LD + 16 * c + 8 * g]);
        bf16x8 va = *reinterpret_cast<const bf16x8*>(&Vs[buf][(32 * t + l32) * LD + 16 * c + 8 * g]);
        s = mfma32(ka, qf[c], s);
        dp = mfma32(va, dof[c], dp);
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
        for (int i = 0; i < DT; ++i) {
          bf16x8 a = frag_from_mc_accorder(&Ks[buf][(32 * t + 16 * cc) * LD + 32 * i], LD, lane);
          acc[i] = mfma32(a, dsf, acc[i]);
        }
      }
    }
    if (more) {
      lk.store(Ks[buf ^ 1], LD, tid);
      lv.store(Vs[buf ^ 1], LD, tid);
    }
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
// grid.x = ceil(Nk / 128); each wave owns 32 keys and walks all query tiles.
template <int DHP>
__global__ void __launch_bounds__(256, DHP == 64 ? 2 : 1) attn_bwd_dkv_bf16_kernel(const AttnK p) {
  constexpr int KC = DHP / 16, DT = DHP / 32;
  constexpr int LD = DHP + 8;
  __shared__ __attribute__((aligned(16))) bf16 Qs[2][64 * LD];
  __shared__ __attribute__((aligned(16))) bf16 Ds[2][64 * LD];
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
  const bf16* krow = (const bf16*)p.k + ((size_t)b * p.Nk + ki) * p.ldk + h * p.dh;
  const bf16* vrow = (const bf16*)p.v + ((size_t)b * p.Nk + ki) * p.ldv + h * p.dh;
  const float* lse_b = p.lse + ((size_t)b * p.H + h) * p.Nq;
  const float* dlt_b = p.delta + ((size_t)b * p.H + h) * p.Nq;

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

  // this workgroup's share of the 64-query tiles
  const int nqt_all = (p.Nq + 63) / 64, tps = (nqt_all + p.qsplits - 1) / p.qsplits;
  const int qt0 = qs * tps, nqt = min(nqt_all, qt0 + tps);
  TileLoader<DHP, 256> lq, ld_;
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
  lq.load(qb, p.ldq, qt0 * 64, p.Nq, p.dh, tid);
  ld_.load(dob, p.lddo, qt0 * 64, p.Nq, p.dh, tid);
  load_stats(qt0);
  lq.store(Qs[0], LD, tid);
  ld_.store(Ds[0], LD, tid);
  store_stats(0);
  __syncthreads();

  for (int qt = qt0; qt < nqt; ++qt) {
    const int buf = (qt - qt0) & 1;
    const bool more = qt + 1 < nqt;
    if (more) {
      lq.load(qb, p.ldq, (qt + 1) * 64, p.Nq, p.dh, tid);
      ld_.load(dob, p.lddo, (qt + 1) * 64, p.Nq, p.dh, tid);
      load_stats(qt + 1);
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int c = 0; c < KC; ++c) {
        bf16x8 qa = *reinterpret_cast<const bf16x8*>(&Qs[buf][(32 * t + l32) * LD + 16 * c + 8 * g]);
        bf16x8 da = *reinterpret_cast<const bf16x8*>(&Ds[buf][(32 * t + l32) * LD + 16 * c + 8 * g]);
        s = mfma32(qa, kf[c], s);
        dp = mfma32(da, vf[c], dp);
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
          bf16x8 da = frag_from_mc_accorder(&Ds[buf][(32 * t + 16 * cc) * LD + 32 * i], LD, lane);
          bf16x8 qa = frag_from_mc_accorder(&Qs[buf][(32 * t + 16 * cc) * LD + 32 * i], LD, lane);
          dvacc[i] = mfma32(da, pf, dvacc[i]);
          dkacc[i] = mfma32(qa, dsf, dkacc[i]);
        }
      }
    }
    if (more) {
      lq.store(Qs[buf ^ 1], LD, tid);
      ld_.store(Ds[buf ^ 1], LD, tid);
      store_stats(buf ^ 1);
    }
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

// ------------------------------------------------------------------ backward for d_head = 64, tiles copied global -> LDS
// Both backward kernels read a streamed tile two ways (by rows as an MFMA A operand, and through the
// transposing load), so one chunk permutation has to keep both conflict-free: position = chunk ^ key,
// key = row bits (0, 2, 1) -- a bijection of row & 7 (8 consecutive rows of a row-fragment read land in
// 8 different positions) whose bit 2 is row bit 1 (the 4 rows of a transposing read fall into 4
// different 64-byte bank groups).
__device__ __forceinline__ int attn_ukey(int row) { return (row & 1) | ((row & 4) >> 1) | ((row & 2) << 1); }

// This wave's share of a [64 x 64] tile copy: rows 16 * wave .. + 15 in two 8-row pieces.
struct AttnTileCopy {
  uint32_t off[2];
  __device__ __forceinline__ void init(int wave, int lane, int ld) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int row = 16 * wave + 8 * j + (lane >> 3);
      off[j] = (uint32_t)(row * ld + 8 * ((lane & 7) ^ attn_ukey(row))) * 2u;
    }
  }
  // rows row0 .. row0 + 63 of the (batch, head) slice behind r; rows past its end read as zeros
  __device__ __forceinline__ void issue(rsrc_t r, int row0, int ld, bf16* stage, int wave) const {
#pragma unroll
    for (int j = 0; j < 2; ++j)
      async_copy_16B_buf(r, off[j] + (uint32_t)row0 * (uint32_t)ld * 2u, 0, stage + (16 * wave + 8 * j) * 64);
  }
};
// Per-lane element offsets of the fragment reads, computed once: a row fragment of rows 32 * t + l32 is at
// row[c] + 32 * 64 * t, a transposed fragment (the slot order of frag_from_mc_accorder) of rows r0 .. r0 + 15
// (r0 a multiple of 16, which leaves the keys alone), columns 32 * i .. + 31, at tr[i] + 64 * r0 and 8 rows below.
struct AttnFragOff {
  int row[4], tr[2];
  __device__ __forceinline__ void init(int lane) {
    const int g = lane >> 5, l32 = lane & 31, b = lane >> 4, j = lane & 15;
#pragma unroll
    for (int c = 0; c < 4; ++c) row[c] = l32 * 64 + 8 * ((2 * c + g) ^ attn_ukey(l32));
    const int r = 4 * (b >> 1) + (j >> 2);
#pragma unroll
    for (int i = 0; i < 2; ++i) tr[i] = r * 64 + 8 * ((4 * i + 2 * (b & 1) + ((j & 3) >> 1)) ^ attn_ukey(r)) + 4 * (j & 1);
  }
};
__device__ __forceinline__ bf16x8 attn_row_frag(const bf16* tile, const AttnFragOff& f, int t, int c) {
  return *reinterpret_cast<const bf16x8*>(tile + f.row[c] + 32 * 64 * t);
}
__device__ __forceinline__ bf16x8 attn_tr_frag(const bf16* tile, const AttnFragOff& f, int r0, int i) {
  const bf16* a0 = tile + f.tr[i] + 64 * r0;
  const bf16x4 lo = lds_read_tr(a0);
  const bf16x4 hi = lds_read_tr(a0 + 8 * 64);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

__global__ void __launch_bounds__(256, 3) attn_bwd_dq_dtl_kernel(const AttnK p) {
  constexpr int KC = 4, DT = 2, TILE = 64 * 64;
  __shared__ __attribute__((aligned(1024))) bf16 Ks[2][TILE];
  __shared__ __attribute__((aligned(1024))) bf16 Vs[2][TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, l32 = lane & 31;
  int qtile, bh;
  attn_block_map(blockIdx.x, (p.Nq + 127) / 128, p.B * p.H, qtile, bh);
  const int b = bh / p.H, h = bh % p.H;
  const int qi = qtile * 128 + wave * 32 + l32;
  const bool qok = qi < p.Nq;
  const bf16* kb = (const bf16*)p.k + (size_t)b * p.Nk * p.ldk + h * 64;
  const bf16* vb = (const bf16*)p.v + (size_t)b * p.Nk * p.ldv + h * 64;
  const rsrc_t kr = make_rsrc(kb, (uint32_t)(((size_t)(p.Nk - 1) * p.ldk + 64) * 2));
  const rsrc_t vr = make_rsrc(vb, (uint32_t)(((size_t)(p.Nk - 1) * p.ldv + 64) * 2));
  const bf16* qrow = (const bf16*)p.q + ((size_t)b * p.Nq + qi) * p.ldq + h * 64;
  const bf16* dorow = (const bf16*)p.dout + ((size_t)b * p.Nq + qi) * p.lddo + h * 64;

  AttnFragOff fo;
  fo.init(lane);
  AttnTileCopy ck, cv;
  ck.init(wave, lane, p.ldk);
  cv.init(wave, lane, p.ldv);
  ck.issue(kr, 0, p.ldk, Ks[0], wave);
  cv.issue(vr, 0, p.ldv, Vs[0], wave);

  bf16x8 qf[KC], dof[KC];
#pragma unroll
  for (int c = 0; c < KC; ++c) {
    qf[c] = ld8(qrow + 16 * c + 8 * g, qok);
    dof[c] = ld8(dorow + 16 * c + 8 * g, qok);
  }
  const size_t sidx = ((size_t)b * p.H + h) * p.Nq + qi;
  const float lse2 = qok ? p.lse[sidx] * LOG2E : INFINITY;
  // delta = rowsum(dO * O) from the dO fragments the lane holds (lane ^ 32 has the other half of the
  // head dimension); stored for the dK/dV kernel, which runs after this one on the same stream
  float dlt = 0.f;
  {
    const bf16* orow = (const bf16*)p.o + ((size_t)b * p.Nq + qi) * p.ldo + h * 64;
#pragma unroll
    for (int c = 0; c < KC; ++c) {
      const bf16x8 of = ld8(orow + 16 * c + 8 * g, qok);
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
    if (kt + 1 < nkt) {      // stage buf ^ 1 was left by every wave at the barrier ending the previous iteration
      ck.issue(kr, (kt + 1) * 64, p.ldk, Ks[buf ^ 1], wave);
      cv.issue(vr, (kt + 1) * 64, p.ldv, Vs[buf ^ 1], wave);
    }
    // keys past Nk need no masking: their K and V rows are zero in LDS, so dP = 0 and the finite dS
    // they get multiplies a zero K row in the dQ product
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int c = 0; c < KC; ++c) {
        s = mfma32(attn_row_frag(Ks[buf], fo, t, c), qf[c], s);
        dp = mfma32(attn_row_frag(Vs[buf], fo, t, c), dof[c], dp);
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
        for (int i = 0; i < DT; ++i) acc[i] = mfma32(attn_tr_frag(Ks[buf], fo, 32 * t + 16 * cc, i), dsf, acc[i]);
      }
    }
    wait_vmcnt<0>();
    __syncthreads();
  }
  if (qok) {
    bf16* ob = (bf16*)p.dq + ((size_t)b * p.Nq + qi) * p.lddq + h * 64;
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 o;
#pragma unroll
        for (int u = 0; u < 4; ++u) o[u] = (bf16)(acc[i][4 * r4 + u] * p.scale);
        *reinterpret_cast<bf16x4*>(ob + 32 * i + 8 * r4 + 4 * g) = o;
      }
  }
}

__global__ void __launch_bounds__(256, 2) attn_bwd_dkv_dtl_kernel(const AttnK p) {
  constexpr int KC = 4, DT = 2, TILE = 64 * 64;
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
  const bf16* qb = (const bf16*)p.q + (size_t)b * p.Nq * p.ldq + h * 64;
  const bf16* dob = (const bf16*)p.dout + (size_t)b * p.Nq * p.lddo + h * 64;
  const rsrc_t qr = make_rsrc(qb, (uint32_t)(((size_t)(p.Nq - 1) * p.ldq + 64) * 2));
  const rsrc_t dr = make_rsrc(dob, (uint32_t)(((size_t)(p.Nq - 1) * p.lddo + 64) * 2));
  const bf16* krow = (const bf16*)p.k + ((size_t)b * p.Nk + ki) * p.ldk + h * 64;
  const bf16* vrow = (const bf16*)p.v + ((size_t)b * p.Nk + ki) * p.ldv + h * 64;
  const float* lse_b = p.lse + ((size_t)b * p.H + h) * p.Nq;
  const float* dlt_b = p.delta + ((size_t)b * p.H + h) * p.Nq;

  // this workgroup's share of the 64-query tiles
  const int nqt_all = (p.Nq + 63) / 64, tps = (nqt_all + p.qsplits - 1) / p.qsplits;
  const int qt0 = qs * tps, nqt = min(nqt_all, qt0 + tps);
  AttnFragOff fo;
  fo.init(lane);
  AttnTileCopy cq, cd;
  cq.init(wave, lane, p.ldq);
  cd.init(wave, lane, p.lddo);
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
    kf[c] = ld8(krow + 16 * c + 8 * g, kok);
    vf[c] = ld8(vrow + 16 * c + 8 * g, kok);
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
        s = mfma32(attn_row_frag(Qs[buf], fo, t, c), kf[c], s);
        dp = mfma32(attn_row_frag(Ds[buf], fo, t, c), vf[c], dp);
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
          dvacc[i] = mfma32(attn_tr_frag(Ds[buf], fo, 32 * t + 16 * cc, i), pf, dvacc[i]);
          dkacc[i] = mfma32(attn_tr_frag(Qs[buf], fo, 32 * t + 16 * cc, i), dsf, dkacc[i]);
        }
      }
    }
    if (more) store_stats(buf ^ 1);
    wait_vmcnt<0>();
    __syncthreads();
  }
  if (kok && p.qsplits > 1) {
    // fp32 partial sums of this query range; reduced in a fixed order by attn_dkv_reduce_kernel
    const size_t hd = (size_t)p.H * 64, rows = (size_t)p.B * p.Nk;
    float* pk = p.dkv_partial + ((size_t)qs * rows + (size_t)b * p.Nk + ki) * hd + h * 64;
    float* pv = pk + (size_t)p.qsplits * rows * hd;
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int col = 32 * i + 8 * r4 + 4 * g;
        f32x4 ok_, ov;
#pragma unroll
        for (int u = 0; u < 4; ++u) { ok_[u] = dkacc[i][4 * r4 + u] * p.scale; ov[u] = dvacc[i][4 * r4 + u]; }
        *reinterpret_cast<f32x4*>(pk + col) = ok_;
        *reinterpret_cast<f32x4*>(pv + col) = ov;
      }
  } else if (kok) {
    bf16* dkb = (bf16*)p.dk + ((size_t)b * p.Nk + ki) * p.lddk + h * 64;
    bf16* dvb = (bf16*)p.dv + ((size_t)b * p.Nk + ki) * p.lddv + h * 64;
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int col = 32 * i + 8 * r4 + 4 * g;
        bf16x4 ok_, ov;
#pragma unroll
        for (int u = 0; u < 4; ++u) { ok_[u] = (bf16)(dkacc[i][4 * r4 + u] * p.scale); ov[u] = (bf16)dvacc[i][4 * r4 + u]; }
        *reinterpret_cast<bf16x4*>(dkb + col) = ok_;
        *reinterpret_cast<bf16x4*>(dvb + col) = ov;
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
    // two query tiles per wave halve the LDS traffic but cost occupancy; measured slower on MI355X
    // (the kernel is bound by the softmax arithmetic, not by LDS), so one tile per wave is used
    const bool qt2 = false;
    dim3 grid(((a.Nq + (qt2 ? 255 : 127)) / (qt2 ? 256 : 128)) * a.B * a.H);
    // d_head = 64 (every stage and encoder of the workloads but the DiT's 72): K / V copied straight to LDS;
    // the copies address a (batch, head) slice with 32-bit byte offsets
    const bool dtl = a.d_head == 64 && (size_t)a.Nk * std::max(a.ldk, a.ldv) * 2 < (1ull << 31);
    if (dtl) {
      if (a.causal) hipLaunchKernelGGL((attn_fwd_dtl_kernel<true>), grid, dim3(256), 0, s, k);
      else hipLaunchKernelGGL((attn_fwd_dtl_kernel<false>), grid, dim3(256), 0, s, k);
    } else if (a.d_head <= 64) {
      if (qt2) {
        if (a.causal) hipLaunchKernelGGL((attn_fwd_bf16_kernel<64, true, 2>), grid, dim3(256), 0, s, k);
        else hipLaunchKernelGGL((attn_fwd_bf16_kernel<64, false, 2>), grid, dim3(256), 0, s, k);
      } else {
        if (a.causal) hipLaunchKernelGGL((attn_fwd_bf16_kernel<64, true, 1>), grid, dim3(256), 0, s, k);
        else hipLaunchKernelGGL((attn_fwd_bf16_kernel<64, false, 1>), grid, dim3(256), 0, s, k);
      }
    } else {
      if (a.causal) hipLaunchKernelGGL((attn_fwd_bf16_kernel<96, true, 1>), grid, dim3(256), 0, s, k);
      else hipLaunchKernelGGL((attn_fwd_bf16_kernel<96, false, 1>), grid, dim3(256), 0, s, k);
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
    // d_head = 64: streamed tiles copied straight to LDS; a (batch, head) slice is addressed with 32-bit byte offsets
    const bool dtl = a.d_head == 64 && (size_t)std::max(a.Nq, a.Nk) * std::max(std::max(a.ldq, a.lddo), std::max(a.ldk, a.ldv)) * 2 < (1ull << 31);
    {
      KScope ks(KK_ATTN_BWD_DQ, fl, by, s, a.Nq, a.Nk, a.d_head);
      if (dtl) hipLaunchKernelGGL(attn_bwd_dq_dtl_kernel, gq, dim3(256), 0, s, k);
      else if (a.d_head <= 64) hipLaunchKernelGGL(attn_bwd_dq_bf16_kernel<64>, gq, dim3(256), 0, s, k);
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
        if (dtl) hipLaunchKernelGGL(attn_bwd_dkv_dtl_kernel, gk2, dim3(256), 0, s, k2);
        else if (a.d_head <= 64) hipLaunchKernelGGL(attn_bwd_dkv_bf16_kernel<64>, gk2, dim3(256), 0, s, k2);
        else hipLaunchKernelGGL(attn_bwd_dkv_bf16_kernel<96>, gk2, dim3(256), 0, s, k2);
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
