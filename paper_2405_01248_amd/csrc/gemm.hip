// GEMM kernels for the projections and MLPs of a stage (forward y = x W^T, backward
// dx = dy W and dW = dy^T x), fp32 accumulation, with fused epilogues.
//
// bf16 path: MFMA 32x32x16 tiles fed from LDS.  An operand whose contraction index is
// contiguous in memory is staged [rows][BK] and read with 16-byte LDS loads; an operand
// whose contraction index is the slow one (weights in dx, both operands in dW) is staged
// [BK][cols] exactly as it sits in HBM and read with the transposing LDS load, so no
// transposed copy of a weight or activation is ever materialised.
// fp32 path: plain FMA tiles (used by the small fp32 configuration only).
#include "dp_device.h"
#include "dp_kernels.h"
#include "dp_errors.h"
#include "dp_ktime.h"

namespace dp {

template <typename T>
struct EpiParams {
  int M, N;
  T* out; int ldo;
  float* out32; int ldo32; int accumulate;
  float* partial;                 // split-K partial tiles [z][M][N] when gridDim.z > 1
  const T* bias;
  T* pre_out; int ld_pre;
  int act;
  const T* dact_pre; int ld_dact; int dact_kind;
  const T* gate; int gate_ld; int rows_per_batch;
  const void* residual; int ld_res; int residual_f32; int out_fused_f32;
};

// Epilogue of one accumulator element (bounds already checked by the caller).
template <typename T>
__device__ __forceinline__ void epi_fused(const EpiParams<T>& e, int m, int n, float v) {
  if (e.bias) v += to_f<T>(e.bias[n]);
  if (e.pre_out) e.pre_out[(size_t)m * e.ld_pre + n] = from_f<T>(v);
  if (e.act) v = act_apply(e.act, v);
  if (e.dact_pre) v *= act_grad(e.dact_kind, to_f<T>(e.dact_pre[(size_t)m * e.ld_dact + n]));
  if (e.gate) v *= to_f<T>(e.gate[(size_t)(m / e.rows_per_batch) * e.gate_ld + n]);
  if (e.residual) v += to_f<T>(((const T*)e.residual)[(size_t)m * e.ld_res + n]);
  e.out[(size_t)m * e.ldo + n] = from_f<T>(v);
}

template <typename T>
__device__ __forceinline__ void epi_store(const EpiParams<T>& e, int m, int n, float v) {
  if (m < e.M && n < e.N) {
    if (e.partial) e.partial[((size_t)blockIdx.z * e.M + m) * e.N + n] = v;
    else if (e.out32) {
      float* p = e.out32 + (size_t)m * e.ldo32 + n;
      *p = e.accumulate ? (*p + v) : v;
    } else epi_fused<T>(e, m, n, v);
  }
}

// ------------------------------------------------------------------ bf16 MFMA kernel
struct GemmBf16Params {
  const bf16* A; const bf16* B;
  int M, N, K, lda, ldb;
  int k_tiles_per_split;
  EpiParams<bf16> epi;
};

template <int BM, int BN, int BK, bool A_MC, bool B_MC>
struct GemmSmem {
  // [rows][BK + 8] for contraction-contiguous operands; [BK][cols + 16] for the others
  static constexpr int A_LD = A_MC ? (BM + 16) : (BK + 8);
  static constexpr int B_LD = B_MC ? (BN + 16) : (BK + 8);
  static constexpr int A_ELEMS = A_MC ? BK * A_LD : BM * A_LD;
  static constexpr int B_ELEMS = B_MC ? BK * B_LD : BN * B_LD;
};

template <int BM, int BN, int BK, int WGM, int WGN, bool A_MC, bool B_MC>
__global__ void __launch_bounds__(WGM * WGN * 64)
gemm_bf16_kernel(const GemmBf16Params p) {
  using S = GemmSmem<BM, BN, BK, A_MC, B_MC>;
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
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

  const int total_kt = (p.K + BK - 1) / BK;
  const int kt_begin = blockIdx.z * p.k_tiles_per_split;
  const int kt_end = min(total_kt, kt_begin + p.k_tiles_per_split);

  bf16x8 ra[A_PER], rb[B_PER];
#define DP_GEMM_LOAD_GLOBAL(kt_)                                                              \
  {                                                                                           \
    const int k0_ = (kt_) * BK;                                                               \
    _Pragma("unroll") for (int i = 0; i < A_PER; ++i) {                                       \
      const int id = tid + i * NT;                                                            \
      if (A_MC) {                                                                             \
        const int kk = id / (BM / 8), c = id % (BM / 8);                                      \
        const int gk = k0_ + kk, gm = m0 + c * 8;                                             \
        ra[i] = ld8(p.A + (size_t)gk * p.lda + gm, gk < p.K && gm < p.M);                     \
      } else {                                                                                \
        const int r = id / (BK / 8), c = id % (BK / 8);                                       \
        const int gm = m0 + r, gk = k0_ + c * 8;                                              \
        ra[i] = ld8(p.A + (size_t)gm * p.lda + gk, gm < p.M && gk < p.K);                     \
      }                                                                                       \
    }                                                                                         \
    _Pragma("unroll") for (int i = 0; i < B_PER; ++i) {                                       \
      const int id = tid + i * NT;                                                            \
      if (B_MC) {                                                                             \
        const int kk = id / (BN / 8), c = id % (BN / 8);                                      \
        const int gk = k0_ + kk, gn = n0 + c * 8;                                             \
        rb[i] = ld8(p.B + (size_t)gk * p.ldb + gn, gk < p.K && gn < p.N);                     \
      } else {                                                                                \
        const int r = id / (BK / 8), c = id % (BK / 8);                                       \
        const int gn = n0 + r, gk = k0_ + c * 8;                                              \
        rb[i] = ld8(p.B + (size_t)gn * p.ldb + gk, gn < p.N && gk < p.K);                     \
      }                                                                                       \
    }                                                                                         \
  }
#define DP_GEMM_STORE_LDS(buf_)                                                               \
  {                                                                                           \
    bf16* as_ = As + (buf_) * S::A_ELEMS;                                                     \
    bf16* bs_ = Bs + (buf_) * S::B_ELEMS;                                                     \
    _Pragma("unroll") for (int i = 0; i < A_PER; ++i) {                                       \
      const int id = tid + i * NT;                                                            \
      if (A_MC) { const int kk = id / (BM / 8), c = id % (BM / 8); *reinterpret_cast<bf16x8*>(as_ + kk * S::A_LD + c * 8) = ra[i]; } \
      else      { const int r = id / (BK / 8), c = id % (BK / 8);  *reinterpret_cast<bf16x8*>(as_ + r * S::A_LD + c * 8) = ra[i]; }  \
    }                                                                                         \
    _Pragma("unroll") for (int i = 0; i < B_PER; ++i) {                                       \
      const int id = tid + i * NT;                                                            \
      if (B_MC) { const int kk = id / (BN / 8), c = id % (BN / 8); *reinterpret_cast<bf16x8*>(bs_ + kk * S::B_LD + c * 8) = rb[i]; } \
      else      { const int r = id / (BK / 8), c = id % (BK / 8);  *reinterpret_cast<bf16x8*>(bs_ + r * S::B_LD + c * 8) = rb[i]; }  \
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
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        if (A_MC) fa[i] = frag_from_mc(as + (ks * 16) * S::A_LD + wm0 + i * 32, S::A_LD, lane);
        else      fa[i] = *reinterpret_cast<const bf16x8*>(as + (wm0 + i * 32 + l32) * S::A_LD + ks * 16 + 8 * g);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        if (B_MC) fb[j] = frag_from_mc(bs + (ks * 16) * S::B_LD + wn0 + j * 32, S::B_LD, lane);
        else      fb[j] = *reinterpret_cast<const bf16x8*>(bs + (wn0 + j * 32 + l32) * S::B_LD + ks * 16 + 8 * g);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(fa[i], fb[j], acc[i][j]);
    }
    if (more) DP_GEMM_STORE_LDS(buf ^ 1);
    __syncthreads();
  }

  // Epilogue: accumulators -> LDS (fp32, reusing the operand tiles) -> 8 consecutive columns
  // per thread, so that bias / residual / saved pre-activation loads and all stores are
  // 16-byte accesses along the contiguous dimension.
  constexpr int C_LD = BN + 4;
  static_assert((size_t)BM * C_LD * sizeof(float) <= 2 * (size_t)(S::A_ELEMS + S::B_ELEMS) * sizeof(bf16), "C tile must fit");
  float* Cs = reinterpret_cast<float*>(smem_raw);
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        Cs[(wm0 + i * 32 + 8 * (r >> 2) + 4 * g + (r & 3)) * C_LD + wn0 + j * 32 + l32] = acc[i][j][r];
  __syncthreads();
  const EpiParams<bf16>& e = p.epi;
  for (int idx = tid; idx < BM * BN / 8; idx += NT) {
    const int lm = idx / (BN / 8), ln = (idx % (BN / 8)) * 8;
    const int m = m0 + lm, n = n0 + ln;
    if (m >= p.M || n >= p.N) continue;
    float v[8];
    *reinterpret_cast<f32x4*>(&v[0]) = *reinterpret_cast<const f32x4*>(&Cs[lm * C_LD + ln]);
    *reinterpret_cast<f32x4*>(&v[4]) = *reinterpret_cast<const f32x4*>(&Cs[lm * C_LD + ln + 4]);
    if (e.partial || e.out32) {
      float* o = e.partial ? e.partial + ((size_t)blockIdx.z * p.M + m) * p.N + n : e.out32 + (size_t)m * e.ldo32 + n;
      if (!e.partial && e.accumulate) {
        const f32x4 o0 = *reinterpret_cast<const f32x4*>(o), o1 = *reinterpret_cast<const f32x4*>(o + 4);
#pragma unroll
        for (int t = 0; t < 4; ++t) { v[t] += o0[t]; v[4 + t] += o1[t]; }
      }
      *reinterpret_cast<f32x4*>(o) = *reinterpret_cast<const f32x4*>(&v[0]);
      *reinterpret_cast<f32x4*>(o + 4) = *reinterpret_cast<const f32x4*>(&v[4]);
      continue;
    }
    if (e.bias) {
      const bf16x8 bv = *reinterpret_cast<const bf16x8*>(e.bias + n);
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] += (float)bv[t];
    }
    if (e.pre_out) {
      bf16x8 o;
#pragma unroll
      for (int t = 0; t < 8; ++t) o[t] = (bf16)v[t];
      *reinterpret_cast<bf16x8*>(e.pre_out + (size_t)m * e.ld_pre + n) = o;
    }
    if (e.act) {
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] = act_apply(e.act, v[t]);
    }
    if (e.dact_pre) {
      const bf16x8 pv = *reinterpret_cast<const bf16x8*>(e.dact_pre + (size_t)m * e.ld_dact + n);
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] *= act_grad(e.dact_kind, (float)pv[t]);
    }
    if (e.gate) {
      const bf16x8 gv = *reinterpret_cast<const bf16x8*>(e.gate + (size_t)(m / e.rows_per_batch) * e.gate_ld + n);
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] *= (float)gv[t];
    }
    if (e.residual) {
      if (e.residual_f32) {
        const float* rp = (const float*)e.residual + (size_t)m * e.ld_res + n;
        const f32x4 r0 = *reinterpret_cast<const f32x4*>(rp), r1 = *reinterpret_cast<const f32x4*>(rp + 4);
#pragma unroll
        for (int t = 0; t < 4; ++t) { v[t] += r0[t]; v[4 + t] += r1[t]; }
      } else {
        const bf16x8 rv = *reinterpret_cast<const bf16x8*>((const bf16*)e.residual + (size_t)m * e.ld_res + n);
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] += (float)rv[t];
      }
    }
    if (e.out_fused_f32) {
      float* op = reinterpret_cast<float*>(e.out) + (size_t)m * e.ldo + n;
      *reinterpret_cast<f32x4*>(op) = *reinterpret_cast<const f32x4*>(&v[0]);
      *reinterpret_cast<f32x4*>(op + 4) = *reinterpret_cast<const f32x4*>(&v[4]);
    } else {
      bf16x8 o;
#pragma unroll
      for (int t = 0; t < 8; ++t) o[t] = (bf16)v[t];
      *reinterpret_cast<bf16x8*>(e.out + (size_t)m * e.ldo + n) = o;
    }
  }
}

#undef DP_GEMM_LOAD_GLOBAL
#undef DP_GEMM_STORE_LDS

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
  return e;
}

static int choose_splits(int M, int N, int K, int BM, int BN, int BK) {
  const long tiles = (long)((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const int kt = (K + BK - 1) / BK;
  int s = 1;
  // aim for >= 512 workgroups (two per CU) while keeping >= 8 k-tiles per split
  while (tiles * s < 512 && kt / (s * 2) >= 8 && s < 64) s *= 2;
  return s;
}

size_t gemm_splitk_ws_bytes(int M, int N, int K) {
  int s = choose_splits(M, N, K, 128, 128, 64);
  return s > 1 ? (size_t)s * M * N * sizeof(float) : 0;
}

template <int BM, int BN, int BK, int WGM, int WGN, bool A_MC, bool B_MC>
static int launch_bf16_cfg(const GemmArgs& a, hipStream_t s) {
  using S = GemmSmem<BM, BN, BK, A_MC, B_MC>;
  GemmBf16Params p;
  p.A = (const bf16*)a.A; p.B = (const bf16*)a.B;
  p.M = a.M; p.N = a.N; p.K = a.K; p.lda = a.lda; p.ldb = a.ldb;
  p.epi = make_epi<bf16>(a);
  const int kt = (a.K + BK - 1) / BK;
  int splits = 1;
  if (a.out_f32) {
    splits = choose_splits(a.M, a.N, a.K, BM, BN, BK);
    if (splits > 1) {
      const size_t need = (size_t)splits * a.M * a.N * sizeof(float);
      if (!a.splitk_ws || a.splitk_ws_bytes < need) splits = 1;
    }
  }
  p.k_tiles_per_split = (kt + splits - 1) / splits;
  splits = (kt + p.k_tiles_per_split - 1) / p.k_tiles_per_split;
  if (splits > 1) p.epi.partial = a.splitk_ws;
  dim3 grid((a.N + BN - 1) / BN, (a.M + BM - 1) / BM, splits);
  const size_t smem = 2 * (size_t)(S::A_ELEMS + S::B_ELEMS) * sizeof(bf16);
  auto kern = gemm_bf16_kernel<BM, BN, BK, WGM, WGN, A_MC, B_MC>;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
      return set_error(DP_EHIP, "hipFuncSetAttribute(gemm) failed");
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(WGM * WGN * 64), smem, s, p);
  if (hipGetLastError() != hipSuccess) return set_error(DP_EHIP, "gemm launch failed");
  if (splits > 1) return launch_reduce_partials(a.splitk_ws, splits, (size_t)a.M * a.N, a.out_f32, a.accumulate, s);
  return DP_OK;
}

template <int BM, int BN, int BK, int WGM, int WGN>
static int launch_bf16_layout(const GemmArgs& a, hipStream_t s) {
  if (!a.a_mc && !a.b_mc) return launch_bf16_cfg<BM, BN, BK, WGM, WGN, false, false>(a, s);
  if (!a.a_mc && a.b_mc) return launch_bf16_cfg<BM, BN, BK, WGM, WGN, false, true>(a, s);
  if (a.a_mc && a.b_mc) return launch_bf16_cfg<BM, BN, BK, WGM, WGN, true, true>(a, s);
  return launch_bf16_cfg<BM, BN, BK, WGM, WGN, true, false>(a, s);
}

int launch_gemm(const GemmArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return set_error(DP_EINVAL, "gemm: non-positive size");
  if (!a.A || !a.B || (!a.out && !a.out_f32)) return set_error(DP_EINVAL, "gemm: null operand");
  if (a.out_f32 && a.ldo32 < a.N) return set_error(DP_EINVAL, "gemm: ldo32 < N");
  if (a.out_f32 && a.ldo32 != a.N) return set_error(DP_EUNSUPPORTED, "gemm: fp32 output must be dense");
  if (a.dtype == BF16) {
    // 16-byte vector loads: every row start and the contiguous extent must be multiples of 8 elements
    const int a_inner = a.a_mc ? a.M : a.K, b_inner = a.b_mc ? a.N : a.K;
    if ((a.lda % 8) || (a.ldb % 8) || (a_inner % 8) || (b_inner % 8))
      return set_error(DP_EUNSUPPORTED, "gemm(bf16): leading dims and contiguous extents must be multiples of 8");
    if (((uintptr_t)a.A % 16) || ((uintptr_t)a.B % 16)) return set_error(DP_EALIGN, "gemm(bf16): operands must be 16-byte aligned");
    if (a.lda < a_inner || a.ldb < b_inner) return set_error(DP_EINVAL, "gemm: leading dim too small");
    if (a.N % 8) return set_error(DP_EUNSUPPORTED, "gemm(bf16): N must be a multiple of 8");
    const int elds[] = {a.out ? a.ldo : 8, a.pre_out ? a.ld_pre : 8, a.dact_pre ? a.ld_dact : 8, a.gate ? a.gate_ld : 8, a.residual ? a.ld_res : 8};
    for (int x : elds) if (x % 8 || x < 8) return set_error(DP_EUNSUPPORTED, "gemm(bf16): epilogue leading dims must be multiples of 8");
    const void* eps[] = {a.out, a.out_f32, a.bias, a.pre_out, a.dact_pre, a.gate, a.residual, a.splitk_ws};
    for (const void* x : eps) if ((uintptr_t)x % 16) return set_error(DP_EALIGN, "gemm(bf16): epilogue operands must be 16-byte aligned");
    KScope ks(a.a_mc ? KK_GEMM_TN : (a.b_mc ? KK_GEMM_NN : KK_GEMM_NT), 2.0 * a.M * a.N * a.K,
              2.0 * ((double)a.M * a.K + (double)a.N * a.K + (double)a.M * a.N), s, a.M, a.N, a.K);
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
