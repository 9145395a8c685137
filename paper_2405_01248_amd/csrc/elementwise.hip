// Bandwidth-bound kernels of a stage: LayerNorm forward/backward (affine or adaLN
// modulated), GeGLU, SiLU, gated-residual backward, column sums (bias gradients),
// split-K partial reduction, embedding gather.  One wave per token row with 16-byte
// accesses; all reductions are in a fixed order (no float atomics), so results are
// run-to-run identical.  Templated on the storage type (bf16 or fp32); math is fp32.
#include "dp_device.h"
#include "dp_kernels.h"
#include "dp_errors.h"
#include "dp_ktime.h"

namespace dp {

template <typename T> struct Vec;
template <> struct Vec<bf16> { static constexpr int N = 8; typedef bf16x8 type; };
template <> struct Vec<float> { static constexpr int N = 4; typedef f32x4 type; };

template <typename T> __device__ __forceinline__ void load_vec(const T* p, float* out) {
  typename Vec<T>::type v = *reinterpret_cast<const typename Vec<T>::type*>(p);
#pragma unroll
  for (int i = 0; i < Vec<T>::N; ++i) out[i] = to_f<T>(v[i]);
}
template <typename T> __device__ __forceinline__ void store_vec(T* p, const float* in) {
  typename Vec<T>::type v;
#pragma unroll
  for (int i = 0; i < Vec<T>::N; ++i) v[i] = from_f<T>(in[i]);
  *reinterpret_cast<typename Vec<T>::type*>(p) = v;
}

// V consecutive fp32 values (V = 4 or 8)
template <int V> __device__ __forceinline__ void load_f32(const float* p, float* out) {
#pragma unroll
  for (int i = 0; i < V; i += 4) *reinterpret_cast<f32x4*>(out + i) = *reinterpret_cast<const f32x4*>(p + i);
}
template <int V> __device__ __forceinline__ void store_f32(float* p, const float* in) {
#pragma unroll
  for (int i = 0; i < V; i += 4) *reinterpret_cast<f32x4*>(p + i) = *reinterpret_cast<const f32x4*>(in + i);
}

constexpr int LN_MAXCH = 4;   // a lane holds up to 4 vectors of the row: d <= 64 * 4 * Vec::N

// ------------------------------------------------------------------ LayerNorm forward
template <typename TX, typename T>
__global__ void __launch_bounds__(256) ln_fwd_kernel(int rows, int d, float eps, const TX* __restrict__ x, T* __restrict__ y,
                                                     const T* __restrict__ gamma, const T* __restrict__ beta,
                                                     const T* __restrict__ scale, const T* __restrict__ shift, int mod_ld,
                                                     int rows_per_batch, float* __restrict__ mean, float* __restrict__ rstd,
                                                     float* __restrict__ x32_out) {
  constexpr int V = Vec<T>::N;
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const TX* xr = x + (size_t)row * d;
  float v[LN_MAXCH][V];
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < LN_MAXCH; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < d) {
      if (sizeof(TX) == 4) load_f32<V>(reinterpret_cast<const float*>(xr + col), v[c]);
      else load_vec<T>(reinterpret_cast<const T*>(xr + col), v[c]);
      if (sizeof(TX) != 4 && x32_out) store_f32<V>(x32_out + (size_t)row * d + col, v[c]);
#pragma unroll
      for (int i = 0; i < V; ++i) s += v[c][i];
    }
  }
  // gain and shift are fetched right behind the row, not after the two reductions: on a few rows the kernel's
  // time is its chain of memory round trips
  using VT = typename Vec<T>::type;
  VT ga[LN_MAXCH], sh[LN_MAXCH];
  const size_t mrow = scale ? (size_t)(row / rows_per_batch) * mod_ld : 0;
  const T* gsrc = scale ? scale + mrow : gamma;
  const T* ssrc = scale ? shift + mrow : beta;
#pragma unroll
  for (int c = 0; c < LN_MAXCH; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < d && gsrc) {
      ga[c] = *reinterpret_cast<const VT*>(gsrc + col);
      sh[c] = *reinterpret_cast<const VT*>(ssrc + col);
    }
  }
  const float mu = wave_sum(s) / d;
  float q = 0.f;
#pragma unroll
  for (int c = 0; c < LN_MAXCH; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < d) {
#pragma unroll
      for (int i = 0; i < V; ++i) { v[c][i] -= mu; q += v[c][i] * v[c][i]; }
    }
  }
  const float rs = rsqrtf(wave_sum(q) / d + eps);
  if (lane == 0) {
    if (mean) mean[row] = mu;
    if (rstd) rstd[row] = rs;
  }
#pragma unroll
  for (int c = 0; c < LN_MAXCH; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < d) {
      float o[V];
      if (scale) {
#pragma unroll
        for (int i = 0; i < V; ++i) o[i] = v[c][i] * rs * (1.0f + to_f<T>(ga[c][i])) + to_f<T>(sh[c][i]);
      } else if (gamma) {
#pragma unroll
        for (int i = 0; i < V; ++i) o[i] = v[c][i] * rs * to_f<T>(ga[c][i]) + to_f<T>(sh[c][i]);
      } else {
#pragma unroll
        for (int i = 0; i < V; ++i) o[i] = v[c][i] * rs;
      }
      store_vec<T>(y + (size_t)row * d + col, o);
    }
  }
}

template <typename TX, typename T>
static int ln_fwd_t(const LnArgs& a, hipStream_t s) {
  hipLaunchKernelGGL((ln_fwd_kernel<TX, T>), dim3((a.rows + 3) / 4), dim3(256), 0, s, a.rows, a.d, a.eps, (const TX*)a.x, (T*)a.y,
                     (const T*)a.gamma, (const T*)a.beta, (const T*)a.scale, (const T*)a.shift, a.mod_ld,
                     a.rows_per_batch > 0 ? a.rows_per_batch : a.rows, a.mean, a.rstd, a.x32_out);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "ln_fwd launch failed");
}

// Split-K reduction onto the fp32 residual stream fused with the LayerNorm that follows (bf16 storage).
// NCH: number of 512-column chunks a row spans.
template <int NCH>
__global__ void __launch_bounds__(256) reduce_residual_ln_kernel(int rows, int d, float eps, const float* __restrict__ partial, int splits,
                                                                 const bf16* __restrict__ bias, float* __restrict__ x, bf16* __restrict__ y,
                                                                 const bf16* __restrict__ gamma, const bf16* __restrict__ beta) {
  constexpr int V = 8;
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const size_t plane = (size_t)rows * d;
  // The partial sums are added in ascending split order (fixed summation order), but their loads are issued four
  // planes at a time for all of the row's chunks: on a slice of a few samples the kernel runs on a few dozen
  // workgroups and its time is the chain of memory round trips, one per plane when load and add alternate.
  float v[NCH][V], acc[NCH][V];
  bf16x8 bi[NCH], ga[NCH], be[NCH];     // fetched with the row, used after the reductions
  const float* prow = partial + (size_t)row * d;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < d) {
      load_f32<V>(x + (size_t)row * d + col, v[c]);
      load_f32<V>(prow + col, acc[c]);
      if (bias) bi[c] = *reinterpret_cast<const bf16x8*>(bias + col);
      ga[c] = *reinterpret_cast<const bf16x8*>(gamma + col);
      be[c] = *reinterpret_cast<const bf16x8*>(beta + col);
    }
  }
  int z = 1;
  for (; z + 3 < splits; z += 4) {
    float t[4][NCH][V];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const int col = (c * 64 + lane) * V;
        if (col < d) load_f32<V>(prow + (size_t)(z + u) * plane + col, t[u][c]);
      }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const int col = (c * 64 + lane) * V;
        if (col < d) {
#pragma unroll
          for (int i = 0; i < V; ++i) acc[c][i] += t[u][c][i];
        }
      }
  }
  for (; z < splits; ++z) {
    float t[NCH][V];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (c * 64 + lane) * V;
      if (col < d) load_f32<V>(prow + (size_t)z * plane + col, t[c]);
    }
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (c * 64 + lane) * V;
      if (col < d) {
#pragma unroll
        for (int i = 0; i < V; ++i) acc[c][i] += t[c][i];
      }
    }
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < d) {
      if (bias) {
#pragma unroll
        for (int i = 0; i < V; ++i) acc[c][i] += (float)bi[c][i];
      }
#pragma unroll
      for (int i = 0; i < V; ++i) { v[c][i] += acc[c][i]; s += v[c][i]; }
      store_f32<V>(x + (size_t)row * d + col, v[c]);
    }
  }
  const float mu = wave_sum(s) / d;
  float q = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < d) {
#pragma unroll
      for (int i = 0; i < V; ++i) { v[c][i] -= mu; q += v[c][i] * v[c][i]; }
    }
  }
  const float rs = rsqrtf(wave_sum(q) / d + eps);
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < d) {
      float o[V];
#pragma unroll
      for (int i = 0; i < V; ++i) o[i] = v[c][i] * rs * (float)ga[c][i] + (float)be[c][i];
      store_vec<bf16>(y + (size_t)row * d + col, o);
    }
  }
}

int launch_reduce_residual_ln(const float* partial, int splits, int rows, int d, const void* bias, float* x, void* y,
                              const void* gamma, const void* beta, float eps, hipStream_t s) {
  if (!partial || splits < 1 || rows <= 0 || !x || !y || !gamma || !beta) return set_error(DP_EINVAL, "reduce_residual_ln: bad arguments");
  if (d <= 0 || d % 8 || d > 64 * LN_MAXCH * 8) return set_error(DP_EUNSUPPORTED, "reduce_residual_ln: d must be a multiple of 8, at most 2048");
  KScope ks(KK_REDUCE, 0.0, (double)rows * d * (4.0 * splits + 8.0 + 2.0), s, rows, d, splits);
  const dim3 grid((rows + 3) / 4);
#define DP_RRLN(n_) hipLaunchKernelGGL(reduce_residual_ln_kernel<n_>, grid, dim3(256), 0, s, rows, d, eps, partial, splits, (const bf16*)bias, x, \
                                       (bf16*)y, (const bf16*)gamma, (const bf16*)beta)
  switch ((d + 511) / 512) {
    case 1: DP_RRLN(1); break;
    case 2: DP_RRLN(2); break;
    case 3: DP_RRLN(3); break;
    default: DP_RRLN(4); break;
  }
#undef DP_RRLN
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "reduce_residual_ln launch failed");
}

static int check_ln_dim(int dtype, int d) {
  const int V = dtype == BF16 ? 8 : 4;
  if (d <= 0 || d % V) return set_error(DP_EUNSUPPORTED, "layernorm: d must be a positive multiple of 8 (bf16) / 4 (fp32)");
  if (d > 64 * LN_MAXCH * V) return set_error(DP_EUNSUPPORTED, "layernorm: d too large (max 2048 bf16 / 1024 fp32)");
  return DP_OK;
}

int launch_ln_fwd(const LnArgs& a, hipStream_t s) {
  if (a.rows <= 0 || !a.x || !a.y) return set_error(DP_EINVAL, "ln_fwd: bad arguments");
  if (int e = check_ln_dim(a.dtype, a.d)) return e;
  if ((a.gamma == nullptr) != (a.beta == nullptr) || (a.scale == nullptr) != (a.shift == nullptr))
    return set_error(DP_EINVAL, "ln_fwd: gamma/beta and scale/shift come in pairs");
  if (a.x32_out && (a.x_f32 || a.dtype != BF16 || ((uintptr_t)a.x32_out % 16))) return set_error(DP_EINVAL, "ln_fwd: the widened copy goes with a bf16 input and a 16-byte aligned destination");
  KScope ks(KK_LN_FWD, 0.0, a.rows * (double)a.d * (dtype_size(a.dtype) + (a.x_f32 ? 4 : dtype_size(a.dtype)) + (a.x32_out ? 4 : 0)) + 8.0 * a.rows, s, a.rows, a.d);
  if (a.dtype == BF16) return a.x_f32 ? ln_fwd_t<float, bf16>(a, s) : ln_fwd_t<bf16, bf16>(a, s);
  return ln_fwd_t<float, float>(a, s);
}

// ------------------------------------------------------------------ LayerNorm backward
constexpr int LNB_ROWS = 16;   // rows per workgroup (4 per wave)

// grid = (chunks_per_batch, n_batches).  partial: [batch][chunk][2][d]
// NCH = number of 64-lane vector chunks a row spans (d <= 64 * V * NCH).  A wave owns every fourth row of the
// workgroup's 16.  All loads of a row (dy, x, the residual gradient) are issued before the first is used; rows
// of a single chunk (d <= 512 in bf16) are taken two at a time, which doubles the bytes in flight per wave --
// the kernel moves ~16 bytes per element and is bound by how much of that is outstanding, not by arithmetic.
template <typename T, int NCH>
__global__ void __launch_bounds__(256) ln_bwd_kernel(int d, int rows_per_batch, const T* __restrict__ dy, const float* __restrict__ x,
                                                     const float* __restrict__ mean, const float* __restrict__ rstd,
                                                     const T* __restrict__ gamma, const T* __restrict__ scale, int mod_ld,
                                                     const float* __restrict__ dres, const T* __restrict__ dres_t,
                                                     T* __restrict__ dx, float* __restrict__ dx32, float* __restrict__ partial) {
  constexpr int V = Vec<T>::N;
  using VT = typename Vec<T>::type;
  extern __shared__ float cols[];   // [4 waves][2][d]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.y;
  const int r_begin = blockIdx.x * LNB_ROWS, r_end = min(rows_per_batch, r_begin + LNB_ROWS);
  float gsum[NCH][V], bsum[NCH][V], gain[NCH][V];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (c * 64 + lane) * V;
#pragma unroll
    for (int i = 0; i < V; ++i) { gsum[c][i] = 0.f; bsum[c][i] = 0.f; gain[c][i] = 1.f; }
    if (col < d) {
      if (scale) {
        load_vec<T>(scale + (size_t)b * mod_ld + col, gain[c]);
#pragma unroll
        for (int i = 0; i < V; ++i) gain[c][i] += 1.0f;
      } else if (gamma) {
        load_vec<T>(gamma + col, gain[c]);
      }
    }
  }
  struct Row {
    size_t row; float mu, rs, s1, s2;
    VT dyr[NCH], drt[NCH];            // raw loads
    float xr[NCH][V], drf[NCH][V];
    float g[NCH][V], xh[NCH][V];
  };
  auto issue = [&](Row& R, int r) {
    R.row = (size_t)b * rows_per_batch + r;
    R.mu = mean[R.row]; R.rs = rstd[R.row];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (c * 64 + lane) * V;
      if (col < d) {
        R.dyr[c] = *reinterpret_cast<const VT*>(dy + R.row * d + col);
        load_f32<V>(x + R.row * d + col, R.xr[c]);
        if (dres) load_f32<V>(dres + R.row * d + col, R.drf[c]);
        else if (dres_t) R.drt[c] = *reinterpret_cast<const VT*>(dres_t + R.row * d + col);
      }
    }
  };
  auto reduce_in = [&](Row& R) {
    R.s1 = 0.f; R.s2 = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (c * 64 + lane) * V;
      if (col < d) {
#pragma unroll
        for (int i = 0; i < V; ++i) {
          const float dyv = to_f<T>(R.dyr[c][i]);
          R.xh[c][i] = (R.xr[c][i] - R.mu) * R.rs;
          gsum[c][i] += dyv * R.xh[c][i];
          bsum[c][i] += dyv;
          R.g[c][i] = dyv * gain[c][i];
          R.s1 += R.g[c][i];
          R.s2 += R.g[c][i] * R.xh[c][i];
        }
      }
    }
  };
  auto finish = [&](Row& R) {
    const float m1 = wave_sum(R.s1) / d, m2 = wave_sum(R.s2) / d;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (c * 64 + lane) * V;
      if (col < d) {
        float o[V];
#pragma unroll
        for (int i = 0; i < V; ++i) o[i] = R.rs * (R.g[c][i] - m1 - R.xh[c][i] * m2);
        if (dres) {
#pragma unroll
          for (int i = 0; i < V; ++i) o[i] += R.drf[c][i];
        } else if (dres_t) {
#pragma unroll
          for (int i = 0; i < V; ++i) o[i] += to_f<T>(R.drt[c][i]);
        }
        if (dx32) store_f32<V>(dx32 + R.row * d + col, o);
        if (dx) store_vec<T>(dx + R.row * d + col, o);
      }
    }
  };
  if (NCH == 1) {
    for (int r = r_begin + wave; r < r_end; r += 8) {
      const bool two = r + 4 < r_end;                        // wave-uniform
      Row A, B;
      issue(A, r);
      if (two) issue(B, r + 4);
      reduce_in(A);
      if (two) reduce_in(B);
      finish(A);
      if (two) finish(B);
    }
  } else {
    // wider rows: a second row's registers would cost occupancy (measured slower at d = 640 and 1152)
    for (int r = r_begin + wave; r < r_end; r += 4) {
      Row A;
      issue(A, r);
      reduce_in(A);
      finish(A);
    }
  }
  if (!partial) return;
  // fixed-order reduction of the four waves' column sums
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (c * 64 + lane) * V;
    if (col < d) {
#pragma unroll
      for (int i = 0; i < V; ++i) {
        cols[(wave * 2 + 0) * d + col + i] = gsum[c][i];
        cols[(wave * 2 + 1) * d + col + i] = bsum[c][i];
      }
    }
  }
  __syncthreads();
  float* out = partial + ((size_t)b * gridDim.x + blockIdx.x) * 2 * d;
  for (int i = threadIdx.x; i < 2 * d; i += 256)
    out[i] = ((cols[i] + cols[2 * d + i]) + cols[4 * d + i]) + cols[6 * d + i];
}

// out_k[b * ld + col] = (acc ? old : 0) + sum_chunks partial[b][chunk][k][col], k = 0 (gain grad), 1 (shift grad).
// grid = (ceil(2d / COLS), n_batches); COLS columns x 1024 / COLS chunk groups per workgroup; every thread sums
// its chunks in ascending order and the group sums are added in ascending order (fixed order).  Fewer columns
// per workgroup mean more workgroups: the unbatched reduction of a narrow model (2d = 640 columns, 1024 chunks)
// ran on 20 workgroups with 32 columns each and took 21 us; with 8 it runs on 80.
template <int COLS>
__global__ void __launch_bounds__(1024) ln_bwd_reduce_kernel(const float* __restrict__ partial, int nchunk, int d, float* out0,
                                                             float* out1, int ld, int accumulate) {
  constexpr int GROUPS = 1024 / COLS;
  __shared__ float red[GROUPS][COLS + 1];
  const int lc = threadIdx.x % COLS, grp = threadIdx.x / COLS;
  const int col = blockIdx.x * COLS + lc, b = blockIdx.y;     // col indexes the [2][d] row of a chunk
  float s = 0.f;
  if (col < 2 * d) {
    const float* p = partial + (size_t)b * nchunk * 2 * d + col;
    for (int c = grp; c < nchunk; c += GROUPS) s += p[(size_t)c * 2 * d];
  }
  red[grp][lc] = s;
  __syncthreads();
  if (grp == 0 && col < 2 * d) {
    float t = 0.f;
#pragma unroll 8
    for (int g = 0; g < GROUPS; ++g) t += red[g][lc];
    float* o = (col < d ? out0 + col : out1 + (col - d)) + (size_t)b * ld;
    *o = accumulate ? *o + t : t;
  }
}

size_t ln_bwd_partial_bytes(int rows, int d, int rows_per_batch) {
  if (rows_per_batch <= 0) rows_per_batch = rows;
  const int nb = rows / rows_per_batch;
  const int nchunk = (rows_per_batch + LNB_ROWS - 1) / LNB_ROWS;
  return (size_t)nb * nchunk * 2 * d * sizeof(float);
}

template <typename T, int NCH>
static void ln_bwd_launch(const LnBwdArgs& a, int rpb, int nb, int nchunk, float* partial, hipStream_t s) {
  hipLaunchKernelGGL((ln_bwd_kernel<T, NCH>), dim3(nchunk, nb), dim3(256), (size_t)8 * a.d * sizeof(float), s, a.d, rpb, (const T*)a.dy,
                     (const float*)a.x, a.mean, a.rstd, (const T*)a.gamma, (const T*)a.scale, a.mod_ld,
                     a.dres_storage ? nullptr : (const float*)a.dres, a.dres_storage ? (const T*)a.dres : nullptr, (T*)a.dx, a.dx32, partial);
}
template <typename T>
static int ln_bwd_t(const LnBwdArgs& a, int rpb, int nb, int nchunk, float* partial, hipStream_t s) {
  const int nch = (a.d + 64 * Vec<T>::N - 1) / (64 * Vec<T>::N);
  switch (nch) {
    case 1: ln_bwd_launch<T, 1>(a, rpb, nb, nchunk, partial, s); break;
    case 2: ln_bwd_launch<T, 2>(a, rpb, nb, nchunk, partial, s); break;
    case 3: ln_bwd_launch<T, 3>(a, rpb, nb, nchunk, partial, s); break;
    default: ln_bwd_launch<T, LN_MAXCH>(a, rpb, nb, nchunk, partial, s); break;
  }
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "ln_bwd launch failed");
}

int launch_ln_bwd(const LnBwdArgs& a, hipStream_t s) {
  if (a.rows <= 0 || !a.dy || !a.x || !a.mean || !a.rstd || (!a.dx && !a.dx32)) return set_error(DP_EINVAL, "ln_bwd: bad arguments");
  if (int e = check_ln_dim(a.dtype, a.d)) return e;
  const bool modulated = a.scale != nullptr;
  const int rpb = modulated ? a.rows_per_batch : a.rows;
  if (rpb <= 0 || a.rows % rpb) return set_error(DP_EINVAL, "ln_bwd: rows must be a multiple of rows_per_batch");
  const int nb = a.rows / rpb, nchunk = (rpb + LNB_ROWS - 1) / LNB_ROWS;
  const bool want_cols = modulated ? (a.dscale && a.dshift) : (a.dgamma && a.dbeta);
  float* partial = nullptr;
  if (want_cols) {
    if (!a.partial || a.partial_bytes < ln_bwd_partial_bytes(a.rows, a.d, rpb)) return set_error(DP_EWORKSPACE, "ln_bwd: partial buffer too small");
    partial = a.partial;
  }
  int e;
  {
    KScope ks(KK_LN_BWD, 0.0, a.rows * (double)a.d * (dtype_size(a.dtype) + 4.0 + (a.dres ? (a.dres_storage ? dtype_size(a.dtype) : 4.0) : 0.0) + (a.dx ? dtype_size(a.dtype) : 0.0) + (a.dx32 ? 4.0 : 0.0)) + 8.0 * a.rows, s, a.rows, a.d);
    e = a.dtype == BF16 ? ln_bwd_t<bf16>(a, rpb, nb, nchunk, partial, s) : ln_bwd_t<float>(a, rpb, nb, nchunk, partial, s);
  }
  if (e || !want_cols || a.defer_reduce) return e;
  return launch_ln_bwd_reduce(a, s);
}

// Second half of launch_ln_bwd: fixed-order sum of the per-workgroup column partials into the parameter
// (or modulation) gradients.  Separate so that a caller can put it on another stream (defer_reduce).
int launch_ln_bwd_reduce(const LnBwdArgs& a, hipStream_t s) {
  const bool modulated = a.scale != nullptr;
  const int rpb = modulated ? a.rows_per_batch : a.rows;
  if (rpb <= 0 || a.rows % rpb || !a.partial) return set_error(DP_EINVAL, "ln_bwd_reduce: bad arguments");
  const int nb = a.rows / rpb, nchunk = (rpb + LNB_ROWS - 1) / LNB_ROWS;
  KScope ks(KK_REDUCE, 0.0, (double)nb * nchunk * 2 * a.d * 4, s, nchunk, 2 * a.d);
  if (modulated)
    hipLaunchKernelGGL(ln_bwd_reduce_kernel<32>, dim3((2 * a.d + 31) / 32, nb), dim3(1024), 0, s, a.partial, nchunk, a.d, a.dscale, a.dshift, a.dmod_ld, 0);
  else if (2 * a.d <= 1024)
    hipLaunchKernelGGL(ln_bwd_reduce_kernel<8>, dim3((2 * a.d + 7) / 8, 1), dim3(1024), 0, s, a.partial, nchunk, a.d, a.dgamma, a.dbeta, a.d, a.accumulate);
  else
    hipLaunchKernelGGL(ln_bwd_reduce_kernel<16>, dim3((2 * a.d + 15) / 16, 1), dim3(1024), 0, s, a.partial, nchunk, a.d, a.dgamma, a.dbeta, a.d, a.accumulate);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "ln_bwd_reduce launch failed");
}

// ------------------------------------------------------------------ GeGLU
template <typename T>
__global__ void geglu_fwd_kernel(const T* __restrict__ u, T* __restrict__ g, size_t rows, int inner) {
  constexpr int V = Vec<T>::N;
  const int per_row = inner / V;
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= rows * per_row) return;
  const size_t r = i / per_row; const int c = (int)(i % per_row) * V;
  float a[V], b[V], o[V];
  load_vec<T>(u + r * 2 * inner + c, a);
  load_vec<T>(u + r * 2 * inner + inner + c, b);
#pragma unroll
  for (int k = 0; k < V; ++k) o[k] = a[k] * gelu_erf_f(b[k]);
  store_vec<T>(g + r * inner + c, o);
}
template <typename T>
__global__ void geglu_bwd_kernel(const T* __restrict__ dg, const T* __restrict__ u, T* __restrict__ du, size_t rows, int inner) {
  constexpr int V = Vec<T>::N;
  const int per_row = inner / V;
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= rows * per_row) return;
  const size_t r = i / per_row; const int c = (int)(i % per_row) * V;
  float a[V], b[V], dgo[V], o1[V], o2[V];
  load_vec<T>(u + r * 2 * inner + c, a);
  load_vec<T>(u + r * 2 * inner + inner + c, b);
  load_vec<T>(dg + r * inner + c, dgo);
#pragma unroll
  for (int k = 0; k < V; ++k) { o1[k] = dgo[k] * gelu_erf_f(b[k]); o2[k] = dgo[k] * a[k] * gelu_erf_grad_f(b[k]); }
  store_vec<T>(du + r * 2 * inner + c, o1);
  store_vec<T>(du + r * 2 * inner + inner + c, o2);
}

static int check_vec(int dtype, int n, const char* what) {
  const int V = dtype == BF16 ? 8 : 4;
  if (n <= 0 || n % V) return set_errorf(DP_EUNSUPPORTED, "%s: width must be a positive multiple of %d", what, V);
  return DP_OK;
}

int launch_geglu_fwd(int dtype, const void* u, void* g, int rows, int inner, hipStream_t s) {
  if (int e = check_vec(dtype, inner, "geglu")) return e;
  const int V = dtype == BF16 ? 8 : 4;
  const size_t n = (size_t)rows * (inner / V);
  KScope ks(KK_GEGLU_FWD, 0.0, 3.0 * rows * (double)inner * dtype_size(dtype), s, rows, inner);
  if (dtype == BF16) hipLaunchKernelGGL(geglu_fwd_kernel<bf16>, dim3((n + 255) / 256), dim3(256), 0, s, (const bf16*)u, (bf16*)g, (size_t)rows, inner);
  else hipLaunchKernelGGL(geglu_fwd_kernel<float>, dim3((n + 255) / 256), dim3(256), 0, s, (const float*)u, (float*)g, (size_t)rows, inner);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "geglu_fwd launch failed");
}
int launch_geglu_bwd(int dtype, const void* dg, const void* u, void* du, int rows, int inner, hipStream_t s) {
  if (int e = check_vec(dtype, inner, "geglu")) return e;
  const int V = dtype == BF16 ? 8 : 4;
  const size_t n = (size_t)rows * (inner / V);
  KScope ks(KK_GEGLU_BWD, 0.0, 5.0 * rows * (double)inner * dtype_size(dtype), s, rows, inner);
  if (dtype == BF16) hipLaunchKernelGGL(geglu_bwd_kernel<bf16>, dim3((n + 255) / 256), dim3(256), 0, s, (const bf16*)dg, (const bf16*)u, (bf16*)du, (size_t)rows, inner);
  else hipLaunchKernelGGL(geglu_bwd_kernel<float>, dim3((n + 255) / 256), dim3(256), 0, s, (const float*)dg, (const float*)u, (float*)du, (size_t)rows, inner);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "geglu_bwd launch failed");
}

// ------------------------------------------------------------------ column sums
constexpr int CS_ROWS = 64;    // rows per workgroup (16 per wave)

// Stage 1: partial[chunk][col] = sum of x over the chunk's rows.  A lane owns Vec::N consecutive
// columns (16-byte loads); the four waves of a workgroup take rows round-robin and are added
// in a fixed order.
template <typename T>
__global__ void __launch_bounds__(256) colsum_kernel(const T* __restrict__ x, int ldx, int rows, int cols, float* __restrict__ partial) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[4][64 * V];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = (blockIdx.x * 64 + lane) * V;
  const int r0 = blockIdx.y * CS_ROWS, r1 = min(rows, r0 + CS_ROWS);
  float s[V];
#pragma unroll
  for (int i = 0; i < V; ++i) s[i] = 0.f;
  if (col < cols) {
    for (int r = r0 + wave; r < r1; r += 4) {
      float v[V];
      load_vec<T>(x + (size_t)r * ldx + col, v);
#pragma unroll
      for (int i = 0; i < V; ++i) s[i] += v[i];
    }
  }
#pragma unroll
  for (int i = 0; i < V; ++i) red[wave][lane * V + i] = s[i];
  __syncthreads();
  for (int t = threadIdx.x; t < 64 * V; t += 256) {
    const int c = blockIdx.x * 64 * V + t;
    if (c < cols) partial[(size_t)blockIdx.y * cols + c] = ((red[0][t] + red[1][t]) + red[2][t]) + red[3][t];
  }
}

// Stage 2: out[c] = (accumulate ? out[c] : 0) + sum_r partial[r][c]; 32 columns x 32 row groups per
// workgroup, each thread sums its rows in ascending order, the 32 group sums are added in ascending order.
__global__ void __launch_bounds__(1024) rows_reduce_kernel(const float* __restrict__ partial, int nrows, int ncols,
                                                           float* __restrict__ out, int accumulate) {
  __shared__ float red[32][33];
  const int lc = threadIdx.x & 31, grp = threadIdx.x >> 5;
  const int col = blockIdx.x * 32 + lc;
  float s = 0.f;
  if (col < ncols)
    for (int r = grp; r < nrows; r += 32) s += partial[(size_t)r * ncols + col];
  red[grp][lc] = s;
  __syncthreads();
  if (grp == 0 && col < ncols) {
    float t = 0.f;
#pragma unroll
    for (int g = 0; g < 32; ++g) t += red[g][lc];
    out[col] = accumulate ? out[col] + t : t;
  }
}

size_t colsum_partial_bytes(int rows, int cols) { return (size_t)((rows + CS_ROWS - 1) / CS_ROWS) * cols * sizeof(float); }

int launch_colsum(int dtype, const void* x, int ldx, int rows, int cols, float* out, int accumulate, float* partial,
                  size_t partial_bytes, hipStream_t s) {
  const int V = dtype == BF16 ? 8 : 4;
  if (rows <= 0 || cols <= 0 || cols % V || ldx % V || !x || !out) return set_error(DP_EINVAL, "colsum: bad arguments (cols must be a multiple of 8 (bf16) / 4 (fp32))");
  if (!partial || partial_bytes < colsum_partial_bytes(rows, cols)) return set_error(DP_EWORKSPACE, "colsum: partial buffer too small");
  dim3 grid((cols + 64 * V - 1) / (64 * V), (rows + CS_ROWS - 1) / CS_ROWS);
  KScope ks(KK_REDUCE, 0.0, (double)rows * cols * dtype_size(dtype), s, rows, cols);
  if (dtype == BF16) hipLaunchKernelGGL(colsum_kernel<bf16>, grid, dim3(256), 0, s, (const bf16*)x, ldx, rows, cols, partial);
  else hipLaunchKernelGGL(colsum_kernel<float>, grid, dim3(256), 0, s, (const float*)x, ldx, rows, cols, partial);
  if (hipGetLastError() != hipSuccess) return set_error(DP_EHIP, "colsum launch failed");
  hipLaunchKernelGGL(rows_reduce_kernel, dim3((cols + 31) / 32), dim3(1024), 0, s, partial, (int)grid.y, cols, out, accumulate);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "rows_reduce launch failed");
}

// out[i] = (accumulate ? out[i] : 0) + sum_z partial[z * n + i], four elements per thread (n % 4 == 0)
__global__ void reduce_partials_kernel(const float* __restrict__ partial, int nz, size_t n4, float* __restrict__ out, int accumulate) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= n4) return;
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
  for (int z = 0; z < nz; ++z) s += reinterpret_cast<const f32x4*>(partial)[(size_t)z * n4 + i];
  f32x4* o = reinterpret_cast<f32x4*>(out) + i;
  *o = accumulate ? *o + s : s;
}
int launch_reduce_partials(const float* partial, int nz, size_t n, float* out, int accumulate, hipStream_t s) {
  if (n % 4) return set_error(DP_EUNSUPPORTED, "reduce_partials: element count must be a multiple of 4");
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((n / 4 + 255) / 256), dim3(256), 0, s, partial, nz, n / 4, out, accumulate);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "reduce_partials launch failed");
}

// Two tensors in one launch: out (n4 vectors of 4) and out_b (nb4 vectors), each summed over nz planes in plane order.
__global__ void reduce_partials2_kernel(const float* __restrict__ partial, int nz, size_t n4, float* __restrict__ out,
                                        const float* __restrict__ partial_b, size_t nb4, float* __restrict__ out_b, int accumulate) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const float* src = partial; float* dst = out; size_t plane = n4;
  if (i >= n4) {
    i -= n4;
    if (i >= nb4) return;
    src = partial_b; dst = out_b; plane = nb4;
  }
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
  for (int z = 0; z < nz; ++z) s += reinterpret_cast<const f32x4*>(src)[(size_t)z * plane + i];
  f32x4* o = reinterpret_cast<f32x4*>(dst) + i;
  *o = accumulate ? *o + s : s;
}
int launch_reduce_partials2(const float* partial, int nz, size_t n, float* out, const float* partial_b, size_t n_b, float* out_b,
                            int accumulate, hipStream_t s) {
  if (n % 4 || n_b % 4) return set_error(DP_EUNSUPPORTED, "reduce_partials: element counts must be multiples of 4");
  if (n_b && (!partial_b || !out_b)) return set_error(DP_EINVAL, "reduce_partials: second tensor missing");
  const size_t total = n / 4 + n_b / 4;
  hipLaunchKernelGGL(reduce_partials2_kernel, dim3((total + 255) / 256), dim3(256), 0, s, partial, nz, n / 4, out, partial_b, n_b / 4, out_b, accumulate);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "reduce_partials launch failed");
}

// ------------------------------------------------------------------ SiLU and its backward
template <typename T>
__global__ void silu_kernel(const T* __restrict__ x, T* __restrict__ y, size_t n) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < n) y[i] = from_f<T>(silu_f(to_f<T>(x[i])));
}
template <typename T>
__global__ void silu_bwd_kernel(const float* __restrict__ dz, const T* __restrict__ c, float* __restrict__ dc, int accumulate, size_t n) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float v = dz[i] * silu_grad_f(to_f<T>(c[i]));
  dc[i] = accumulate ? dc[i] + v : v;
}
int launch_silu(int dtype, const void* x, void* y, size_t n, hipStream_t s) {
  if (dtype == BF16) hipLaunchKernelGGL(silu_kernel<bf16>, dim3((n + 255) / 256), dim3(256), 0, s, (const bf16*)x, (bf16*)y, n);
  else hipLaunchKernelGGL(silu_kernel<float>, dim3((n + 255) / 256), dim3(256), 0, s, (const float*)x, (float*)y, n);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "silu launch failed");
}
int launch_silu_bwd(int dtype, const float* dz, const void* c, float* dc, int accumulate, size_t n, hipStream_t s) {
  if (dtype == BF16) hipLaunchKernelGGL(silu_bwd_kernel<bf16>, dim3((n + 255) / 256), dim3(256), 0, s, dz, (const bf16*)c, dc, accumulate, n);
  else hipLaunchKernelGGL(silu_bwd_kernel<float>, dim3((n + 255) / 256), dim3(256), 0, s, dz, (const float*)c, dc, accumulate, n);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "silu_bwd launch failed");
}

// ------------------------------------------------------------------ gated branch backward
// grid = (ceil(d / (16 V)), B), 16 waves per workgroup.  A workgroup owns 16 V columns (V = 8 bf16 / 4 fp32
// per lane, 16-byte accesses) of one batch; a wave covers 4 rows at a time (lane = row-in-group * 16 +
// column chunk), the 16 waves 64 rows.  Column sums: over a wave's 4 row lanes by shuffles, over the
// waves through LDS in wave order (fixed order).
constexpr int GB_WAVES = 16;
template <typename T>
__global__ void __launch_bounds__(64 * GB_WAVES) gate_bwd_kernel(const float* __restrict__ dres, const T* __restrict__ branch,
                                                                 const T* __restrict__ gate, int gate_ld, T* __restrict__ dbranch,
                                                                 float* __restrict__ dgate, int dgate_ld, int rows_per_batch, int d) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[GB_WAVES][16 * V];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int cl = lane & 15, rl = lane >> 4;
  const int b = blockIdx.y, col = (blockIdx.x * 16 + cl) * V;
  float s[V], g[V];
#pragma unroll
  for (int i = 0; i < V; ++i) s[i] = 0.f;
  if (col < d) {
    load_vec<T>(gate + (size_t)b * gate_ld + col, g);
#pragma unroll 2
    for (int r = wave * 4 + rl; r < rows_per_batch; r += 4 * GB_WAVES) {
      const size_t o = ((size_t)b * rows_per_batch + r) * d + col;
      float dr[V], br[V], ob[V];
      load_f32<V>(dres + o, dr);
      load_vec<T>(branch + o, br);
#pragma unroll
      for (int i = 0; i < V; ++i) { s[i] = fmaf(dr[i], br[i], s[i]); ob[i] = dr[i] * g[i]; }
      store_vec<T>(dbranch + o, ob);
    }
  }
#pragma unroll
  for (int i = 0; i < V; ++i) {
    s[i] += __shfl_xor(s[i], 16, 64);
    s[i] += __shfl_xor(s[i], 32, 64);
  }
  if (rl == 0) {
#pragma unroll
    for (int i = 0; i < V; ++i) red[wave][cl * V + i] = s[i];
  }
  __syncthreads();
  if (threadIdx.x < 16 * V) {
    const int gc = blockIdx.x * 16 * V + threadIdx.x;
    if (gc < d) {
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < GB_WAVES; ++w) t += red[w][threadIdx.x];
      dgate[(size_t)b * dgate_ld + gc] = t;
    }
  }
}
int launch_gate_bwd(int dtype, const void* dres, const void* branch, const void* gate, int gate_ld, void* dbranch, float* dgate,
                    int dgate_ld, int B, int rows_per_batch, int d, hipStream_t s) {
  const int V = dtype == BF16 ? 8 : 4;
  if (B <= 0 || rows_per_batch <= 0 || d <= 0 || d % V || gate_ld % V) return set_error(DP_EINVAL, "gate_bwd: bad sizes");
  const void* ptrs[] = {dres, branch, gate, dbranch};
  for (const void* q : ptrs) if (!q || ((uintptr_t)q % 16)) return set_error(DP_EALIGN, "gate_bwd: operands must be non-null and 16-byte aligned");
  if (!dgate) return set_error(DP_EINVAL, "gate_bwd: dgate is NULL");
  dim3 grid((d + 16 * V - 1) / (16 * V), B);
  if (dtype == BF16) hipLaunchKernelGGL(gate_bwd_kernel<bf16>, grid, dim3(64 * GB_WAVES), 0, s, (const float*)dres, (const bf16*)branch, (const bf16*)gate, gate_ld, (bf16*)dbranch, dgate, dgate_ld, rows_per_batch, d);
  else hipLaunchKernelGGL(gate_bwd_kernel<float>, grid, dim3(64 * GB_WAVES), 0, s, (const float*)dres, (const float*)branch, (const float*)gate, gate_ld, (float*)dbranch, dgate, dgate_ld, rows_per_batch, d);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "gate_bwd launch failed");
}

// ------------------------------------------------------------------ cast, embedding
template <typename T>
__global__ void cast_kernel(const float* __restrict__ in, T* __restrict__ out, size_t n) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < n) out[i] = from_f<T>(in[i]);
}
int launch_cast_from_f32(int dtype, const float* in, void* out, size_t n, hipStream_t s) {
  if (dtype == BF16) hipLaunchKernelGGL(cast_kernel<bf16>, dim3((n + 255) / 256), dim3(256), 0, s, in, (bf16*)out, n);
  else hipLaunchKernelGGL(cast_kernel<float>, dim3((n + 255) / 256), dim3(256), 0, s, in, (float*)out, n);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "cast launch failed");
}

template <typename T>
__global__ void cast_to_f32_kernel(const T* __restrict__ in, float* __restrict__ out, size_t n) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < n) out[i] = to_f<T>(in[i]);
}
int launch_cast_to_f32(int dtype, const void* in, float* out, size_t n, hipStream_t s) {
  if (dtype == BF16) hipLaunchKernelGGL(cast_to_f32_kernel<bf16>, dim3((n + 255) / 256), dim3(256), 0, s, (const bf16*)in, out, n);
  else hipLaunchKernelGGL(cast_to_f32_kernel<float>, dim3((n + 255) / 256), dim3(256), 0, s, (const float*)in, out, n);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "cast launch failed");
}

// bf16 -> OCP E4M3 with a per-tensor scale: the product with 1 / scale is formed in fp32, clamped to the format's
// largest finite value (+-448) and converted by the hardware's round-to-nearest-even conversion; 8 values per thread.
__global__ void __launch_bounds__(256) quantize_fp8_kernel(const bf16* __restrict__ x, int ldx, unsigned char* __restrict__ q, int ldq,
                                                           int rows, int cols, float inv_scale) {
  const size_t i = blockIdx.x * (size_t)256 + threadIdx.x;
  const int per_row = cols / 8;
  if (i >= (size_t)rows * per_row) return;
  const size_t r = i / per_row; const int c = (int)(i % per_row) * 8;
  const bf16x8 v = *reinterpret_cast<const bf16x8*>(x + r * ldx + c);
  float f[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) f[t] = fminf(fmaxf((float)v[t] * inv_scale, -448.0f), 448.0f);
  int lo = 0, hi = 0;
  lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], lo, false);
  lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], lo, true);
  hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], hi, false);
  hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], hi, true);
  u32x2 o = {(uint32_t)lo, (uint32_t)hi};
  *reinterpret_cast<u32x2*>(q + r * ldq + c) = o;
}
int launch_quantize_fp8(const void* x, int ldx, void* q, int ldq, int rows, int cols, float inv_scale, hipStream_t s) {
  if (rows <= 0 || cols <= 0 || !x || !q) return set_error(DP_EINVAL, "quantize_fp8: bad arguments");
  if (cols % 8 || ldx % 8 || ldq % 8 || ldx < cols || ldq < cols) return set_error(DP_EUNSUPPORTED, "quantize_fp8: cols and leading dims must be multiples of 8");
  if (((uintptr_t)x % 16) || ((uintptr_t)q % 8)) return set_error(DP_EALIGN, "quantize_fp8: operands must be 16- / 8-byte aligned");
  if (!(inv_scale > 0.f) || !(inv_scale < INFINITY)) return set_error(DP_EINVAL, "quantize_fp8: the scale must be positive and finite");
  const size_t n = (size_t)rows * (cols / 8);
  if ((n + 255) / 256 > 0x7fffffffull) return set_error(DP_EUNSUPPORTED, "quantize_fp8: tensor too large");
  KScope ks(KK_OTHER, 0.0, 3.0 * (double)rows * cols, s, rows, cols, 0);
  hipLaunchKernelGGL(quantize_fp8_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const bf16*)x, ldx, (unsigned char*)q, ldq, rows, cols, inv_scale);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "quantize_fp8 launch failed");
}

// One wave per token row.  Token ids outside [0, vocab) are clamped (ids live on the device
// and cannot be validated on the host); the sum is rounded once to the storage type.
template <typename T>
__global__ void __launch_bounds__(256) embed_kernel(const int32_t* __restrict__ ids, const T* __restrict__ tok, const T* __restrict__ pos,
                                                    T* __restrict__ x, int rows, int seq, int d, int vocab) {
  constexpr int V = Vec<T>::N;
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  int id = ids[row];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
  const T* t = tok + (size_t)id * d;
  const T* p = pos + (size_t)(row % seq) * d;
  for (int col = lane * V; col < d; col += 64 * V) {
    float a[V], b[V];
    load_vec<T>(t + col, a);
    load_vec<T>(p + col, b);
#pragma unroll
    for (int i = 0; i < V; ++i) a[i] += b[i];
    store_vec<T>(x + (size_t)row * d + col, a);
  }
}
int launch_embed(int dtype, const int32_t* ids, const void* tok, const void* pos, void* x, int rows, int seq, int d, int vocab,
                 hipStream_t s) {
  if (int e = check_vec(dtype, d, "embed")) return e;
  if (rows <= 0 || seq <= 0 || vocab <= 0) return set_error(DP_EINVAL, "embed: bad sizes");
  if (dtype == BF16) hipLaunchKernelGGL(embed_kernel<bf16>, dim3((rows + 3) / 4), dim3(256), 0, s, ids, (const bf16*)tok, (const bf16*)pos, (bf16*)x, rows, seq, d, vocab);
  else hipLaunchKernelGGL(embed_kernel<float>, dim3((rows + 3) / 4), dim3(256), 0, s, ids, (const float*)tok, (const float*)pos, (float*)x, rows, seq, d, vocab);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "embed launch failed");
}

// ---------------------------------------------------------------- batched 16-bit transpose
// dst[c, r] = src[r, c] for up to kTransposeMax dense row-major matrices in one launch (the weight
// matrices of a block, transposed once per backward pass so that dx = dy W runs as y = x W'^T on
// contraction-contiguous operands).  One workgroup moves a 64 x 64 tile through LDS.
__global__ void __launch_bounds__(256) transpose16_batch_kernel(const TransposeBatch tb) {
  __shared__ uint16_t tile[64][66];
  int mi = 0;
  while (mi + 1 < tb.n && (int)blockIdx.x >= tb.tile_start[mi + 1]) ++mi;
  const uint16_t* src = (const uint16_t*)tb.src[mi];
  uint16_t* dst = (uint16_t*)tb.dst[mi];
  const int R = tb.rows[mi], C = tb.cols[mi];
  const int tcols = (C + 63) / 64;
  const int t = blockIdx.x - tb.tile_start[mi];
  const int r0 = (t / tcols) * 64, c0 = (t % tcols) * 64;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int id = threadIdx.x + i * 256, r = id >> 3, c = (id & 7) * 8;
    if (r0 + r < R && c0 + c < C) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(src + (size_t)(r0 + r) * C + c0 + c);
#pragma unroll
      for (int e = 0; e < 4; ++e) { tile[r][c + 2 * e] = (uint16_t)(v[e] & 0xffff); tile[r][c + 2 * e + 1] = (uint16_t)(v[e] >> 16); }
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int id = threadIdx.x + i * 256, c = id >> 3, r = (id & 7) * 8;   // output row c0 + c, output columns r0 + r .. + 7
    if (c0 + c < C && r0 + r < R) {
      u32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = (uint32_t)tile[r + 2 * e][c] | ((uint32_t)tile[r + 2 * e + 1][c] << 16);
      *reinterpret_cast<u32x4*>(dst + (size_t)(c0 + c) * R + r0 + r) = v;
    }
  }
}
int launch_transpose16_batch(const TransposeBatch& tb, hipStream_t s) {
  if (tb.n <= 0 || tb.n > kTransposeMax) return set_error(DP_EINVAL, "transpose: bad matrix count");
  for (int i = 0; i < tb.n; ++i) {
    if (!tb.src[i] || !tb.dst[i] || tb.rows[i] <= 0 || tb.cols[i] <= 0) return set_error(DP_EINVAL, "transpose: bad matrix");
    if ((tb.rows[i] % 8) || (tb.cols[i] % 8)) return set_error(DP_EUNSUPPORTED, "transpose: dims must be multiples of 8");
    if (((uintptr_t)tb.src[i] % 16) || ((uintptr_t)tb.dst[i] % 16)) return set_error(DP_EALIGN, "transpose: operands must be 16-byte aligned");
    const int tiles = ((tb.rows[i] + 63) / 64) * ((tb.cols[i] + 63) / 64);
    if (tb.tile_start[i + 1] - tb.tile_start[i] != tiles || (i == 0 && tb.tile_start[0] != 0))
      return set_error(DP_EINVAL, "transpose: tile table does not match the shapes");
  }
  double bytes = 0.0;
  for (int i = 0; i < tb.n; ++i) bytes += 4.0 * tb.rows[i] * tb.cols[i];
  KScope ks(KK_OTHER, 0.0, bytes, s, tb.n, 0, 0);
  hipLaunchKernelGGL(transpose16_batch_kernel, dim3(tb.tile_start[tb.n]), dim3(256), 0, s, tb);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "transpose launch failed");
}

}  // namespace dp
