// The frozen image encoder as a second non-trainable component (Sec. 2.1; Sec. 2.3: its layers are the
// moderately long and the extra-long non-trainable layers; Sec. 5: such layers run on part of the batch):
// GroupNorm and row-softmax kernels, and the host side of image_encoder_fwd_partial -- layer sequences of
// 3x3 convolutions (implicit GEMM, conv.hip), residual blocks and the single-head attention block, built
// from the library's GEMM kernels.  Channels-last bf16 tensors; statistics and softmax in fp32 / fp64.
#include "../../include/dpipe.h"
#include "dp_device.h"
#include "dp_kernels.h"
#include "dp_errors.h"
#include "dp_host.h"
#include "dp_ktime.h"

#include <cmath>
#include <cstring>

namespace dp {

// ------------------------------------------------------------------ GroupNorm
// Pass 1: every workgroup sums x and x^2 per channel over its share of one sample's pixels.  A thread owns
// one 16-byte piece (8 channels) of every PPB-th pixel; the pixel sub-groups are then added in ascending
// order, so the partial sums do not depend on timing.
constexpr int GN_THREADS = 256;
__global__ void __launch_bounds__(GN_THREADS) gn_partial_kernel(const bf16* __restrict__ x, int HW, int C, int pix_per_block,
                                                                float* __restrict__ partial) {
  __shared__ float red[GN_THREADS * 16];
  const int C8 = C / 8, PPB = GN_THREADS / C8;
  const int tid = threadIdx.x, j = tid % C8, sub = tid / C8;
  const int b = blockIdx.y, p0 = blockIdx.x * pix_per_block, p1 = min(HW, p0 + pix_per_block);
  float s[8], q[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) { s[t] = 0.f; q[t] = 0.f; }
  if (sub < PPB) {
    const bf16* xb = x + (size_t)b * HW * C + j * 8;
    for (int p = p0 + sub; p < p1; p += PPB) {
      const bf16x8 v = *reinterpret_cast<const bf16x8*>(xb + (size_t)p * C);
#pragma unroll
      for (int t = 0; t < 8; ++t) { const float f = (float)v[t]; s[t] += f; q[t] = fmaf(f, f, q[t]); }
    }
  }
#pragma unroll
  for (int t = 0; t < 8; ++t) { red[tid * 16 + t] = s[t]; red[tid * 16 + 8 + t] = q[t]; }
  __syncthreads();
  if (tid < C8) {
    float* o = partial + (((size_t)b * gridDim.x + blockIdx.x) * C + tid * 8) * 2;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      float ss = 0.f, qq = 0.f;
      for (int u = 0; u < PPB; ++u) { ss += red[(u * C8 + tid) * 16 + t]; qq += red[(u * C8 + tid) * 16 + 8 + t]; }
      o[2 * t] = ss; o[2 * t + 1] = qq;
    }
  }
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Pass 2: one workgroup per (sample, group) adds the partial sums of the group's channels over all blocks in
// double precision (thread-strided, a fixed butterfly inside each wave, the four waves in ascending order) and
// writes, per channel, the scale and shift of the normalisation: y = x * ab[0] + ab[1] with
// ab[0] = rstd * gamma, ab[1] = beta - mean * rstd * gamma.  (A single wave per pair left the 256 pairs of an
// 8-sample call with one wave per CU walking up to 64 dependent strided loads each: 12 us on average.)
__global__ void __launch_bounds__(256) gn_finalize_kernel(const float* __restrict__ partial, int nblocks, int HW, int C, int groups,
                                                          float eps, const bf16* __restrict__ gamma, const bf16* __restrict__ beta,
                                                          float* __restrict__ ab, int B) {
  __shared__ double red[2][4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wg = blockIdx.x;
  const int b = wg / groups, g = wg % groups, cpg = C / groups;
  double s = 0.0, q = 0.0;
  const int n = nblocks * cpg;
  for (int i = tid; i < n; i += 256) {
    const int blk = i / cpg, c = g * cpg + i % cpg;
    const float* pp = partial + (((size_t)b * nblocks + blk) * C + c) * 2;
    s += (double)pp[0]; q += (double)pp[1];
  }
  s = wave_sum_f64(s); q = wave_sum_f64(q);
  if (lane == 0) { red[0][wave] = s; red[1][wave] = q; }
  __syncthreads();
  s = ((red[0][0] + red[0][1]) + red[0][2]) + red[0][3];
  q = ((red[1][0] + red[1][1]) + red[1][2]) + red[1][3];
  const double cnt = (double)HW * cpg, mean = s / cnt;
  double var = q / cnt - mean * mean;
  var = var > 0.0 ? var : 0.0;
  const double rstd = 1.0 / sqrt(var + (double)eps);
  for (int c = tid; c < cpg; c += 256) {
    const int ch = g * cpg + c;
    const double a = rstd * (double)(float)gamma[ch];
    ab[((size_t)b * C + ch) * 2] = (float)a;
    ab[((size_t)b * C + ch) * 2 + 1] = (float)((double)(float)beta[ch] - mean * a);
  }
}

// Pass 3: y = x * scale_c + shift_c, then SiLU if asked; 8 channels per thread.
__global__ void __launch_bounds__(256) gn_apply_kernel(const bf16* __restrict__ x, bf16* __restrict__ y, const float* __restrict__ ab,
                                                       size_t HW, int C, size_t total_chunks, int silu) {
  const size_t i = blockIdx.x * (size_t)256 + threadIdx.x;
  if (i >= total_chunks) return;
  const int C8 = C / 8;
  const size_t pix = i / C8; const int c = (int)(i % C8) * 8;
  const size_t b = pix / HW;
  const bf16x8 v = *reinterpret_cast<const bf16x8*>(x + pix * C + c);
  const float* a = ab + (b * C + c) * 2;
  f32x4 a0 = *reinterpret_cast<const f32x4*>(a), a1 = *reinterpret_cast<const f32x4*>(a + 4);
  f32x4 a2 = *reinterpret_cast<const f32x4*>(a + 8), a3 = *reinterpret_cast<const f32x4*>(a + 12);
  const float sc[8] = {a0[0], a0[2], a1[0], a1[2], a2[0], a2[2], a3[0], a3[2]};
  const float sh[8] = {a0[1], a0[3], a1[1], a1[3], a2[1], a2[3], a3[1], a3[3]};
  bf16x8 o;
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    float f = fmaf((float)v[t], sc[t], sh[t]);
    if (silu) f = silu_f(f);
    o[t] = (bf16)f;
  }
  *reinterpret_cast<bf16x8*>(y + pix * C + c) = o;
}

static int gn_blocks(int B, int HW, int C, int* pix_per_block) {
  const int C8 = C / 8, PPB = GN_THREADS / C8;
  // (the block count per sample does not depend on the number of samples: a sample's sums are grouped the same way in every slice)
  long want = std::max<long>(1, std::min<long>(HW / std::max(1, PPB * 4), 256));
  const int ppb = (int)((HW + want - 1) / want);
  if (pix_per_block) *pix_per_block = ppb;
  return (HW + ppb - 1) / ppb;
}

size_t gn_scratch_bytes(int B, int HW, int C) {
  if (B <= 0 || HW <= 0 || C <= 0 || C % 8 || C / 8 > GN_THREADS) return 0;
  return align_up((size_t)B * gn_blocks(B, HW, C, nullptr) * C * 2 * sizeof(float), 256) + (size_t)B * C * 2 * sizeof(float);
}

int launch_groupnorm(const GroupNormArgs& a, hipStream_t s) {
  if (a.dtype != BF16) return set_error(DP_EUNSUPPORTED, "groupnorm: bf16 storage only");
  if (a.B <= 0 || a.HW <= 0 || a.C <= 0 || a.groups <= 0 || !(a.eps > 0.f)) return set_error(DP_EINVAL, "groupnorm: bad sizes");
  if (a.C % 8 || a.C / 8 > GN_THREADS || a.C % a.groups) return set_error(DP_EUNSUPPORTED, "groupnorm: channels must be a multiple of 8 and of the group count, at most 2048");
  if (a.B > 65535) return set_error(DP_EUNSUPPORTED, "groupnorm: more than 65535 samples");
  if (!a.x || !a.y || !a.gamma || !a.beta || !a.scratch) return set_error(DP_EINVAL, "groupnorm: null operand");
  if (((uintptr_t)a.x % 16) || ((uintptr_t)a.y % 16) || ((uintptr_t)a.scratch % 16)) return set_error(DP_EALIGN, "groupnorm: operands must be 16-byte aligned");
  if (a.scratch_bytes < gn_scratch_bytes(a.B, a.HW, a.C)) return set_error(DP_EWORKSPACE, "groupnorm: scratch too small");
  int ppb = 0;
  const int nb = gn_blocks(a.B, a.HW, a.C, &ppb);
  float* partial = a.scratch;
  float* ab = (float*)((char*)a.scratch + align_up((size_t)a.B * nb * a.C * 2 * sizeof(float), 256));
  const double bytes = 2.0 * 2.0 * (double)a.B * a.HW * a.C + 2.0 * (double)a.B * a.HW * a.C;   // x read twice, y written once
  const bool ready = a.ready_partial != nullptr && a.ready_blocks > 0;
  KScope ks(KK_GROUPNORM, 0.0, ready ? bytes - 2.0 * (double)a.B * a.HW * a.C : bytes, s, a.B * a.HW, a.C, a.groups);
  if (!ready) hipLaunchKernelGGL(gn_partial_kernel, dim3(nb, a.B), dim3(GN_THREADS), 0, s, (const bf16*)a.x, a.HW, a.C, ppb, partial);
  hipLaunchKernelGGL(gn_finalize_kernel, dim3(a.B * a.groups), dim3(256), 0, s, ready ? a.ready_partial : partial, ready ? a.ready_blocks : nb,
                     a.HW, a.C, a.groups, a.eps, (const bf16*)a.gamma, (const bf16*)a.beta, ab, a.B);
  const size_t chunks = (size_t)a.B * a.HW * (a.C / 8);
  hipLaunchKernelGGL(gn_apply_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, s, (const bf16*)a.x, (bf16*)a.y, ab, (size_t)a.HW,
                     a.C, chunks, a.silu);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "groupnorm launch failed");
}

// ------------------------------------------------------------------ row softmax (the attention block's probabilities)
// One wave per row of fp32 logits: maximum, sum of exponentials, normalised probabilities in bf16.
__global__ void __launch_bounds__(256) softmax_rows_kernel(const float* __restrict__ s, bf16* __restrict__ p, long rows, int cols, float scale_log2) {
  const int lane = threadIdx.x & 63;
  const long row = blockIdx.x * 4L + (threadIdx.x >> 6);
  if (row >= rows) return;
  const float* sr = s + row * cols;
  bf16* pr = p + row * cols;
  float mx = -INFINITY;
  for (int c = lane * 4; c < cols; c += 256) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(sr + c);
    mx = fmaxf(fmaxf(mx, fmaxf(v[0], v[1])), fmaxf(v[2], v[3]));
  }
  mx = wave_max(mx) * scale_log2;          // the scale is positive: it commutes with the maximum
  float sum = 0.f;
  for (int c = lane * 4; c < cols; c += 256) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(sr + c);
#pragma unroll
    for (int t = 0; t < 4; ++t) sum += __builtin_amdgcn_exp2f(fmaf(v[t], scale_log2, -mx));
  }
  const float inv = 1.0f / wave_sum(sum);
  for (int c = lane * 4; c < cols; c += 256) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(sr + c);
    bf16x4 o;
#pragma unroll
    for (int t = 0; t < 4; ++t) o[t] = (bf16)(__builtin_amdgcn_exp2f(fmaf(v[t], scale_log2, -mx)) * inv);
    *reinterpret_cast<bf16x4*>(pr + c) = o;
  }
}

int launch_softmax_rows(int dtype, const float* s, void* p, long rows, int cols, float scale, hipStream_t st) {
  if (dtype != BF16) return set_error(DP_EUNSUPPORTED, "softmax_rows: bf16 output only");
  if (rows <= 0 || cols <= 0 || cols % 4 || !(scale > 0.f)) return set_error(DP_EINVAL, "softmax_rows: bad sizes (cols must be a multiple of 4, scale positive)");
  if (!s || !p || ((uintptr_t)s % 16) || ((uintptr_t)p % 8)) return set_error(DP_EALIGN, "softmax_rows: null or misaligned operand");
  if ((rows + 3) / 4 > 0x7fffffffL) return set_error(DP_EUNSUPPORTED, "softmax_rows: too many rows");
  KScope ks(KK_SOFTMAX, 0.0, 4.0 * (double)rows * cols + 2.0 * (double)rows * cols, st, (int)rows, cols, 0);
  hipLaunchKernelGGL(softmax_rows_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, s, (bf16*)p, rows, cols, scale * 1.4426950408889634f);
  return hipGetLastError() == hipSuccess ? DP_OK : set_error(DP_EHIP, "softmax_rows launch failed");
}

}  // namespace dp

using namespace dp;

// ============================================================ host side of the component
struct dp_image_encoder {
  dp_image_encoder_desc d;
  std::vector<dp_image_layer> layers;
  std::vector<ParamInfo> params;
  std::vector<int> first_param;          // index of a layer's first parameter
  std::vector<int> h, w, c;              // shape of the output of layer l at index l + 1; index 0 = the input
};

namespace dp {

struct ImgBuf {
  void *ping, *pong, *t1, *t2, *t3, *q, *k, *v, *a, *probs;
  float *scores, *gn; size_t gn_bytes; size_t bytes;
  // GroupNorm partial sums written by the convolution that produced tensor stat_of (stat_blocks blocks of 256 pixels per sample)
  float* gnc; size_t gnc_bytes; const void* stat_of; int stat_blocks;
};

static size_t layer_act_elems(const dp_image_encoder& e, int l, int n) {
  const size_t in_px = (size_t)e.h[l] * e.w[l], out_px = (size_t)e.h[l + 1] * e.w[l + 1];
  const size_t cmax = std::max(e.c[l], e.c[l + 1]);
  return (size_t)n * std::max(in_px, out_px) * cmax;
}

static void plan_image(const dp_image_encoder& e, void* base, int lb, int le, int n, ImgBuf& b) {
  Plan p(base);
  size_t maxact = 0, gn = 0, gnc = 0, attn_rows = 0, attn_px = 0; int attn_c = 0;
  for (int l = lb; l < le; ++l) {
    maxact = std::max(maxact, layer_act_elems(e, l, n));
    gnc = std::max(gnc, (size_t)n * ((size_t)e.h[l + 1] * e.w[l + 1] / 256 + 1) * e.c[l + 1] * 2 * sizeof(float));
    const int HW = e.h[l] * e.w[l];
    if (e.layers[l].kind != DP_IMG_CONV) gn = std::max(gn, std::max(gn_scratch_bytes(n, HW, e.c[l]), gn_scratch_bytes(n, HW, e.c[l + 1])));
    if (e.layers[l].kind == DP_IMG_ATTN) { attn_rows = std::max(attn_rows, (size_t)n * HW); attn_px = std::max(attn_px, (size_t)HW); attn_c = std::max(attn_c, e.c[l]); }
  }
  b.ping = p.take(maxact * 2); b.pong = p.take(maxact * 2); b.t1 = p.take(maxact * 2); b.t2 = p.take(maxact * 2); b.t3 = p.take(maxact * 2);
  b.gn_bytes = gn; b.gn = gn ? (float*)p.take(gn) : nullptr;
  b.gnc_bytes = gnc; b.gnc = (float*)p.take(gnc); b.stat_of = nullptr; b.stat_blocks = 0;
  if (attn_rows) {
    const size_t qb = attn_rows * attn_c * 2;
    b.q = p.take(qb); b.k = p.take(qb); b.v = p.take((size_t)attn_px * attn_c * 2); b.a = p.take(qb);   // v: one sample's values, transposed
    b.scores = (float*)p.take(attn_px * attn_px * 4); b.probs = p.take(attn_px * attn_px * 2);
  } else { b.q = b.k = b.v = b.a = b.probs = nullptr; b.scores = nullptr; }
  b.bytes = p.off;
}

// y = x W^T + bias on M rows.  rows_per_sample > 0: the tile configuration is chosen for one sample's rows, so that the
// arithmetic behind a sample's outputs is the same whatever the number of samples in the call.
static GemmArgs linear(const void* x, long M, int K, const void* W, int N, const void* bias, void* y, int rows_per_sample = 0) {
  GemmArgs g; memset(&g, 0, sizeof(g));
  g.dtype = BF16; g.A = x; g.B = W; g.M = (int)M; g.N = N; g.K = K; g.lda = K; g.ldb = K; g.out = y; g.ldo = N; g.bias = bias;
  if (rows_per_sample > 0) g.force_cfg = 1 + gemm_choose_cfg(rows_per_sample, N, K);
  return g;
}

// One layer on n samples: src [n, H, W, C_in] -> dst [n, Ho, Wo, C_out]; src and dst never alias.
static int image_layer(const dp_image_encoder& e, int l, const void* const* P, const void* src, void* dst, int n, ImgBuf& w, hipStream_t st) {
  const dp_image_layer& L = e.layers[l];
  const int H = e.h[l], W = e.w[l], ci = e.c[l], co = e.c[l + 1], HW = H * W;
  auto conv = [&](const void* x, int cin, int cout, int stride, const void* wt, const void* bias, const void* res, void* y) {
    ConvArgs a; memset(&a, 0, sizeof(a));
    a.dtype = BF16; a.B = n; a.H = H; a.W = W; a.Cin = cin; a.Cout = cout; a.stride = stride; a.x = x; a.w = wt; a.bias = bias; a.residual = res; a.y = y;
    // the convolution's epilogue can produce the first pass of a GroupNorm over its output
    const int out_px = ((H - 1) / stride + 1) * ((W - 1) / stride + 1);
    int applied = 0;
    if (w.gnc && (size_t)n * (out_px / 256 + 1) * cout * 2 * sizeof(float) <= w.gnc_bytes) { a.gn_partial = w.gnc; a.gn_applied = &applied; }
    w.stat_of = nullptr;
    const int rc = launch_conv3x3(a, st);
    if (rc == DP_OK && applied) { w.stat_of = y; w.stat_blocks = out_px / 256; }
    return rc;
  };
  auto gn = [&](const void* x, int ch, const void* gamma, const void* beta, int silu, void* y) {
    GroupNormArgs a; memset(&a, 0, sizeof(a));
    a.dtype = BF16; a.B = n; a.HW = HW; a.C = ch; a.groups = e.d.groups; a.eps = e.d.gn_eps; a.silu = silu;
    a.x = x; a.gamma = gamma; a.beta = beta; a.y = y; a.scratch = w.gn; a.scratch_bytes = w.gn_bytes;
    if (w.stat_of == x && w.stat_blocks > 0) { a.ready_partial = w.gnc; a.ready_blocks = w.stat_blocks; }
    return launch_groupnorm(a, st);
  };
  switch (L.kind) {
    case DP_IMG_CONV:
      return conv(src, ci, co, L.stride, P[0], P[1], nullptr, dst);
    case DP_IMG_NORM_CONV:
      DP_TRY(gn(src, ci, P[0], P[1], 1, w.t1));
      return conv(w.t1, ci, co, 1, P[2], P[3], nullptr, dst);
    case DP_IMG_RESNET: {
      DP_TRY(gn(src, ci, P[0], P[1], 1, w.t1));
      DP_TRY(conv(w.t1, ci, co, 1, P[2], P[3], nullptr, w.t2));
      DP_TRY(gn(w.t2, co, P[4], P[5], 1, w.t1));
      const void* skip = src;
      if (ci != co) {
        DP_TRY(launch_gemm(linear(src, (long)n * HW, ci, P[8], co, P[9], w.t3, HW), st));
        skip = w.t3;
      }
      return conv(w.t1, co, co, 1, P[6], P[7], skip, dst);
    }
    case DP_IMG_ATTN: {
      const long R = (long)n * HW;
      DP_TRY(gn(src, ci, P[0], P[1], 0, w.t1));
      DP_TRY(launch_gemm(linear(w.t1, R, ci, P[2], ci, P[3], w.q, HW), st));
      DP_TRY(launch_gemm(linear(w.t1, R, ci, P[4], ci, P[5], w.k, HW), st));
      const float scale = 1.0f / sqrtf((float)ci);
      for (int s = 0; s < n; ++s) {
        const size_t off = (size_t)s * HW * ci * 2;
        // The values are produced transposed, v^T [c, HW] = W_v h_s^T (the weight as the row operand), so that the
        // product with the probabilities contracts over a contiguous index on both sides.  Their bias is added after
        // the attention instead: every row of the probabilities sums to one, so P (V + 1 b^T) = P V + 1 b^T.
        DP_TRY(launch_gemm(linear(P[6], ci, ci, (const char*)w.t1 + off, HW, nullptr, w.v), st));
        GemmArgs g; memset(&g, 0, sizeof(g));          // scores = q_s k_s^T, fp32
        g.dtype = BF16; g.A = (const char*)w.q + off; g.B = (const char*)w.k + off; g.M = HW; g.N = HW; g.K = ci; g.lda = ci; g.ldb = ci;
        g.out_f32 = w.scores; g.ldo32 = HW;
        DP_TRY(launch_gemm(g, st));
        DP_TRY(launch_softmax_rows(BF16, w.scores, w.probs, HW, HW, scale, st));
        g = linear(w.probs, HW, HW, w.v, ci, P[7], (char*)w.a + off);      // a_s = probs v_s + b_v
        DP_TRY(launch_gemm(g, st));
      }
      GemmArgs g = linear(w.a, R, ci, P[8], ci, P[9], dst, HW);
      g.residual = src; g.ld_res = ci;
      w.stat_of = nullptr;          // dst is written by a GEMM: no statistics come with it
      return launch_gemm(g, st);
    }
    default: return set_error(DP_EINVAL, "unknown image layer kind");
  }
}

static int image_run(const dp_image_encoder& e, const void* const* params, const void* in, void* out, int lb, int le, int off, int n,
                     ImgBuf& w, hipStream_t st, std::vector<hipEvent_t>* ev) {
  const void* cur = (const char*)in + (size_t)off * e.h[lb] * e.w[lb] * e.c[lb] * 2;
  for (int l = lb; l < le; ++l) {
    if (ev && hipEventRecord((*ev)[l - lb], st) != hipSuccess) return set_error(DP_EHIP, "hipEventRecord failed");
    void* dst = (l == le - 1) ? (void*)((char*)out + (size_t)off * e.h[le] * e.w[le] * e.c[le] * 2) : (((l - lb) & 1) ? w.pong : w.ping);
    DP_TRY(image_layer(e, l, params + e.first_param[l], cur, dst, n, w, st));
    cur = dst;
  }
  if (ev && hipEventRecord((*ev)[le - lb], st) != hipSuccess) return set_error(DP_EHIP, "hipEventRecord failed");
  return DP_OK;
}

static int check_image_call(const dp_image_encoder* e, const void* const* params, const void* in, const void* out, int gb, int lb, int le,
                            int off, int n, const void* ws, size_t ws_bytes) {
  if (!e) return set_error(DP_EINVAL, "image encoder handle is NULL");
  if (!params) return set_error(DP_EINVAL, "params is NULL");
  const int nl = (int)e->layers.size();
  if (lb < 0 || le > nl || lb >= le) return set_errorf(DP_EINVAL, "layer range [%d, %d) invalid (0..%d)", lb, le, nl);
  if (gb <= 0 || off < 0 || n < 0 || (long)off + n > gb) return set_errorf(DP_EINVAL, "sample range [%d, %d) outside the global batch of %d", off, off + n, gb);
  for (int i = e->first_param[lb]; i < (le < nl ? e->first_param[le] : (int)e->params.size()); ++i)
    if (int err = check_ptr(params[i], e->params[i].name.c_str())) return err;
  DP_TRY(check_ptr(in, "input tensor")); DP_TRY(check_ptr(out, "output tensor")); DP_TRY(check_ptr(ws, "workspace", 256));
  if (in == out) return set_error(DP_EINVAL, "input and output tensors must differ");
  const size_t need = dp_image_encoder_workspace_bytes(e, lb, le, n);
  if (ws_bytes < need) return set_errorf(DP_EWORKSPACE, "workspace too small: %zu bytes given, %zu needed", ws_bytes, need);
  return DP_OK;
}

}  // namespace dp

extern "C" {

int dp_image_encoder_create(const dp_image_encoder_desc* desc, const dp_image_layer* layers, dp_image_encoder** out) {
  if (!desc || !layers || !out) return set_error(DP_EINVAL, "dp_image_encoder_create: NULL argument");
  const dp_image_encoder_desc& d = *desc;
  if (d.dtype != DP_BF16) return set_error(d.dtype == DP_F32 ? DP_EUNSUPPORTED : DP_EINVAL, "image encoder: bf16 storage only");
  if (d.height <= 0 || d.width <= 0 || d.in_ch <= 0 || d.groups <= 0 || d.n_layers <= 0) return set_error(DP_EINVAL, "sizes must be positive");
  if (d.n_layers > 4096 || (long)d.height * d.width > (1L << 26)) return set_error(DP_EUNSUPPORTED, "too many layers or pixels");
  if (!(d.gn_eps > 0.f)) return set_error(DP_EINVAL, "gn_eps must be positive");
  if (d.in_ch % 8) return set_error(DP_EUNSUPPORTED, "in_ch must be a multiple of 8 (pad the image with zero channels)");
  dp_image_encoder* e = new (std::nothrow) dp_image_encoder();
  if (!e) return set_error(DP_EINVAL, "out of host memory");
  int rc = DP_OK;
  try {
    e->d = d;
    e->h.push_back(d.height); e->w.push_back(d.width); e->c.push_back(d.in_ch);
    for (int l = 0; l < d.n_layers && rc == DP_OK; ++l) {
      const dp_image_layer& L = layers[l];
      const int ci = e->c.back(), H = e->h.back(), W = e->w.back();
      if (L.c_in != ci) rc = set_errorf(DP_EINVAL, "layer %d: c_in %d does not match the %d channels it receives", l, L.c_in, ci);
      else if (L.c_out <= 0 || L.c_out % 8 || L.c_out > 2048) rc = set_errorf(DP_EUNSUPPORTED, "layer %d: c_out must be a positive multiple of 8, at most 2048", l);
      else if (L.kind < DP_IMG_CONV || L.kind > DP_IMG_NORM_CONV) rc = set_errorf(DP_EINVAL, "layer %d: unknown kind", l);
      else if (L.kind == DP_IMG_CONV ? (L.stride != 1 && L.stride != 2) : L.stride != 1) rc = set_errorf(DP_EINVAL, "layer %d: stride must be 1 (2 allowed for a plain convolution)", l);
      else if (L.kind == DP_IMG_ATTN && L.c_out != ci) rc = set_errorf(DP_EINVAL, "layer %d: the attention block keeps the channel count", l);
      else if (L.kind != DP_IMG_CONV && (ci % d.groups || (L.kind == DP_IMG_RESNET && L.c_out % d.groups))) rc = set_errorf(DP_EINVAL, "layer %d: channels must be a multiple of the group count", l);
      else if (L.kind == DP_IMG_ATTN && ((long)H * W % 8 || (long)H * W > 65536)) rc = set_errorf(DP_EUNSUPPORTED, "layer %d: the attention block needs a pixel count that is a multiple of 8, at most 65536", l);
      if (rc != DP_OK) break;
      e->layers.push_back(L);
      e->first_param.push_back((int)e->params.size());
      const std::string pre = "layer" + std::to_string(l) + ".";
      const int64_t co = L.c_out;
      auto add = [&](const char* n, int64_t r, int64_t c) { e->params.push_back({pre + n, r, c}); };
      switch (L.kind) {
        case DP_IMG_CONV: add("w", co, 9 * ci); add("b", co, 0); break;
        case DP_IMG_RESNET:
          add("norm1_g", ci, 0); add("norm1_b", ci, 0); add("conv1_w", co, 9 * ci); add("conv1_b", co, 0);
          add("norm2_g", co, 0); add("norm2_b", co, 0); add("conv2_w", co, 9 * co); add("conv2_b", co, 0);
          if (ci != co) { add("skip_w", co, ci); add("skip_b", co, 0); }
          break;
        case DP_IMG_ATTN:
          add("norm_g", ci, 0); add("norm_b", ci, 0);
          for (const char* n : {"q", "k", "v", "proj"}) { add((std::string(n) + "_w").c_str(), ci, ci); add((std::string(n) + "_b").c_str(), ci, 0); }
          break;
        default: add("norm_g", ci, 0); add("norm_b", ci, 0); add("w", co, 9 * ci); add("b", co, 0); break;
      }
      const int s = L.kind == DP_IMG_CONV ? L.stride : 1;
      e->h.push_back((H - 1) / s + 1); e->w.push_back((W - 1) / s + 1); e->c.push_back(L.c_out);
    }
  } catch (...) {
    rc = set_error(DP_EINVAL, "dp_image_encoder_create: out of host memory");
  }
  if (rc != DP_OK) { delete e; return rc; }
  *out = e;
  return DP_OK;
}

void dp_image_encoder_destroy(dp_image_encoder* enc) { delete enc; }
int dp_image_encoder_param_count(const dp_image_encoder* enc) { return enc ? (int)enc->params.size() : set_error(DP_EINVAL, "image encoder handle is NULL"); }
int dp_image_encoder_param_shape(const dp_image_encoder* enc, int idx, int64_t shape[2], const char** name) {
  if (!enc || !shape) return set_error(DP_EINVAL, "dp_image_encoder_param_shape: NULL argument");
  if (idx < 0 || idx >= (int)enc->params.size()) return set_error(DP_EINVAL, "parameter index out of range");
  shape[0] = enc->params[idx].rows; shape[1] = enc->params[idx].cols;
  if (name) *name = enc->params[idx].name.c_str();
  return DP_OK;
}
int dp_image_encoder_layer_shape(const dp_image_encoder* enc, int layer, int64_t hwc[3]) {
  if (!enc || !hwc) return set_error(DP_EINVAL, "dp_image_encoder_layer_shape: NULL argument");
  if (layer < -1 || layer >= (int)enc->layers.size()) return set_error(DP_EINVAL, "layer index out of range");
  hwc[0] = enc->h[layer + 1]; hwc[1] = enc->w[layer + 1]; hwc[2] = enc->c[layer + 1];
  return DP_OK;
}
size_t dp_image_encoder_workspace_bytes(const dp_image_encoder* enc, int layer_begin, int layer_end, int max_samples) {
  if (!enc || max_samples <= 0 || layer_begin < 0 || layer_end > (int)enc->layers.size() || layer_begin >= layer_end) return 0;
  ImgBuf b;
  plan_image(*enc, nullptr, layer_begin, layer_end, max_samples, b);
  return b.bytes;
}

int image_encoder_fwd_partial(dp_image_encoder* enc, const void* const* params, const void* in, void* out, int global_batch,
                              int layer_begin, int layer_end, int sample_offset, int num_samples, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  DP_TRY(check_image_call(enc, params, in, out, global_batch, layer_begin, layer_end, sample_offset, num_samples, workspace, workspace_bytes));
  if (num_samples == 0) return DP_OK;
  ImgBuf w;
  plan_image(*enc, workspace, layer_begin, layer_end, num_samples, w);
  return image_run(*enc, params, in, out, layer_begin, layer_end, sample_offset, num_samples, w, (hipStream_t)hip_stream, nullptr);
}

int dp_image_encoder_profile(dp_image_encoder* enc, const void* const* params, const void* in, void* out, int global_batch,
                             const int* batches, int n_batches, int reps, void* workspace, size_t workspace_bytes,
                             dp_layer_cost* rows, int max_rows, int* n_rows, void* hip_stream) {
  if (!enc || !batches || !rows || !n_rows || n_batches <= 0 || reps < 1) return set_error(DP_EINVAL, "dp_image_encoder_profile: bad argument");
  const int nl = (int)enc->layers.size();
  if (max_rows < nl * n_batches) return set_error(DP_EINVAL, "dp_image_encoder_profile: too few rows");
  for (int i = 0; i < n_batches; ++i) {
    if (batches[i] < 1) return set_error(DP_EINVAL, "dp_image_encoder_profile: batch sizes must be positive");
    DP_TRY(check_image_call(enc, params, in, out, global_batch, 0, nl, 0, batches[i], workspace, workspace_bytes));
  }
  hipStream_t s = (hipStream_t)hip_stream;
  std::vector<hipEvent_t> ev;
  int rc = DP_OK, nout = 0;
  try {
    for (int i = 0; i <= nl && rc == DP_OK; ++i) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) rc = set_error(DP_EHIP, "hipEventCreate failed");
      else ev.push_back(e);
    }
    for (int bi = 0; bi < n_batches && rc == DP_OK; ++bi) {
      const int n = batches[bi];
      ImgBuf w;
      plan_image(*enc, workspace, 0, nl, n, w);
      std::vector<std::vector<float>> t(nl);
      for (int r = 0; r < reps && rc == DP_OK; ++r) {
        rc = image_run(*enc, params, in, out, 0, nl, 0, n, w, s, &ev);
        if (rc == DP_OK && hipStreamSynchronize(s) != hipSuccess) rc = set_error(DP_EHIP, "hipStreamSynchronize failed");
        for (int l = 0; l < nl && rc == DP_OK; ++l) {
          float ms = 0.f;
          if (hipEventElapsedTime(&ms, ev[l], ev[l + 1]) != hipSuccess) rc = set_error(DP_EHIP, "hipEventElapsedTime failed");
          t[l].push_back(ms);
        }
      }
      for (int l = 0; l < nl && rc == DP_OK; ++l) {
        const int64_t act = (int64_t)n * enc->h[l + 1] * enc->w[l + 1] * enc->c[l + 1] * 2;
        rows[nout++] = dp_layer_cost{2, l, n, median(t[l]), 0.f, act, act, 0, 0};
      }
    }
  } catch (...) {
    rc = set_error(DP_EINVAL, "dp_image_encoder_profile: out of host memory");
  }
  for (auto& e : ev) (void)hipEventDestroy(e);
  if (rc != DP_OK) return rc;
  *n_rows = nout;
  return DP_OK;
}

}  // extern "C"
