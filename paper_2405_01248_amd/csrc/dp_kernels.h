// Host-side launch interface of the kernels (internal to the library).
// Every launcher validates its operand shapes on the host before the launch and
// returns a negative dpipe error code instead of launching when they do not fit.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace dp {

enum DType { F32 = 0, BF16 = 1 };
inline size_t dtype_size(int dt) { return dt == BF16 ? 2 : 4; }

// ---------------------------------------------------------------- GEMM
// C[M,N] = opA(A) * opB(B) with fp32 accumulation.
//   a_mc = 0: A stored [M,K] (contraction index contiguous); 1: A stored [K,M].
//   b_mc = 0: B stored [N,K] (a weight used as y = x W^T);   1: B stored [K,N].
// Epilogue, in this order, all optional:
//   v = acc + bias[n]; if (pre_out) pre_out[m,n] = v; v = act(v);
//   if (dact_pre) v *= act'(dact_pre[m,n]); if (gate) v *= gate[(m / rows_per_batch) * gate_ld + n];
//   if (residual) v += residual[m,n]; out[m,n] = v  (storage dtype, or fp32 if out_fused_f32)
// or, when out_f32 is set, the raw product goes to fp32:
//   out_f32[m,n] = (accumulate ? out_f32[m,n] : 0) + acc   (split-K partial sums are
//   reduced in a fixed order through `splitk_ws`, so results are run-to-run identical).
struct GemmArgs {
  int dtype;                 // storage dtype of A, B, out, bias, residual, pre_out, dact_pre, gate
  const void* A; const void* B;
  int M, N, K;
  int lda, ldb;              // row strides in elements
  int a_mc, b_mc;
  void* out; int ldo;        // storage-dtype output (or nullptr)
  float* out_f32; int ldo32; int accumulate;
  const void* bias;
  void* pre_out; int ld_pre;
  int act;
  const void* dact_pre; int ld_dact; int dact_kind;
  const void* gate; int gate_ld; int rows_per_batch;
  const void* residual; int ld_res;
  int residual_f32;          // residual is fp32 (the residual stream) although dtype is bf16
  int out_fused_f32;         // `out` receives the fused-epilogue result as fp32 instead of the storage dtype
  float* splitk_ws; size_t splitk_ws_bytes;
  // with out_f32 and a_mc (a weight gradient dy^T x): also colsum_out[m] = (accumulate ? old : 0) + sum_k A[k, m], the
  // bias gradient, from the tiles the kernel stages anyway.  Only where gemm_colsum_supported() says so.
  float* colsum_out;
  int force_cfg;             // 0 = choose by shape; 1 + index forces a tile configuration (measurement only)
  int choice_rows;           // > 0: tile configuration and split-K factor are chosen as if the problem had this many rows
                             // (a caller whose rows are independent samples gets the same arithmetic per row for any M);
                             // < 0: the same guarantee by other means: no split-K and 32x32x16 tiles only, shape chosen from M
  // GeGLU fused into the epilogue (bf16 only; bias is the only other epilogue term allowed):
  //   geglu = 1 (forward): B [2 * geglu_inner, K] and bias are the [value | gate] projection, N = 2 * geglu_inner.
  //     pre_out [M, N] (optional) receives the projection u, out [M, geglu_inner] = value * gelu(gate), both taken
  //     from u as rounded to the storage dtype.  Needs gemm_geglu_fwd_supported().
  //   geglu = 2 (backward): N = geglu_inner, the product is dg; out [M, 2 * geglu_inner] =
  //     [dg * gelu(gate) | dg * value * gelu'(gate)] with value / gate read from geglu_u [M, 2 * geglu_inner].
  int geglu, geglu_inner;
  const void* geglu_u; int ld_geglu;
  // LayerNorm of the result rows folded into the split-K reduction pass (bf16, fp32 residual stream updated
  // in place: out == residual, out_fused_f32, dense rows, bias optional, nothing else in the epilogue).  Only
  // when the GEMM happens to be split along K: *ln_applied (must be given with ln_out) is then set to 1 and
  // ln_out [M, N] holds LN(out; ln_gamma, ln_beta, ln_eps) in the storage dtype; otherwise it is set to 0 and
  // the caller runs the LayerNorm itself.
  const void* ln_gamma; const void* ln_beta; void* ln_out; float ln_eps; int* ln_applied;
};
int launch_gemm(const GemmArgs& a, hipStream_t s);
// Index (as force_cfg - 1) of the tile configuration launch_gemm would choose for y = x W^T with M rows, contraction-contiguous bf16 operands.
int gemm_choose_cfg(int M, int N, int K);
bool gemm_geglu_fwd_supported(const GemmArgs& a);
bool gemm_colsum_supported(const GemmArgs& a);
size_t gemm_splitk_ws_bytes(int M, int N, int K);   // upper bound for out_f32 GEMMs
size_t gemm_epi_splitk_ws_bytes(int M, int N, int K);   // same for storage-dtype outputs (0: such a GEMM is never split)
size_t gemm_epi_splitk_ws_bytes_for(int M, int N, int K, int choice_rows);   // with GemmArgs::choice_rows

// ---------------------------------------------------------------- FP8 (OCP E4M3) projection GEMM
// q[i, j] = e4m3(clamp(x[i, j] * inv_scale, -448, 448)), round to nearest even; x [rows, cols] in bf16 (row stride ldx
// elements), q bytes (row stride ldq).  cols a multiple of 8.
int launch_quantize_fp8(const void* x, int ldx, void* q, int ldq, int rows, int cols, float inv_scale, hipStream_t s);
// out[M, N] (bf16) = out_scale * sum_k A[m, k] B[n, k] (+ bias[n]) for E4M3 operands A [M, K], B [N, K] (row strides in
// bytes), fp32 accumulation on v_mfma_f32_32x32x64_f8f6f4.  K a multiple of 128, N of 8.
struct Fp8GemmArgs {
  const void* A; int lda; const void* B; int ldb; int M, N, K; float out_scale; const void* bias; void* out; int ldo;
};
int launch_gemm_fp8(const Fp8GemmArgs& a, hipStream_t s);

// ---------------------------------------------------------------- convolution (frozen image encoder)
// y[b, i, j, :] = sum_{u, v} x[b, i * stride + u - 1, j * stride + v - 1, :] w[:, 3u + v, :]^T + bias (+ residual),
// zero padding 1.  Channels-last bf16 tensors: x [B, H, W, Cin], w [Cout, 9 * Cin] (taps row-major, channels
// last), y and residual [B, Ho, Wo, Cout] with Ho = (H - 1) / stride + 1.  Cin, Cout multiples of 8.
struct ConvArgs {
  int dtype;
  int B, H, W, Cin, Cout, stride;
  const void* x; const void* w; const void* bias; const void* residual; void* y;
  int force_staged;   // 1: always the register-staged kernel (measurement and tests of that path)
  // Optional: per-channel sums and sums of squares of the output (as rounded to bf16) per block of 256 output pixels, in
  // the layout of GroupNorm's first pass, gn_partial[((b * (HoWo / 256) + block) * Cout + c) * 2 + {0, 1}], so that a
  // GroupNorm of y can skip that pass.  Only when Ho * Wo is a multiple of 256 and the direct-to-LDS kernel runs:
  // *gn_applied (required with gn_partial) tells whether they were written.
  float* gn_partial; int* gn_applied;
};
int launch_conv3x3(const ConvArgs& a, hipStream_t s);

// GroupNorm over channels-last x [B, HW, C]: per (sample, group of C / groups consecutive channels) mean and
// biased variance over the group's channels at all pixels; y = (x - mean) * rstd * gamma + beta, then SiLU
// if silu != 0.  Three launches: per-block partial sums, their fixed-order combination (in double) into a
// per-(sample, channel) scale and shift, and the elementwise pass.  scratch: fp32, gn_scratch_bytes().
struct GroupNormArgs {
  int dtype;
  int B, HW, C, groups; float eps; int silu;
  const void* x; const void* gamma; const void* beta; void* y;
  float* scratch; size_t scratch_bytes;
  // partial sums already produced by the convolution that wrote x (ConvArgs::gn_partial): ready_blocks blocks per sample
  const float* ready_partial; int ready_blocks;
};
size_t gn_scratch_bytes(int B, int HW, int C);
int launch_groupnorm(const GroupNormArgs& a, hipStream_t s);

// p[r, :] = softmax(scale * s[r, :]) for fp32 logits s [rows, cols] (dense), written in the storage dtype.
int launch_softmax_rows(int dtype, const float* s, void* p, long rows, int cols, float scale, hipStream_t st);

// ---------------------------------------------------------------- attention
// Per (batch b, head h): O = softmax(Q K^T * scale [+ causal mask]) V.
// Element (b, n, h, t) of X lives at X + (b * rows_X + n) * ld_X + h * d_head + t, so Q/K/V
// may be column blocks of a fused projection output.  lse is [B, H, Nq] fp32 (natural log).
struct AttnArgs {
  int dtype;
  int B, H, Nq, Nk, d_head;
  int causal;
  float scale;
  const void* q; int ldq;
  const void* k; int ldk;
  const void* v; int ldv;
  void* o; int ldo;
  float* lse;               // may be nullptr in forward when nothing is saved
  // backward only
  const void* dout; int lddo;
  float* delta;             // [B,H,Nq] scratch: rowsum(dO * O)
  void* dq; int lddq;
  void* dk; int lddk;
  void* dv; int lddv;
  float* dkv_ws; size_t dkv_ws_bytes;   // optional fp32 scratch: lets the dK/dV kernel split the query range when there are few key tiles
};
size_t attn_dkv_ws_bytes(int B, int H, int Nk, int d_head);   // enough for any split the launcher may choose
int launch_attn_fwd(const AttnArgs& a, hipStream_t s);
int launch_attn_bwd(const AttnArgs& a, hipStream_t s);

// ---------------------------------------------------------------- norm / elementwise
// LayerNorm over the last dim of x [rows, d]; gamma/beta (storage dtype) may be null.
// If scale/shift are given (per batch, row b of a [B, mod_ld] matrix; batch = row / rows_per_batch)
// the output is xhat * (1 + scale) + shift.  mean/rstd (fp32 [rows]) may be null.
struct LnArgs {
  int dtype; int rows, d; float eps;
  const void* x; int x_f32;     // x_f32: x is fp32 (the residual stream) although dtype is bf16
  void* y;
  const void* gamma; const void* beta;
  const void* scale; const void* shift; int mod_ld; int rows_per_batch;
  float* mean; float* rstd;
  float* x32_out;               // optional, storage-dtype x only: the rows of x widened to fp32 (the stage input entering the fp32 residual stream)
};
int launch_ln_fwd(const LnArgs& a, hipStream_t s);
// x[r, :] += sum_z partial[z][r, :] (+ bias), then y[r, :] = LN(x[r, :]; gamma, beta, eps) in bf16: the split-K
// reduction of a projection onto the fp32 residual stream and the LayerNorm that follows it, one wave per row.
// partial: [splits][rows][d] fp32; d a multiple of 8, at most 2048.
int launch_reduce_residual_ln(const float* partial, int splits, int rows, int d, const void* bias, float* x, void* y,
                              const void* gamma, const void* beta, float eps, hipStream_t s);

// dx = [dres +] LN backward of dy.  x (the LayerNorm input) and dres are fp32 residual-stream
// tensors; the result is written to dx32 (fp32) and/or dx (storage dtype).  Affine: dgamma/dbeta (fp32 [d], accumulate flag).
// Modulated: dscale/dshift rows written to fp32 [B, dmod_ld] (overwrite) and the
// effective gain is (1 + scale).  partial is scratch of ln_bwd_partial_bytes().
struct LnBwdArgs {
  int dtype; int rows, d;
  const void* dy; const void* x; const float* mean; const float* rstd;
  const void* gamma;
  const void* scale; int mod_ld; int rows_per_batch;
  const void* dres;        // optional residual-stream gradient added to dx: fp32, or the storage dtype if dres_storage
  int dres_storage;
  void* dx; float* dx32;
  float* dgamma; float* dbeta; int accumulate;
  float* dscale; float* dshift; int dmod_ld;
  float* partial; size_t partial_bytes;
  int defer_reduce;        // 1: only write the column partials; the caller runs launch_ln_bwd_reduce (maybe on another stream)
};
int launch_ln_bwd(const LnBwdArgs& a, hipStream_t s);
int launch_ln_bwd_reduce(const LnBwdArgs& a, hipStream_t s);
size_t ln_bwd_partial_bytes(int rows, int d, int rows_per_batch);

// g[m, j] = u[m, j] * gelu_erf(u[m, inner + j])
int launch_geglu_fwd(int dtype, const void* u, void* g, int rows, int inner, hipStream_t s);
// du[m, j] = dg * gelu(gate); du[m, inner + j] = dg * val * gelu'(gate)
int launch_geglu_bwd(int dtype, const void* dg, const void* u, void* du, int rows, int inner, hipStream_t s);

// out[n] = (accumulate ? out[n] : 0) + sum_m x[m, n]   (fp32 out; deterministic two-stage)
int launch_colsum(int dtype, const void* x, int ldx, int rows, int cols, float* out, int accumulate,
                  float* partial, size_t partial_bytes, hipStream_t s);
size_t colsum_partial_bytes(int rows, int cols);

// out[i] = (accumulate ? out[i] : 0) + sum_z partial[z * n + i]
int launch_reduce_partials(const float* partial, int nz, size_t n, float* out, int accumulate, hipStream_t s);
// the same for two tensors in one launch (the second may be absent: n_b = 0)
int launch_reduce_partials2(const float* partial, int nz, size_t n, float* out, const float* partial_b, size_t n_b, float* out_b,
                            int accumulate, hipStream_t s);

// y = silu(x) elementwise (storage dtype), n elements
int launch_silu(int dtype, const void* x, void* y, size_t n, hipStream_t s);
// dc[i] (+)= dsilu_in[i] * silu'(c[i])   (fp32 in, storage-dtype c, fp32 out)
int launch_silu_bwd(int dtype, const float* dz, const void* c, float* dc, int accumulate, size_t n, hipStream_t s);

// Gated-branch backward helper (dres is the fp32 residual-stream gradient): dbranch[m,n] = dres[m,n] * gate[b,n];
// dgate[b,n] = sum_{rows of batch b} dres[m,n] * branch[m,n]   (fp32, overwrite)
int launch_gate_bwd(int dtype, const void* dres, const void* branch, const void* gate, int gate_ld,
                    void* dbranch, float* dgate, int dgate_ld, int B, int rows_per_batch, int d, hipStream_t s);

// storage dtype -> fp32
int launch_cast_to_f32(int dtype, const void* in, float* out, size_t n, hipStream_t s);
// fp32 [rows, cols] -> storage dtype
int launch_cast_from_f32(int dtype, const float* in, void* out, size_t n, hipStream_t s);

// x[row, :] = tok[ids[row], :] + pos[row % seq, :]
int launch_embed(int dtype, const int32_t* ids, const void* tok, const void* pos, void* x, int rows, int seq,
                 int d, int vocab, hipStream_t s);

// dst[c, r] = src[r, c] for up to kTransposeMax dense row-major 16-bit matrices in one launch.
// tile_start[i] is the number of 64 x 64 tiles of the matrices before matrix i (tile_start[n] = total).
constexpr int kTransposeMax = 16;
struct TransposeBatch {
  int n;
  const void* src[kTransposeMax]; void* dst[kTransposeMax];
  int rows[kTransposeMax], cols[kTransposeMax];
  int tile_start[kTransposeMax + 1];
};
inline void transpose_batch_add(TransposeBatch& tb, const void* src, void* dst, int rows, int cols) {
  const int i = tb.n++;
  tb.src[i] = src; tb.dst[i] = dst; tb.rows[i] = rows; tb.cols[i] = cols;
  if (i == 0) tb.tile_start[0] = 0;
  tb.tile_start[i + 1] = tb.tile_start[i] + ((rows + 63) / 64) * ((cols + 63) / 64);
}
int launch_transpose16_batch(const TransposeBatch& tb, hipStream_t s);

}  // namespace dp
