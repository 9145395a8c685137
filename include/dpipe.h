/*
 * dpipe -- C ABI of the stage-compute hot path for MI355X (gfx950).
 *
 * What it computes: the per-micro-batch work of ONE pipeline stage of a diffusion
 * backbone -- the forward and backward of a contiguous range of transformer blocks
 * (the quantity sum_l P^f_l + sum_l P^b_l that defines a stage's time T_0(s), Sec. 4.1,
 * equation for T_0) -- the additional no-grad forward of self-conditioning (Sec. 4.3,
 * equation for T_{0,SC}: 2 sum P^f + sum P^b), and the frozen text encoder's forward on
 * a partial batch (Sec. 5: partial-batch layer (component, layer, #samples); input split
 * and output concatenation across pipeline bubbles), plus the per-layer timing export in
 * the cost-profile form the partitioner consumes (Table "Notations": P^f_l(B), P^b_l(B),
 * C^f, C^b, G_l, O_l).
 *
 * Conventions
 *  - Every pointer marked [device] is HIP device memory owned by the caller; stage_fwd,
 *    stage_bwd and encoder_fwd_partial never allocate or free device memory and never
 *    synchronise (the first call that uses the side stream, see dp_stage_set_overlap, creates
 *    that stream and a pool of events: host objects, released by dp_stage_destroy).  `params` / `dparams` are HOST arrays of device pointers.
 *  - `hip_stream` is a hipStream_t passed as void*; all work is enqueued on it in order.
 *  - Tensors are row-major with the last dimension contiguous.  Storage dtype is the
 *    descriptor's dtype (bf16 or fp32); parameter gradients are always fp32.
 *  - Weights are [out_features, in_features] (y = x W^T).
 *  - Every function returns DP_OK (0) or a negative error code; nothing throws or aborts.
 *    Invalid descriptors, NULL or misaligned pointers (16 bytes), too-small workspaces and
 *    unsupported shapes are rejected on the host before anything is launched.
 *    dp_last_error() gives the calling thread's last message.
 */
#ifndef DPIPE_H
#define DPIPE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dp_stage dp_stage;     /* opaque, host memory */
typedef struct dp_encoder dp_encoder; /* opaque, host memory */

enum { DP_OK = 0, DP_EINVAL = -1, DP_EUNSUPPORTED = -2, DP_EWORKSPACE = -3, DP_EALIGN = -4, DP_EHIP = -5 };
enum dp_block_kind { DP_BLOCK_UNET_XATTN_GEGLU = 0, DP_BLOCK_DIT_ADALN_ZERO = 1 };
enum dp_dtype { DP_F32 = 0, DP_BF16 = 1 };

/* A stage = n_blocks identical transformer blocks on a micro-batch of `batch` samples
 * with `tokens` tokens of width d_model = n_heads * d_head.
 *  DP_BLOCK_UNET_XATTN_GEGLU: pre-LN self-attention (no q/k/v bias), pre-LN cross-attention
 *    to ctx [batch, ctx_tokens, ctx_dim] (frozen text-encoder states, Sec. 2.1; no gradient
 *    to ctx), pre-LN GeGLU feed-forward with hidden width ff_inner (value half first, erf GELU).
 *  DP_BLOCK_DIT_ADALN_ZERO: (shift,scale,gate)x2 = Linear(SiLU(cond)); modulated non-affine LN;
 *    self-attention and a GELU MLP of width ff_inner, each gated into the residual.
 *    gelu_tanh selects the tanh approximation.  ctx_tokens / ctx_dim are ignored.
 * bf16 limits: d_model, ctx_dim, ff_inner multiples of 8; d_head multiple of 8, <= 96;
 * d_model <= 2048.  fp32 limits: multiples of 4, d_model <= 1024, tokens <= 7500. */
typedef struct {
  int kind, dtype, n_blocks, batch, tokens, d_model, n_heads, d_head, ctx_tokens, ctx_dim, ff_inner;
  float ln_eps;
  int gelu_tanh;
} dp_stage_desc;

/* Validates desc and creates a host-side handle.  *out is untouched on error. */
int dp_stage_create(const dp_stage_desc* desc, dp_stage** out);
void dp_stage_destroy(dp_stage* st);

/* Parameters are passed as a flat array in a fixed order: block 0's tensors, block 1's, ...
 * U-Net block (17): ln1_g ln1_b attn1_wqkv[3d,d] attn1_wo attn1_bo ln2_g ln2_b attn2_wq
 *   attn2_wkv[2d,ctx_dim] attn2_wo attn2_bo ln3_g ln3_b ff_w1[2*inner,d] ff_b1 ff_w2[d,inner] ff_b2
 * DiT block (10): ada_w[6d,d] ada_b attn_wqkv[3d,d] attn_bqkv attn_wo attn_bo fc1_w fc1_b fc2_w fc2_b
 * dp_stage_param_shape: shape[1] = 0 for vectors; *name points to static storage
 * ("block<i>.<tensor>"). */
int dp_stage_param_count(const dp_stage* st);
int dp_stage_param_shape(const dp_stage* st, int idx, int64_t shape[2], const char** name);

/* stage_bwd runs the weight- and bias-gradient kernels and the per-call weight transposes (all off the
 * critical path) on a second, library-owned stream forked from and joined to hip_stream with events,
 * so that they overlap the activation-gradient chain; a saving stage_fwd of U-Net blocks runs the
 * context K/V projections of all blocks there.  enabled = 0 issues everything on hip_stream in program order
 * (used when single kernels are to be timed); results are bit-identical either way.  Default 1. */
int dp_stage_set_overlap(dp_stage* st, int enabled);

/* Epilogue fusions of the U-Net block's GeGLU feed-forward (bf16 stages; the fp32 path never fuses).
 * mask bit 0: the gated activation is applied in the epilogue of the projection GEMM (forward);
 * bit 1: its backward is applied in the epilogue of the activation-gradient GEMM of the second
 * feed-forward layer, whose raw product then never reaches memory.  Unfused, the same arithmetic
 * runs as separate elementwise kernels; forward results are bit-identical, backward results
 * differ by the rounding of the raw product to bf16 that the fused path skips.  Default 3. */
int dp_stage_set_fusion(dp_stage* st, int mask);

/* Bytes of caller-provided workspace [device].  save_for_bwd = 1: saved activations of all
 * blocks plus backward scratch (pass the same workspace to stage_bwd).  0: scratch for a
 * forward that keeps nothing (the self-conditioning pass).  The workspace must be
 * 256-byte aligned. */
size_t dp_stage_workspace_bytes(const dp_stage* st, int save_for_bwd);

/* y = blocks(x).  x, y [device]: [batch, tokens, d_model].  ctx_or_cond [device]:
 * ctx [batch, ctx_tokens, ctx_dim] (U-Net) or cond [batch, d_model] (DiT).
 * save_for_bwd = 0 is the extra forward of self-conditioning (Sec. 4.3): it touches only
 * the workspace it is given, so it may run between another workspace's forward and backward. */
int stage_fwd(dp_stage* st, const void* const* params, const void* x, const void* ctx_or_cond, void* y,
              void* workspace, size_t workspace_bytes, int save_for_bwd, void* hip_stream);

/* Backward of the last stage_fwd(save_for_bwd = 1) on this workspace.  dy, dx [device]:
 * [batch, tokens, d_model].  d_cond [device]: fp32 [batch, d_model], DiT only (else NULL),
 * overwritten with the sum over blocks.  dparams: host array of fp32 device buffers, one per
 * parameter, same order and shapes; accumulate = 1 adds to them (micro-batch accumulation
 * before the pipeline flush), 0 overwrites. */
int stage_bwd(dp_stage* st, const void* const* params, const void* dy, const void* ctx_or_cond, void* dx,
              void* d_cond, void* const* dparams, int accumulate, void* workspace, size_t workspace_bytes,
              void* hip_stream);

/* Frozen text encoder (Sec. 2.1), forward only.  Pre-LN causal (causal = 1) transformer,
 * biases on every projection, quick-GELU MLP, final LayerNorm.
 * Parameter order: tok_emb[vocab,d] pos_emb[seq,d], then per layer (12 tensors): ln1_g ln1_b
 * wqkv[3d,d] bqkv wo bo ln2_g ln2_b fc1_w[ff,d] fc1_b fc2_w[d,ff] fc2_b, then lnf_g lnf_b. */
typedef struct {
  int dtype, n_layers, d_model, n_heads, d_head, seq, vocab, ff_inner, causal;
  float ln_eps;
} dp_encoder_desc;

int dp_encoder_create(const dp_encoder_desc* desc, dp_encoder** out);
void dp_encoder_destroy(dp_encoder* enc);
int dp_encoder_param_count(const dp_encoder* enc);
int dp_encoder_param_shape(const dp_encoder* enc, int idx, int64_t shape[2], const char** name);
/* Batch-invariant modes (mode 0, the default, is off).  In modes 1 and 2 a sample's result is bit-identical for
 * every num_samples -- what the partial-batch scheme of Sec. 5 (a layer's samples spread over bubbles of different
 * sizes, outputs concatenated) needs if the concatenation has to equal the full-batch result bit for bit.
 *   mode 1: tile shapes and split-K factors of every projection are chosen for one sample's rows instead of the
 *           slice's.  Full speed on slices of up to 4 samples, 12 % slower at 16, 33 % at 64; larger workspace.
 *   mode 2: no split-K, and only tiles built on the 32x32x16 matrix instruction (their shape does not change the
 *           order in which an output element's products are added).  Full speed at 64 samples, 20 % slower on small slices.
 * Set the mode before asking for the workspace size; any other value is DP_EINVAL. */
int dp_encoder_set_batch_invariant(dp_encoder* enc, int mode);
/* Workspace bytes for a call on at most max_samples samples (in the encoder's current mode). */
size_t dp_encoder_workspace_bytes(const dp_encoder* enc, int max_samples);

/* Runs layers [layer_begin, layer_end) on samples [sample_offset, sample_offset + num_samples)
 * of the global batch: the partial-batch layer tuple of Sec. 5.  Layer 0 = embedding
 * (+ position), 1..n_layers = transformer layers, n_layers + 1 = final LayerNorm.
 * ids [device]: int32 [global_batch, seq] (ids outside [0, vocab) are clamped).
 * hidden [device]: [global_batch, seq, d_model], read (unless layer_begin = 0) and written
 * in place for the selected samples only; other rows are untouched, so calls on disjoint
 * sample ranges can be issued in any order or in different bubbles.  num_samples = 0 is a valid
 * empty slice: arguments are still checked, nothing is launched.
 * Invariance: a sample's result is bit-identical run to run and for equal num_samples, whatever the
 * offset and the other samples hold.  By default it is NOT bit-identical across different num_samples (the
 * projections split their contraction by a factor chosen from the row count, which re-associates fp32
 * sums: relative L2 difference of the bf16 output about 4e-3, maximum below 2^-7 of its range), nor across
 * a layer range cut into two calls (the hidden state is rounded to the storage type at the cut).
 * dp_encoder_set_batch_invariant restores bit-identity across num_samples at a cost in speed. */
int encoder_fwd_partial(dp_encoder* enc, const void* const* params, const int32_t* ids, void* hidden,
                        int global_batch, int layer_begin, int layer_end, int sample_offset, int num_samples,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/* One row of the cost profile (Table "Notations"): forward / backward time of layer `layer`
 * of component `component` at batch size `batch` (ms, median of reps), its output size O_l
 * (= the forward activation C^f_{l,l+1} sent to the next layer), the backward message
 * C^b_{l+1,l} and the gradient size G_l, in bytes.  component 0 = backbone stage (layer =
 * block index), 1 = text encoder (layer in the index space above; bwd_ms = 0, grad_bytes = 0), 2 = image
 * encoder (dp_image_encoder_profile). */
typedef struct {
  int component, layer, batch;
  float fwd_ms, bwd_ms;
  int64_t out_bytes, cf_bytes, cb_bytes, grad_bytes;
} dp_layer_cost;

/* Times every block's forward and backward (reps >= 1 repetitions each, hipEvents on the
 * stream; this call synchronises).  Same buffers as stage_fwd / stage_bwd; dparams are
 * overwritten.  Writes n_blocks rows.  The passes run as stage_fwd / stage_bwd run them, side stream included
 * (dp_stage_set_overlap), but the caller's stream waits for a block's side-stream work before the next block's
 * time stamp: a block's weight-gradient kernels are charged to that block, and sum_l (P^f_l + P^b_l) is the
 * time of the step up to what the per-block joins cost (Eq. 3 adds layer times up).  Two things are charged
 * to a neighbour: the context K/V projections of all U-Net blocks (issued at the start of the forward, in
 * block 0's span) and a block's weight transposes (issued one block ahead in the backward). */
int dp_stage_profile(dp_stage* st, const void* const* params, const void* x, const void* ctx_or_cond, void* y,
                     const void* dy, void* dx, void* d_cond, void* const* dparams, void* workspace,
                     size_t workspace_bytes, int reps, dp_layer_cost* rows, int max_rows, int* n_rows,
                     void* hip_stream);

/* Times every encoder layer at each requested partial-batch size (samples [0, b)), in the launch sequence of
 * an ordinary encoder_fwd_partial call over all layers: where a layer's last reduction pass also computes
 * the LayerNorm that opens the next layer (or the final one), that work is charged to the earlier layer and
 * the final LayerNorm's own row can be (almost) empty.  Writes (n_layers + 2) * n_batches rows. */
int dp_encoder_profile(dp_encoder* enc, const void* const* params, const int32_t* ids, void* hidden,
                       int global_batch, const int* batches, int n_batches, int reps, void* workspace,
                       size_t workspace_bytes, dp_layer_cost* rows, int max_rows, int* n_rows, void* hip_stream);

/* Frozen image encoder (Sec. 2.1: the image encoders of diffusion models are auto-encoders; Sec. 2.3 and its
 * execution-time figure: their layers are the moderately long and the extra-long non-trainable layers, which
 * fit a pipeline bubble only on part of the batch, Sec. 5), forward only, bf16 storage, channels-last tensors
 * [batch, height, width, channels].  A layer is one of
 *  DP_IMG_CONV:      y = conv3x3(x; stride 1 or 2, zero padding 1) + b;  parameters w [c_out, 9 * c_in] (taps
 *                    row-major, channels last: w[o, (3u + v) * c_in + c] multiplies x[i * stride + u - 1, j * stride + v - 1, c]), b
 *  DP_IMG_RESNET:    h = conv3x3(silu(GN(x))); h = conv3x3(silu(GN(h))); y = skip(x) + h, skip = identity or a 1x1
 *                    convolution when c_in != c_out;  norm1_g norm1_b conv1_w conv1_b norm2_g norm2_b conv2_w conv2_b
 *                    [skip_w [c_out, c_in] skip_b]
 *  DP_IMG_ATTN:      h = GN(x); q, k, v = 1x1 convolutions of h; a = softmax(q k^T / sqrt(c)) v over the pixels of a
 *                    sample (one head of width c); y = x + 1x1 convolution of a;  norm_g norm_b q_w q_b k_w k_b v_w v_b proj_w proj_b
 *  DP_IMG_NORM_CONV: y = conv3x3(silu(GN(x))) + b (the output head);  norm_g norm_b w b
 * GN = GroupNorm with `groups` groups of consecutive channels, biased variance, eps = gn_eps.  Output height
 * of a stride-s convolution: (height - 1) / s + 1.  Limits: all channel counts multiples of 8 (an RGB image is
 * padded with zero channels) and of `groups` where a GroupNorm reads them, at most 2048; an attention block
 * needs height * width to be a multiple of 8, at most 65536.  DP_F32 is not supported (DP_EUNSUPPORTED). */
typedef struct dp_image_encoder dp_image_encoder; /* opaque, host memory */
enum dp_image_layer_kind { DP_IMG_CONV = 0, DP_IMG_RESNET = 1, DP_IMG_ATTN = 2, DP_IMG_NORM_CONV = 3 };
typedef struct { int kind, c_in, c_out, stride; } dp_image_layer;
typedef struct { int dtype, height, width, in_ch, groups, n_layers; float gn_eps; } dp_image_encoder_desc;

/* layers [host]: n_layers entries, copied.  *out is untouched on error. */
int dp_image_encoder_create(const dp_image_encoder_desc* desc, const dp_image_layer* layers, dp_image_encoder** out);
void dp_image_encoder_destroy(dp_image_encoder* enc);
/* Parameters as a flat array, layer by layer in the orders listed above; names "layer<i>.<tensor>". */
int dp_image_encoder_param_count(const dp_image_encoder* enc);
int dp_image_encoder_param_shape(const dp_image_encoder* enc, int idx, int64_t shape[2], const char** name);
/* hwc = (height, width, channels) of the output of `layer`; layer = -1: the encoder's input. */
int dp_image_encoder_layer_shape(const dp_image_encoder* enc, int layer, int64_t hwc[3]);
/* Workspace bytes [device] for a call on layers [layer_begin, layer_end) and at most max_samples samples. */
size_t dp_image_encoder_workspace_bytes(const dp_image_encoder* enc, int layer_begin, int layer_end, int max_samples);

/* Runs layers [layer_begin, layer_end) on samples [sample_offset, sample_offset + num_samples) of the global
 * batch: the partial-batch tuple (component, layer, #samples) of Sec. 5.  in [device]: the input of layer
 * layer_begin for the whole global batch, [global_batch, h, w, c] of dp_image_encoder_layer_shape(layer_begin - 1);
 * out [device]: the output of layer layer_end - 1, [global_batch, ...]; only the selected samples' rows of `out`
 * are written, so calls on disjoint sample ranges can be issued in any order or in different bubbles, and a
 * later call continues from `out` as its `in`.  in and out must be different buffers.  params [host]: all of the
 * encoder's parameters (only those of the layers in range are read and checked).  num_samples = 0 is a valid
 * empty slice.  Never allocates or synchronises.  A sample's result is bit-identical for every slice size and
 * offset: kernels and the grouping of every sum are chosen from one sample's shape, never from the number of
 * samples; the one choice that follows the slice size, the convolution's tile width, is between two shapes that
 * add in the same order and give the same bits (as long as a layer's input for the slice stays below 2 GiB, the
 * range of the convolution's 32-bit offsets; beyond it another kernel takes over). */
int image_encoder_fwd_partial(dp_image_encoder* enc, const void* const* params, const void* in, void* out, int global_batch,
                              int layer_begin, int layer_end, int sample_offset, int num_samples, void* workspace,
                              size_t workspace_bytes, void* hip_stream);

/* Times every layer at each requested partial-batch size (samples [0, b); in = the images, out = the last
 * layer's output buffer); writes n_layers * n_batches rows with component = 2, bwd_ms = 0, grad_bytes = 0.
 * This call synchronises. */
int dp_image_encoder_profile(dp_image_encoder* enc, const void* const* params, const void* in, void* out, int global_batch,
                             const int* batches, int n_batches, int reps, void* workspace, size_t workspace_bytes,
                             dp_layer_cost* rows, int max_rows, int* n_rows, void* hip_stream);

/* Backbone partitioner (Sec. 4.1, Eq. 1-9; self-conditioning Sec. 4.3, Eq. 17-18), host only: no
 * GPU call is made.  Input is the cost profile of the backbone, rows [host] of component 0 (other
 * components are ignored): one row per (layer, batch) with layers 0..L-1 complete for every batch
 * size that appears.  A stage replicated on r devices runs at local batch micro_batch / r: r must
 * divide micro_batch and that batch size must be in the profile, otherwise that replication is
 * infeasible.  The dynamic programme keeps, for the first l layers in s stages on devices 1..d with
 * the last stage on the last r devices, W = T_0 (Eq. 3, 7), W_SC (Eq. 17) and Y = T_0^{S-C} (Eq. 4-6,
 * 8; clamped at zero) of the candidate that minimises (M + 2S - 2)(p W_SC + (1 - p) W) + Y, and
 * returns the minimum over the replication r of the last stage (Eq. 2), over S = 1..min(L, D,
 * max_stages), plus p T_F with T_F = O_L(micro_batch) / R_p2p + L_p2p.  The first stage has no incoming
 * transfer.  Ties go to fewer stages, then smaller r, earlier cut, smaller replication of the stage
 * before.  Units: ms, bytes, GB/s = 1e9 bytes per second.
 * Errors: DP_EINVAL for null arguments, incomplete or duplicate rows, non-positive sizes or
 * bandwidths, p outside [0, 1], p > 0 without rows at batch = micro_batch; DP_EUNSUPPORTED when no
 * replication vector is feasible or stages x devices^2 x layers exceeds 64M.  `plan` [host] is
 * written on success only; entries past n_stages are zero. */
#define DP_MAX_STAGES 64
typedef struct {
  int micro_batch;          /* B */
  int n_micro_batches;      /* M */
  int n_devices;            /* D, devices of one pipeline-parallel group, <= DP_MAX_STAGES */
  int max_stages;           /* 0: no limit beyond min(L, D) */
  int uniform_replication;  /* 1: every stage on the same number of devices (the setting of Sec. 6) */
  double p2p_gbps, p2p_latency_ms;   /* R_p2p, L_p2p */
  double ar_gbps, ar_latency_ms;     /* R_ar, L_ar */
  double self_cond_prob;             /* p; 0 = Eq. 1 alone */
  int exact_stages;                  /* > 0: partition into exactly this many stages (one point of the search of Sec. 3,
                                        dp_schedule_search); 0: the best stage count up to max_stages */
} dp_partition_opts;
typedef struct {
  int n_stages;
  int first_layer[DP_MAX_STAGES], n_layers[DP_MAX_STAGES], replicas[DP_MAX_STAGES];
  double t0_ms, t0_sc_ms, gap_ms, tf_ms;   /* W, W_SC, Y, T_F of the chosen partition */
  double t_max_ms;                         /* the bound of Eq. 1 / Eq. 18 in expectation */
} dp_partition_plan;
int dp_partition_solve(const dp_layer_cost* rows, int n_rows, const dp_partition_opts* opts, dp_partition_plan* plan);

/* Two backbones of a cascaded model trained on the same devices, pipelined in opposite directions (Sec. 4.2,
 * Eq. 10-16), host only.  rows_down / rows_up: the cost profiles of the two backbones (rows of component 0 of
 * each array).  Both backbones are cut into the same number S of stages; position i of the device chain (low
 * rank first) holds stage i of the down backbone and stage S - 1 - i of the up backbone, both replicated on
 * the same replicas[i] devices.  State (l_d, l_u, s, r, d): the first l_d layers of the down backbone and the
 * last l_u layers of the up backbone in s stages on devices 1..d (the text words the sub-problem the other
 * way round; the two labelings are mirror images); W = max over both backbones' stages of T_0(s) with the
 * communication time of Eq. 3 doubled, Y likewise of T_0^{S-C}(s); the plan minimises (M_CDM + 2S - 2) W + Y
 * (Eq. 12, 13) with M_CDM = opts->n_micro_batches (the paper gives M_CDM no formula).  opts->self_cond_prob
 * must be 0; max_stages, exact_stages and uniform_replication as in dp_partition_solve.  first_layer_up is in
 * the up backbone's own layer numbering.  DP_EUNSUPPORTED when nothing is feasible or the problem is too
 * large (stages x devices^3 x (layers_down x layers_up)^2 > 1.6e10; at most 256 layers per backbone). */
typedef struct {
  int n_stages;
  int first_layer_down[DP_MAX_STAGES], n_layers_down[DP_MAX_STAGES], first_layer_up[DP_MAX_STAGES], n_layers_up[DP_MAX_STAGES],
      replicas[DP_MAX_STAGES];
  double t0_ms, gap_ms;     /* T_0,CDM (Eq. 10) and T_0,CDM^{S-C} (Eq. 11) of the chosen partition */
  double t_max_ms;          /* Eq. 12 */
} dp_bidir_plan;
int dp_partition_solve_bidirectional(const dp_layer_cost* rows_down, int n_down, const dp_layer_cost* rows_up, int n_up,
                                     const dp_partition_opts* opts, dp_bidir_plan* plan);

/* Pipeline bubbles and their filling (Sec. 5, Algorithms 1 and 2), host only: no GPU call is made.
 *
 * dp_bubbles_1f1b simulates one iteration of the FIFO-1F1B schedule of n_stages stages and
 * n_micro_batches micro-batches: stage s runs min(S - 1 - s, M) warm-up forwards, then alternates one
 * forward and one backward, then drains its backwards, micro-batches in order; an operation starts when
 * its stage is free and its input has arrived (forward of the stage before, backward of the stage
 * after, plus comm_fwd_ms[s] / comm_bwd_ms[s] between stages s and s + 1; NULL = 0).  tail_ms[s]
 * (NULL = 0) is busy time after the stage's last backward (gradient synchronisation not overlapped).
 * All arrays [host]: fwd_ms, bwd_ms, replicas, tail_ms have n_stages entries, the comm arrays
 * n_stages - 1.  A bubble is a maximal time span over which the set of idle stages is constant and not
 * empty; n_devices = sum of the replicas of those stages, stage_mask bit s = stage s idle.  Bubbles
 * shorter than min_ms are dropped (the paper uses 10 ms).  They are written in chronological order;
 * *n_out is their number, also when it exceeds max_out (then DP_EWORKSPACE and the first max_out are
 * written); *iteration_ms (may be NULL) is the length of the iteration. */
typedef struct {
  double start_ms, end_ms;
  int n_devices;
  uint64_t stage_mask;
} dp_bubble;
int dp_bubbles_1f1b(int n_stages, const double* fwd_ms, const double* bwd_ms, const int* replicas, int n_micro_batches,
                    const double* comm_fwd_ms, const double* comm_bwd_ms, const double* tail_ms, double min_ms,
                    dp_bubble* out, int max_out, int* n_out, double* iteration_ms);

/* dp_bubbles_fill fills the bubbles, in the order given (chronological), with the layers of the
 * non-trainable components described by the cost rows with component >= 1 (fwd_ms at the local batch
 * sizes profiled; layers 0..L-1 complete for every batch size of a component; components are taken in
 * ascending id).  dep_pairs [2 * n_dep_pairs]: (component, component it depends on); a component is
 * ready in a bubble when all layers of its dependencies were placed in earlier bubbles.  `batch` is the
 * training batch size: a whole-batch layer on the d idle devices of a bubble runs at local batch
 * ceil(batch / d); a local batch size between two profiled ones is interpolated linearly, below the
 * smallest it costs as the smallest, above the largest proportionally.  Per bubble: Algorithm 2 lists
 * the ways to pack whole-batch layers of the ready components; Algorithm 1 adds to each at most one
 * partial-batch layer, the next layer of one component on b samples, b / d one of 4, 8, 12, 16, 24, 32,
 * 48, 64, 96, b smaller than what is left of that layer and as large as fits; the candidate that runs
 * longest is kept.  A layer begun on part of the batch is the first ready layer of its component in the
 * following bubbles and counts as a whole-batch layer on its remaining samples.  Output: one dp_fill
 * row per run of whole-batch layers of a component in a bubble (partial = 0: layers first_layer ..
 * first_layer + n_layers - 1, `samples` = samples of the first of them, the others take the whole
 * batch) and one per partial-batch layer (partial = 1, n_layers = 1, `samples` = b); fill_ms is the
 * run time of the bubble's whole filling.  The summary holds the idle device-time offered, the
 * device-time filled, and leftover_ms: the time of the layers that fit no bubble, run after the
 * pipeline on all n_devices devices.  summary.n_fills is the number of rows, also when it exceeds
 * max_fills (then DP_EWORKSPACE). */
typedef struct {
  int bubble, component, first_layer, n_layers, samples, partial;
  double fill_ms;
} dp_fill;
typedef struct {
  double bubble_device_ms, filled_device_ms, leftover_ms;
  int n_fills;
} dp_fill_summary;
int dp_bubbles_fill(const dp_bubble* bubbles, int n_bubbles, const dp_layer_cost* rows, int n_rows, const int* dep_pairs,
                    int n_dep_pairs, int batch, int n_devices, dp_fill* fills, int max_fills, dp_fill_summary* summary);

/* Search over the pipeline hyper-parameters (Sec. 3, workflow steps 2-5; Table "Pipeline training
 * hyper-parameters": S stages, M micro-batches, D devices per pipeline-parallel group, world size = D x
 * data-parallel degree), host only.  For every D of group_sizes that divides world_size, every M of
 * micro_batch_counts and every S = 1..min(L, D, max_stages): a pipeline group trains training_batch * D /
 * world_size samples per iteration in M micro-batches of B samples (combinations where these are not
 * integers are skipped); the backbone (rows of component 0) is partitioned into exactly S stages
 * (dp_partition_solve; skipped when infeasible); the FIFO-1F1B iteration of that plan is simulated
 * (dp_bubbles_1f1b) with per-stage forward time (1 + p) sum P^f at the stage's local batch B / r, backward
 * time sum P^b, transfers C / R_p2p + L_p2p between stages and the gradient synchronisation sum G / R_ar +
 * L_ar (Eq. 4) after a stage's last backward; its bubbles (at least min_bubble_ms long) are filled with the
 * non-trainable components (rows of component >= 1; dp_bubbles_fill with the group's batch and D devices;
 * dep_pairs as there).  iteration_ms = pipeline_ms + leftover_ms (the frozen layers that fit no bubble, run
 * after the pipeline on the group's devices).  Candidates are written in the order walked (group_sizes, then
 * micro_batch_counts, then S ascending); *best is the index of the least iteration_ms, the earlier one on
 * ties.  *n_cands is the number of feasible combinations, also when it exceeds max_cands (DP_EWORKSPACE; the
 * first max_cands are written and *best refers to them).  DP_EUNSUPPORTED when no combination is feasible. */
typedef struct {
  int world_size, training_batch;
  const int* group_sizes; int n_group_sizes;                 /* candidate D [host] */
  const int* micro_batch_counts; int n_micro_batch_counts;   /* candidate M [host] */
  int max_stages;                                            /* 0: up to min(L, D) */
  int uniform_replication;
  double p2p_gbps, p2p_latency_ms, ar_gbps, ar_latency_ms, self_cond_prob;
  double min_bubble_ms;
  const int* dep_pairs; int n_dep_pairs;
} dp_search_opts;
typedef struct {
  int n_stages, n_micro_batches, group_size, micro_batch;    /* S, M, D, B */
  double pipeline_ms, leftover_ms, iteration_ms;
  double bubble_ratio;           /* idle device-time / (D x pipeline_ms), before filling */
  double bubble_ratio_filled;    /* unfilled idle device-time / (D x iteration_ms) */
  dp_partition_plan plan;
} dp_search_candidate;
int dp_schedule_search(const dp_layer_cost* rows, int n_rows, const dp_search_opts* opts, dp_search_candidate* cands, int max_cands,
                       int* n_cands, int* best);

/* Operator-level entry points: the same kernels the stage calls, exposed one by one for unit
 * tests and per-kernel measurement (the cost profile of Sec. 4 is per layer; these go one
 * level below it).  All pointers [device]; dtype as in dp_dtype.
 *
 * dp_op_gemm: C[M,N] = A * B with fp32 accumulation.  a_kmajor = 0: A is [M,K] row-major,
 * 1: A is stored [K,M].  b_kmajor = 0: B is stored [N,K] (a weight applied as x W^T), 1: B is
 * stored [K,N].  out_is_f32 = 0: C in the storage dtype (+ optional bias [N]); 1: C fp32, dense,
 * overwritten or accumulated into.  `workspace` (fp32 scratch of dp_op_gemm_workspace_bytes; may be
 * NULL, then nothing is split) serves a fixed-order split-K reduction: of the fp32 output, and of a
 * storage-dtype output with few tiles and a long contraction, whose bias is then applied by the
 * reduction pass.  tile_cfg = 0 picks the tile shape from (M,N,K); 1..15 force one (measurement and
 * tests only): 1..6 register-staged tiles, 7..15 direct-to-LDS tiles, which need K % 32 == 0
 * (7, 8, 9, 13, 15) or K % 64 == 0 (10, 11, 12, 14); 12 exists for a_kmajor = b_kmajor = 0 only.  A forced
 * configuration that does not fit the problem returns DP_EUNSUPPORTED without launching. */
size_t dp_op_gemm_workspace_bytes(int M, int N, int K);
int dp_op_gemm(int dtype, const void* A, int lda, int a_kmajor, const void* B, int ldb, int b_kmajor, int M, int N, int K,
               const void* bias, void* C, int ldc, int out_is_f32, int accumulate, void* workspace, size_t workspace_bytes,
               int tile_cfg, void* hip_stream);

/* FP8 variant of the projection GEMM, an extension for MI355X (whose matrix pipe runs 8-bit operands at twice the
 * bf16 rate): meant for the frozen, forward-only components (Sec. 2.1), whose projections need no gradient.
 * Format: OCP E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; subnormals; largest finite value 448; no
 * infinities), one scale per tensor.
 * dp_op_quantize_fp8: q[i, j] = e4m3(clamp(x[i, j] * (1 / scale), -448, 448)), the product formed in fp32 (1 / scale
 * rounded to fp32 first), conversion to the nearest E4M3 value, ties to even.  x [device]: bf16 [rows, cols], row
 * stride ldx elements; q [device]: bytes [rows, cols], row stride ldq; cols, ldx, ldq multiples of 8.
 * dp_op_gemm_fp8: C[M, N] (bf16, row stride ldc) = out_scale * sum_k A[m, k] B[n, k] (+ bias[n], bf16), A [M, K] and
 * B [N, K] E4M3 bytes with row strides lda, ldb (multiples of 16), fp32 accumulation; out_scale is the product of the
 * two tensors' scales.  K a multiple of 128, N and ldc of 8; operands below 4 GiB. */
int dp_op_quantize_fp8(const void* x, int ldx, void* q, int ldq, int rows, int cols, float scale, void* hip_stream);
int dp_op_gemm_fp8(const void* A, int lda, const void* B, int ldb, int M, int N, int K, float out_scale, const void* bias, void* C,
                   int ldc, void* hip_stream);

/* dp_op_gemm for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same operation, arguments and results as dp_op_gemm (bit for bit
 * those of dp_op_gemm given a workspace of dp_op_gemm_workspace_bytes), but the split-K partial sums live in
 * a device array of DP_STATIC_SCRATCH_BYTES that is part of the library image: every GPU the library runs on
 * holds its own copy until the process ends.  The call allocates and frees nothing, on the host's heap or
 * the device.  A problem for which dp_op_gemm_workspace_bytes(M, N, K) exceeds DP_STATIC_SCRATCH_BYTES is
 * rejected with DP_EWORKSPACE before anything is launched.  The device of hip_stream must be the calling
 * thread's current device (the array's address is looked up per device, on the first call on that device).
 * All calls on one GPU share that GPU's array: calls that may overlap on one GPU (different streams, or
 * different threads) race on it; issue them on one stream.  Nothing in the array has to be cleared
 * between calls: a call overwrites every partial sum it later reads. */
#define DP_STATIC_SCRATCH_BYTES (64u << 20)
int dp_op_gemm_static(int dtype, const void* A, int lda, int a_kmajor, const void* B, int ldb, int b_kmajor, int M, int N, int K,
                      const void* bias, void* C, int ldc, int out_is_f32, int accumulate, int tile_cfg, void* hip_stream);

/* dp_op_attention_fwd / _bwd: per (batch, head) O = softmax(Q K^T * scale [causal]) V.
 * Element (b, n, h, t) of a tensor X is X[(b * rows + n) * ldX + h * d_head + t], so Q, K, V may
 * be column blocks of one fused projection output.  lse: fp32 [B, H, Nq] (written by fwd, read
 * by bwd).  delta: fp32 [B, H, Nq] scratch.  The backward does not support the causal mask.
 * bf16: d_head a multiple of 8, at most 96; leading dimensions multiples of 8; operands 16-byte aligned;
 * one batch element's rows of any operand span less than 2 GiB (max(Nq, Nk) * ld * 2 < 2^31), else
 * DP_EUNSUPPORTED.  All of this is checked before anything is launched. */
int dp_op_attention_fwd(int dtype, int B, int H, int Nq, int Nk, int d_head, int causal, float scale, const void* q, int ldq,
                        const void* k, int ldk, const void* v, int ldv, void* o, int ldo, float* lse, void* hip_stream);
int dp_op_attention_bwd(int dtype, int B, int H, int Nq, int Nk, int d_head, float scale, const void* q, int ldq, const void* k,
                        int ldk, const void* v, int ldv, const void* o, int ldo, const float* lse, const void* d_o, int lddo,
                        float* delta, void* dq, int lddq, void* dk, int lddk, void* dv, int lddv, void* hip_stream);

/* Measurement aid: per-launch kernel timing.  Between dp_ktime_begin and dp_ktime_end every
 * kernel class the library launches is bracketed by hipEvents on the caller's stream; each
 * record carries the kernel kind, the algorithmic FLOPs and bytes of that launch (the
 * accounting used for the roofline figures: 2mnk per GEMM, 4 * B * H * Nq * Nk * d_head per
 * attention forward, tensor bytes read + written once for the bandwidth-bound kernels) and
 * its duration.  kind: 0 GEMM y = x W^T, 1 GEMM dx = dy W, 2 GEMM dW = dy^T x, 3 attention
 * forward, 4 attention dQ, 5 attention dK/dV, 6 LayerNorm forward, 7 LayerNorm backward,
 * 8 GeGLU forward, 9 GeGLU backward, 10 partial-sum reductions, 11 other, 12 fp32 GEMM,
 * 13 fp32 attention, 14 3x3 convolution (2 * pixels * c_out * 9 c_in), 15 GroupNorm, 16 row softmax, 17 fp8 GEMM.  dp_ktime_begin allocates host-side events (max_records pairs);
 * dp_ktime_end synchronises the device, writes up to max records and frees them.  `ms` is the
 * time between a record's two events, which includes the dispatch gap around the kernel (an upper
 * bound of the kernel's duration: a few microseconds above what a kernel trace shows).  For scale,
 * dp_ktime_end also records up to 33 empty event pairs on the same stream when the pool has spare
 * events; dp_ktime_event_overhead_ms returns their median reading (0 if none was taken).
 * Not thread-safe; the recording adds launch overhead, so use it in a pass of its own. */
typedef struct {
  int kind, m, n, k;
  float ms;
  double flops, bytes;
} dp_kernel_time;
int dp_ktime_begin(int max_records);
int dp_ktime_end(dp_kernel_time* out, int max, int* n);
float dp_ktime_event_overhead_ms(void);

/* Thread-local description of the last error; never NULL. */
const char* dp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DPIPE_H */
