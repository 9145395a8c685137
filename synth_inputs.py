"""Seeded synthetic inputs for the five workloads (data only).

This module is the single thing the CPU oracle's tests and the HIP path's
tests/bench share.  It holds workload shapes, parameter name/shape tables and
random draws -- none of the transformer-block arithmetic.  Everything is drawn
on the host from ``numpy.random.default_rng(seed)`` in a fixed order
(parameters in table order, then x, ctx/cond/ids, dy, x_sc), rounded to the
storage dtype (bf16 round-to-nearest-even, or fp32) and returned as float64
holding exactly-representable values, so that input quantisation is never
counted as a GPU-vs-oracle difference.

The shapes stand in for the paper's workloads (Sec. "Evaluation": Stable
Diffusion v2.1 / ControlNet at 512x512, i.e. 64x64 and 32x32 latents with a
77-token text context; DiT-type backbones named in the conclusion; the frozen
CLIP text encoder of Sec. 2.1).  No dataset or trained weight is involved.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, asdict

import numpy as np

UNET = "unet_xattn_geglu"
DIT = "dit_adaln_zero"


# --------------------------------------------------------------------------
# storage-dtype rounding helpers (pure data conversion)
# --------------------------------------------------------------------------
def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round to bf16 (nearest-even) and widen back to float64."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(a.shape)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float array (already bf16-representable or not) -> uint16 bf16 bit patterns (RNE)."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16).reshape(a.shape)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def round_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_bf16(a)
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class StageConfig:
    name: str
    kind: str            # UNET or DIT
    dtype: str           # "f32" or "bf16"
    n_blocks: int
    batch: int
    tokens: int
    d_model: int
    n_heads: int
    d_head: int
    ctx_tokens: int = 0  # UNET only
    ctx_dim: int = 0     # UNET only
    ff_inner: int = 0
    ln_eps: float = 1e-5
    gelu_tanh: int = 0
    self_cond: bool = False

    def replace(self, **kw) -> "StageConfig":
        d = asdict(self)
        d.update(kw)
        return StageConfig(**d)


@dataclass(frozen=True)
class EncoderConfig:
    name: str
    dtype: str
    n_layers: int
    d_model: int
    n_heads: int
    d_head: int
    seq: int
    vocab: int
    ff_inner: int
    global_batch: int
    causal: int = 1
    ln_eps: float = 1e-5
    slices: tuple = (1, 4, 16, 64)

    def replace(self, **kw) -> "EncoderConfig":
        d = asdict(self)
        d.update(kw)
        return EncoderConfig(**d)


CONFIG1 = StageConfig("cfg1_tiny_unet_f32", UNET, "f32", 1, 2, 64, 64, 4, 16, 8, 64, 256, 1e-5, 0)
CONFIG2 = StageConfig("cfg2_sd_32x32_d640", UNET, "bf16", 2, 8, 1024, 640, 10, 64, 77, 768, 2560, 1e-5, 0)
CONFIG3 = StageConfig("cfg3_sd_64x64_d320", UNET, "bf16", 2, 8, 4096, 320, 5, 64, 77, 768, 1280, 1e-5, 0)
CONFIG4 = StageConfig("cfg4_dit_xl2_selfcond", DIT, "bf16", 7, 32, 256, 1152, 16, 72, 0, 0, 4608, 1e-6, 1,
                      self_cond=True)
CONFIG5 = EncoderConfig("cfg5_clip_l_text", "bf16", 12, 768, 12, 64, 77, 49408, 3072, 64)

STAGE_CONFIGS = {c.name: c for c in (CONFIG1, CONFIG2, CONFIG3, CONFIG4)}


@dataclass(frozen=True)
class ImageEncoderConfig:
    """A frozen convolutional image encoder (the auto-encoder's encoder of a latent diffusion model):
    `layers` is a tuple of (kind, c_in, c_out, stride) with kind in conv / resnet / attn / norm_conv."""
    name: str
    dtype: str
    height: int
    width: int
    in_ch: int
    groups: int
    layers: tuple
    global_batch: int
    gn_eps: float = 1e-6
    slices: tuple = (1, 2, 4, 8)

    def replace(self, **kw) -> "ImageEncoderConfig":
        d = {f: getattr(self, f) for f in self.__dataclass_fields__}
        d.update(kw)
        return ImageEncoderConfig(**d)

    def layer_dicts(self):
        return [{"kind": k, "cin": ci, "cout": co, "stride": st} for (k, ci, co, st) in self.layers]

    def out_shape(self, upto=None):
        """(H, W, C) after layer `upto - 1` (all layers when None); upto = 0 is the input."""
        h, w, c = self.height, self.width, self.in_ch
        for (k, ci, co, st) in self.layers[:len(self.layers) if upto is None else upto]:
            if k == "conv" and st == 2:
                h, w = (h - 1) // 2 + 1, (w - 1) // 2 + 1
            c = co
        return h, w, c


def vae_encoder_layers(ch=128, mult=(1, 2, 4, 4), in_ch=8, out_ch=8):
    """The encoder of the latent-diffusion auto-encoder: input convolution, per resolution two
    residual blocks and (but for the last) a stride-2 convolution, a middle of residual block /
    attention / residual block, and the GroupNorm + SiLU + convolution head.  in_ch = 8: the three
    image channels padded with zero channels to a 16-byte pixel."""
    L = [("conv", in_ch, ch, 1)]
    c = ch
    for i, m in enumerate(mult):
        for _ in range(2):
            L.append(("resnet", c, ch * m, 1))
            c = ch * m
        if i != len(mult) - 1:
            L.append(("conv", c, c, 2))
    L += [("resnet", c, c, 1), ("attn", c, c, 1), ("resnet", c, c, 1), ("norm_conv", c, out_ch, 1)]
    return tuple(L)


# Stable Diffusion's image encoder at the paper's 512 x 512 training resolution (Sec. "Evaluation"): 16 layers,
# 128..512 channels, 64 x 64 x 8 output (mean and log-variance of the 4-channel latent).
CONFIG6 = ImageEncoderConfig("cfg6_vae_encoder_512", "bf16", 512, 512, 8, 32, vae_encoder_layers(), 8)


# --------------------------------------------------------------------------
# parameter tables: (name, shape, init) in the order the C ABI takes them
# init: "w" -> N(0, 0.02), "one" -> 1, "zero" -> 0
# --------------------------------------------------------------------------
def unet_block_param_specs(c: StageConfig):
    d, dc, inner = c.d_model, c.ctx_dim, c.ff_inner
    return [
        ("ln1_g", (d,), "one"), ("ln1_b", (d,), "zero"),
        ("attn1_wqkv", (3 * d, d), "w"),
        ("attn1_wo", (d, d), "w"), ("attn1_bo", (d,), "w"),
        ("ln2_g", (d,), "one"), ("ln2_b", (d,), "zero"),
        ("attn2_wq", (d, d), "w"),
        ("attn2_wkv", (2 * d, dc), "w"),
        ("attn2_wo", (d, d), "w"), ("attn2_bo", (d,), "w"),
        ("ln3_g", (d,), "one"), ("ln3_b", (d,), "zero"),
        ("ff_w1", (2 * inner, d), "w"), ("ff_b1", (2 * inner,), "w"),
        ("ff_w2", (d, inner), "w"), ("ff_b2", (d,), "w"),
    ]


def dit_block_param_specs(c: StageConfig):
    d, ff = c.d_model, c.ff_inner
    return [
        ("ada_w", (6 * d, d), "w"), ("ada_b", (6 * d,), "w"),
        ("attn_wqkv", (3 * d, d), "w"), ("attn_bqkv", (3 * d,), "w"),
        ("attn_wo", (d, d), "w"), ("attn_bo", (d,), "w"),
        ("fc1_w", (ff, d), "w"), ("fc1_b", (ff,), "w"),
        ("fc2_w", (d, ff), "w"), ("fc2_b", (d,), "w"),
    ]


def stage_param_specs(c: StageConfig):
    per = unet_block_param_specs(c) if c.kind == UNET else dit_block_param_specs(c)
    out = []
    for b in range(c.n_blocks):
        out += [(f"block{b}.{n}", s, i) for (n, s, i) in per]
    return out


def encoder_param_specs(c: EncoderConfig):
    d, ff = c.d_model, c.ff_inner
    out = [("tok_emb", (c.vocab, d), "w"), ("pos_emb", (c.seq, d), "w")]
    for l in range(c.n_layers):
        out += [(f"layer{l}.{n}", s, i) for (n, s, i) in [
            ("ln1_g", (d,), "one"), ("ln1_b", (d,), "zero"),
            ("wqkv", (3 * d, d), "w"), ("bqkv", (3 * d,), "w"),
            ("wo", (d, d), "w"), ("bo", (d,), "w"),
            ("ln2_g", (d,), "one"), ("ln2_b", (d,), "zero"),
            ("fc1_w", (ff, d), "w"), ("fc1_b", (ff,), "w"),
            ("fc2_w", (d, ff), "w"), ("fc2_b", (d,), "w"),
        ]]
    out += [("lnf_g", (d,), "one"), ("lnf_b", (d,), "zero")]
    return out


def _draw_params(rng, specs, dtype, randomize_ln):
    params = {}
    for name, shape, init in specs:
        if init == "w":
            a = rng.normal(0.0, 0.02, size=shape)
        elif init == "one":
            a = 1.0 + (rng.normal(0.0, 0.1, size=shape) if randomize_ln else np.zeros(shape))
        else:
            a = rng.normal(0.0, 0.1, size=shape) if randomize_ln else np.zeros(shape)
        params[name] = round_storage(a, dtype)
    return params


def timestep_conditioning(t: np.ndarray, d: int, rng) -> np.ndarray:
    """Conditioning vectors for the DiT-style stage: a 256-dim sinusoidal
    embedding of the integer timestep (cos half, then sin half, frequencies
    exp(-ln(10000) i/128)) pushed through a randomly initialised two-layer
    SiLU embedder.  This happens upstream of the stage; it is input
    preparation, computed once here in fp64."""
    half = 128
    freqs = np.exp(-math.log(10000.0) * np.arange(half) / half)
    args = t[:, None].astype(np.float64) * freqs[None, :]
    phi = np.concatenate([np.cos(args), np.sin(args)], axis=1)
    w1 = rng.normal(0.0, 0.02, size=(d, 256)); b1 = rng.normal(0.0, 0.02, size=(d,))
    w2 = rng.normal(0.0, 0.02, size=(d, d)); b2 = rng.normal(0.0, 0.02, size=(d,))
    h = phi @ w1.T + b1
    h = h / (1.0 + np.exp(-h))
    c = h @ w2.T + b2
    # the embedder's output has a small scale with N(0,0.02) weights; bring it to O(1)
    # so that SiLU(c) and the modulation it drives are exercised away from zero
    return c / c.std()


def make_stage_inputs(c: StageConfig, seed: int = 0, randomize_ln: bool = False, logit_gain: float = 1.0):
    """Returns dict(params=..., x=, ctx= or cond=, dy=, x_sc=, t=).

    ``logit_gain`` > 1 scales the query rows of the attention projections so
    that the softmax is far from uniform (a stress input for the online
    softmax rescaling); 1.0 gives the plain N(0,0.02) workload."""
    rng = np.random.default_rng(seed)
    specs = stage_param_specs(c)
    params = _draw_params(rng, specs, c.dtype, randomize_ln)
    if logit_gain != 1.0:
        d = c.d_model
        for name in list(params):
            if name.endswith("attn1_wqkv") or name.endswith("attn_wqkv"):
                w = params[name].copy(); w[:d] *= logit_gain; w[d:2 * d] *= logit_gain
                params[name] = round_storage(w, c.dtype)
            elif name.endswith("attn2_wq"):
                params[name] = round_storage(params[name] * logit_gain * logit_gain, c.dtype)
    B, N, d = c.batch, c.tokens, c.d_model
    out = {"params": params}
    out["x"] = round_storage(rng.normal(size=(B, N, d)), c.dtype)
    if c.kind == UNET:
        out["ctx"] = round_storage(rng.normal(size=(B, c.ctx_tokens, c.ctx_dim)), c.dtype)
    else:
        t = rng.integers(0, 1000, size=(B,))
        out["t"] = t
        out["cond"] = round_storage(timestep_conditioning(t, d, rng), c.dtype)
    out["dy"] = round_storage(rng.normal(size=(B, N, d)), c.dtype)
    out["x_sc"] = round_storage(rng.normal(size=(B, N, d)), c.dtype)
    return out


def make_attention_inputs(B, H, Nq, Nk, dh, seed, gain=1.0, row_shift=0.0):
    """q [B,Nq,H*dh], k, v [B,Nk,H*dh], do [B,Nq,H*dh] for the attention operator, bf16-representable.

    gain = 1, row_shift = 0: plain N(0,1) tensors.  Otherwise a stress input for a tiled online
    softmax: queries are scaled by ``gain`` (logit spread), key j is scaled by a ramp rising from
    0.5 to 1.5 along the key index (the extreme logits, hence the row maxima, tend to arrive in late
    key tiles), and the first coordinate of every head carries a per-row constant: keys hold 4 there
    and query i holds r_i sqrt(dh) / 4 with r_i ~ U(-row_shift, row_shift), which adds r_i to every
    logit of row i (a shift that an exact softmax cancels)."""
    rng = np.random.default_rng(seed)
    d = H * dh
    q, k, v, do = (rng.standard_normal((B, n, d)) for n in (Nq, Nk, Nk, Nq))
    if gain != 1.0 or row_shift != 0.0:
        q *= gain
        k *= np.linspace(0.5, 1.5, Nk)[None, :, None]
        r = rng.uniform(-row_shift, row_shift, size=(B, Nq))
        for h in range(H):
            k[:, :, h * dh] = 4.0
            q[:, :, h * dh] = r * math.sqrt(dh) / 4.0
    return tuple(round_bf16(t) for t in (q, k, v, do))


def image_encoder_param_specs(c: ImageEncoderConfig):
    """(name, shape, init) in the order the C ABI takes them.  Convolution weights are [C_out, 9 * C_in]
    (taps row-major, channels last), 1x1 convolutions [C_out, C_in]."""
    out = []
    for l, (kind, ci, co, st) in enumerate(c.layers):
        pre = f"layer{l}."
        if kind == "conv":
            per = [("w", (co, 9 * ci), "w"), ("b", (co,), "w")]
        elif kind == "resnet":
            per = [("norm1_g", (ci,), "one"), ("norm1_b", (ci,), "zero"), ("conv1_w", (co, 9 * ci), "w"), ("conv1_b", (co,), "w"),
                   ("norm2_g", (co,), "one"), ("norm2_b", (co,), "zero"), ("conv2_w", (co, 9 * co), "w"), ("conv2_b", (co,), "w")]
            if ci != co:
                per += [("skip_w", (co, ci), "w"), ("skip_b", (co,), "w")]
        elif kind == "attn":
            per = [("norm_g", (ci,), "one"), ("norm_b", (ci,), "zero")]
            for n in ("q", "k", "v", "proj"):
                per += [(n + "_w", (ci, ci), "w"), (n + "_b", (ci,), "w")]
        elif kind == "norm_conv":
            per = [("norm_g", (ci,), "one"), ("norm_b", (ci,), "zero"), ("w", (co, 9 * ci), "w"), ("b", (co,), "w")]
        else:
            raise ValueError(kind)
        out += [(pre + n, s, i) for (n, s, i) in per]
    return out


def make_image_encoder_inputs(c: ImageEncoderConfig, seed: int = 0, randomize_norm: bool = False, weight_std: float = 0.02):
    """params in table order, then images [global_batch, H, W, in_ch] ~ N(0, 1) (a normalised image; when
    in_ch = 8 the channels 3..7 are the zero padding).  weight_std: the N(0, 0.02) of the other workloads
    makes a 3x3 convolution shrink its input by an order of magnitude per layer; tests may pass
    1 / sqrt(fan_in)-like values to keep activations O(1) through 16 layers."""
    rng = np.random.default_rng(seed)
    params = {}
    for name, shape, init in image_encoder_param_specs(c):
        if init == "w":
            std = weight_std if weight_std > 0 else (1.0 / math.sqrt(shape[1]) if len(shape) == 2 else 0.02)
            a = rng.normal(0.0, std, size=shape)
        elif init == "one":
            a = 1.0 + (rng.normal(0.0, 0.1, size=shape) if randomize_norm else np.zeros(shape))
        else:
            a = rng.normal(0.0, 0.1, size=shape) if randomize_norm else np.zeros(shape)
        params[name] = round_storage(a, c.dtype)
    x = rng.normal(size=(c.global_batch, c.height, c.width, c.in_ch))
    if c.in_ch == 8:
        x[..., 3:] = 0.0
    return {"params": params, "x": round_storage(x, c.dtype)}


def make_encoder_inputs(c: EncoderConfig, seed: int = 0, randomize_ln: bool = False):
    rng = np.random.default_rng(seed)
    params = _draw_params(rng, encoder_param_specs(c), c.dtype, randomize_ln)
    ids = rng.integers(0, c.vocab, size=(c.global_batch, c.seq)).astype(np.int32)
    return {"params": params, "ids": ids}
