"""Frozen image-encoder layers, float64 (test infrastructure only).

The second non-trainable component of a diffusion model next to the text encoder
(Sec. 2.1: the image encoders are variational auto-encoders; Sec. 2.3 and its
execution-time figure: their layers are the moderately long and the extra-long
non-trainable layers, the ones that only fit a pipeline bubble on part of the
batch, Sec. 5).  The paper treats the layers as black boxes; the arithmetic
below is the public formulation of a convolutional auto-encoder's encoder:
3x3 convolutions (stride 1, or 2 to halve the resolution), GroupNorm, SiLU,
residual blocks and a single-head self-attention block over the pixels.

Tensors are channels-last: activations [B, H, W, C], convolution weights
[C_out, 3, 3, C_in] (1x1: [C_out, C_in]).  Parameters are dicts keyed by name.

Layer kinds (`layers` is a list of dicts with "kind" and channel counts):
  conv      y = conv3x3(x; stride) + b
  resnet    h = conv3x3(silu(GN(x))); h = conv3x3(silu(GN(h))); y = skip(x) + h,
            skip = identity, or a 1x1 convolution when the channel count changes
  attn      h = GN(x); q, k, v = 1x1 convolutions of h; a = softmax(q k^T / sqrt(C)) v over the
            H*W pixels of a sample, one head of width C; y = x + 1x1 convolution of a
  norm_conv y = conv3x3(silu(GN(x))) + b   (the encoder's output head)
"""
from __future__ import annotations

import math

import numpy as np

from . import ops


def conv3x3(x, w, b=None, stride=1):
    """Cross-correlation with zero padding 1: y[n, i, j, :] = sum_{u, v} x_pad[n, i*stride + u, j*stride + v, :] w[:, u, v, :]^T (+ b).
    x [B, H, W, Cin], w [Cout, 3, 3, Cin] -> [B, Ho, Wo, Cout], Ho = (H - 1) // stride + 1."""
    B, H, W, _ = x.shape
    w = w.reshape(w.shape[0], 3, 3, x.shape[3])      # also accepts the flat [Cout, 9 * Cin] form, taps row-major, channels last
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    xp = np.zeros((B, H + 2, W + 2, x.shape[3]))
    xp[:, 1:H + 1, 1:W + 1, :] = x
    y = np.zeros((B, Ho, Wo, w.shape[0]))
    for u in range(3):
        for v in range(3):
            win = xp[:, u:u + (Ho - 1) * stride + 1:stride, v:v + (Wo - 1) * stride + 1:stride, :]
            y += win @ w[:, u, v, :].T
    if b is not None:
        y = y + b
    return y


def conv1x1(x, w, b=None):
    return ops.linear_fwd(x, w, b)


def groupnorm(x, gamma, beta, groups, eps=1e-6):
    """Per sample and per group of C / groups consecutive channels: mean and biased variance over the
    group's channels at all pixels; y = (x - mean) / sqrt(var + eps) * gamma_c + beta_c."""
    B, H, W, C = x.shape
    xg = x.reshape(B, H * W, groups, C // groups)
    mu = xg.mean(axis=(1, 3), keepdims=True)
    var = ((xg - mu) ** 2).mean(axis=(1, 3), keepdims=True)
    y = ((xg - mu) / np.sqrt(var + eps)).reshape(B, H, W, C)
    return y * gamma + beta


def resnet_block(p, pre, x, groups, eps):
    g = lambda n: p[pre + n]
    h = conv3x3(ops.silu(groupnorm(x, g("norm1_g"), g("norm1_b"), groups, eps)), g("conv1_w"), g("conv1_b"))
    h = conv3x3(ops.silu(groupnorm(h, g("norm2_g"), g("norm2_b"), groups, eps)), g("conv2_w"), g("conv2_b"))
    skip = conv1x1(x, g("skip_w"), g("skip_b")) if (pre + "skip_w") in p else x
    return skip + h


def attn_block(p, pre, x, groups, eps):
    g = lambda n: p[pre + n]
    B, H, W, C = x.shape
    h = groupnorm(x, g("norm_g"), g("norm_b"), groups, eps).reshape(B, H * W, C)
    q, k, v = (conv1x1(h, g(n + "_w"), g(n + "_b")) for n in ("q", "k", "v"))
    a = ops.attention_fwd(q, k, v, 1)                    # one head of width C: logits scaled by 1 / sqrt(C)
    return x + conv1x1(a, g("proj_w"), g("proj_b")).reshape(B, H, W, C)


def layer_fwd(p, layers, l, x, groups, eps=1e-6):
    L, pre = layers[l], f"layer{l}."
    if L["kind"] == "conv":
        return conv3x3(x, p[pre + "w"], p[pre + "b"], L.get("stride", 1))
    if L["kind"] == "resnet":
        return resnet_block(p, pre, x, groups, eps)
    if L["kind"] == "attn":
        return attn_block(p, pre, x, groups, eps)
    if L["kind"] == "norm_conv":
        return conv3x3(ops.silu(groupnorm(x, p[pre + "norm_g"], p[pre + "norm_b"], groups, eps)), p[pre + "w"], p[pre + "b"])
    raise ValueError(L["kind"])


def encoder_fwd_partial(p, layers, x_in, layer_begin, layer_end, sample_offset, num_samples, groups, eps=1e-6):
    """Layers [layer_begin, layer_end) on samples [sample_offset, sample_offset + num_samples) of
    x_in, the global batch's input of layer `layer_begin` (the partial-batch tuple (component, layer,
    #samples) of Sec. 5).  Returns the output of layer `layer_end - 1` for those samples."""
    x = x_in[sample_offset:sample_offset + num_samples]
    for l in range(layer_begin, layer_end):
        x = layer_fwd(p, layers, l, x, groups, eps)
    return x


def encoder_fwd(p, layers, x, groups, eps=1e-6):
    return encoder_fwd_partial(p, layers, x, 0, len(layers), 0, x.shape[0], groups, eps)
