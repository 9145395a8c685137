"""Frozen CLIP-style text encoder forward, float64 (test infrastructure only).

The non-trainable part of the diffusion model (Sec. 2.1: a frozen text encoder
that only runs forward) executed as partial-batch layers (Sec. 5: a layer is
run on b of the B samples, the input is split and the outputs concatenated
across pipeline bubbles).  The paper treats its layers as black boxes; the
arithmetic is the public pre-norm causal transformer with quick-GELU.

Layer index space: 0 = token + position embedding, 1..n_layers = transformer
layers, n_layers + 1 = final LayerNorm.
"""
from __future__ import annotations

import numpy as np

from . import ops


def embed(p, ids):
    """x = E_tok[ids] + E_pos[0:seq]; ids [b, seq] -> [b, seq, d]."""
    return p["tok_emb"][ids] + p["pos_emb"][None, : ids.shape[1], :]


def layer_fwd(p, l, x, n_heads, eps=1e-5, causal=True):
    """One pre-norm layer: causal multi-head self-attention (biases on q, k, v
    and output projections), then a quick-GELU MLP, each with a residual."""
    d = x.shape[-1]
    g = lambda n: p[f"layer{l}.{n}"]
    h, _, _ = ops.layernorm_fwd(x, g("ln1_g"), g("ln1_b"), eps)
    qkv = ops.linear_fwd(h, g("wqkv"), g("bqkv"))
    a = ops.attention_fwd(qkv[..., :d], qkv[..., d:2 * d], qkv[..., 2 * d:], n_heads, causal=causal)
    x = x + ops.linear_fwd(a, g("wo"), g("bo"))
    h, _, _ = ops.layernorm_fwd(x, g("ln2_g"), g("ln2_b"), eps)
    f = ops.quick_gelu(ops.linear_fwd(h, g("fc1_w"), g("fc1_b")))
    return x + ops.linear_fwd(f, g("fc2_w"), g("fc2_b"))


def encoder_fwd_partial(p, ids, hidden, layer_begin, layer_end, sample_offset, num_samples,
                        n_layers, n_heads, eps=1e-5, causal=True):
    """Run layers [layer_begin, layer_end) on samples [sample_offset,
    sample_offset + num_samples) of the global batch, reading and writing rows of
    ``hidden`` [global_batch, seq, d] in place (the partial-batch tuple
    (component, layer, #samples) of Sec. 5, with the remaining samples left for
    later calls)."""
    sl = slice(sample_offset, sample_offset + num_samples)
    x = hidden[sl]
    for l in range(layer_begin, layer_end):
        if l == 0:
            x = embed(p, ids[sl])
        elif l <= n_layers:
            x = layer_fwd(p, l - 1, x, n_heads, eps, causal)
        elif l == n_layers + 1:
            x, _, _ = ops.layernorm_fwd(x, p["lnf_g"], p["lnf_b"], eps)
        else:
            raise ValueError(l)
    hidden[sl] = x
    return hidden


def encoder_fwd(p, ids, n_layers, n_heads, eps=1e-5, causal=True):
    """Whole encoder on the whole batch: last hidden state after the final LN."""
    d = p["pos_emb"].shape[1]
    hidden = np.zeros(ids.shape + (d,))
    return encoder_fwd_partial(p, ids, hidden, 0, n_layers + 2, 0, ids.shape[0], n_layers, n_heads, eps, causal)
