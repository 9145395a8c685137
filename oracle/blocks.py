"""Transformer blocks and the stage built from them, float64 (test infrastructure only).

A stage is a contiguous range of backbone layers processing one micro-batch
(Sec. 4.1; its cost is the sum of the layers' forward and backward times,
Eq. for T_0).  The paper names the backbones (U-Net and transformer backbones,
Sec. 2.1; DiT-type backbones in the conclusion) without defining their
arithmetic; the definitions below are the public pre-norm formulations.

Parameters are dicts keyed by name (order-free); see each function for names.
"""
from __future__ import annotations

import numpy as np

from . import ops


# =================================================== U-Net-style block
def unet_block_fwd(p, x, ctx, n_heads, eps=1e-5):
    """Self-attention, cross-attention to frozen text-encoder states (Sec. 2.1)
    and a GeGLU feed-forward, each pre-normed with a residual connection.

    p: ln{1,2,3}_{g,b}, attn1_wqkv [3d,d] (rows q|k|v, no bias), attn1_wo, attn1_bo,
       attn2_wq [d,d], attn2_wkv [2d,dc] (rows k|v), attn2_wo, attn2_bo,
       ff_w1 [2*inner,d], ff_b1, ff_w2 [d,inner], ff_b2.
    GeGLU: first half of u is the value, the second half goes through erf-GELU.
    Returns (y, cache)."""
    d = x.shape[-1]
    c = {"x": x, "ctx": ctx}
    h1, c["xh1"], c["rs1"] = ops.layernorm_fwd(x, p["ln1_g"], p["ln1_b"], eps)
    qkv = ops.linear_fwd(h1, p["attn1_wqkv"])
    q, k, v = qkv[..., :d], qkv[..., d:2 * d], qkv[..., 2 * d:]
    a1 = ops.attention_fwd(q, k, v, n_heads)
    x1 = x + ops.linear_fwd(a1, p["attn1_wo"], p["attn1_bo"])
    c.update(h1=h1, q1=q, k1=k, v1=v, a1=a1)

    h2, c["xh2"], c["rs2"] = ops.layernorm_fwd(x1, p["ln2_g"], p["ln2_b"], eps)
    q2 = ops.linear_fwd(h2, p["attn2_wq"])
    kv2 = ops.linear_fwd(ctx, p["attn2_wkv"])
    k2, v2 = kv2[..., :d], kv2[..., d:]
    a2 = ops.attention_fwd(q2, k2, v2, n_heads)
    x2 = x1 + ops.linear_fwd(a2, p["attn2_wo"], p["attn2_bo"])
    c.update(h2=h2, q2=q2, k2=k2, v2=v2, a2=a2)

    h3, c["xh3"], c["rs3"] = ops.layernorm_fwd(x2, p["ln3_g"], p["ln3_b"], eps)
    u = ops.linear_fwd(h3, p["ff_w1"], p["ff_b1"])
    inner = u.shape[-1] // 2
    g = u[..., :inner] * ops.gelu_erf(u[..., inner:])
    y = x2 + ops.linear_fwd(g, p["ff_w2"], p["ff_b2"])
    c.update(h3=h3, u=u, g=g)
    return y, c


def unet_block_bwd(p, c, dy, n_heads):
    """Returns (dx, grads dict).  No gradient flows to ctx (frozen encoder output)."""
    gr = {}
    inner = c["u"].shape[-1] // 2
    # feed-forward
    dg, gr["ff_w2"], gr["ff_b2"] = ops.linear_bwd(dy, c["g"], p["ff_w2"])
    val, gate = c["u"][..., :inner], c["u"][..., inner:]
    du = np.concatenate([dg * ops.gelu_erf(gate), dg * val * ops.gelu_erf_grad(gate)], axis=-1)
    dh3, gr["ff_w1"], gr["ff_b1"] = ops.linear_bwd(du, c["h3"], p["ff_w1"])
    dx2n, gr["ln3_g"], gr["ln3_b"] = ops.layernorm_bwd(dh3, c["xh3"], c["rs3"], p["ln3_g"])
    dx2 = dy + dx2n
    # cross-attention
    da2, gr["attn2_wo"], gr["attn2_bo"] = ops.linear_bwd(dx2, c["a2"], p["attn2_wo"])
    dq2, dk2, dv2 = ops.attention_bwd(da2, c["q2"], c["k2"], c["v2"], n_heads)
    dh2, gr["attn2_wq"], _ = ops.linear_bwd(dq2, c["h2"], p["attn2_wq"])
    _, gr["attn2_wkv"], _ = ops.linear_bwd(np.concatenate([dk2, dv2], axis=-1), c["ctx"], p["attn2_wkv"])
    dx1n, gr["ln2_g"], gr["ln2_b"] = ops.layernorm_bwd(dh2, c["xh2"], c["rs2"], p["ln2_g"])
    dx1 = dx2 + dx1n
    # self-attention
    da1, gr["attn1_wo"], gr["attn1_bo"] = ops.linear_bwd(dx1, c["a1"], p["attn1_wo"])
    dq, dk, dv = ops.attention_bwd(da1, c["q1"], c["k1"], c["v1"], n_heads)
    dh1, gr["attn1_wqkv"], _ = ops.linear_bwd(np.concatenate([dq, dk, dv], axis=-1), c["h1"], p["attn1_wqkv"])
    dxn, gr["ln1_g"], gr["ln1_b"] = ops.layernorm_bwd(dh1, c["xh1"], c["rs1"], p["ln1_g"])
    return dx1 + dxn, gr


# =================================================== DiT-style adaLN-zero block
def dit_block_fwd(p, x, cond, n_heads, eps=1e-6, gelu_tanh=True):
    """m = SiLU(cond) W_ada^T + b_ada, split into (shift1, scale1, gate1, shift2,
    scale2, gate2); modulated non-affine LayerNorm before self-attention and
    before the 4x MLP; each branch gated into the residual.

    p: ada_w [6d,d], ada_b, attn_wqkv [3d,d], attn_bqkv, attn_wo, attn_bo,
       fc1_w [ff,d], fc1_b, fc2_w [d,ff], fc2_b."""
    d = x.shape[-1]
    act = ops.gelu_tanh if gelu_tanh else ops.gelu_erf
    c = {"x": x, "cond": cond, "gelu_tanh": gelu_tanh}
    sc_in = ops.silu(cond)
    m = ops.linear_fwd(sc_in, p["ada_w"], p["ada_b"])          # [B, 6d]
    sh1, sc1, g1, sh2, sc2, g2 = (m[:, None, i * d:(i + 1) * d] for i in range(6))
    _, xh1, rs1 = ops.layernorm_fwd(x, None, None, eps)
    h1 = xh1 * (1.0 + sc1) + sh1
    qkv = ops.linear_fwd(h1, p["attn_wqkv"], p["attn_bqkv"])
    q, k, v = qkv[..., :d], qkv[..., d:2 * d], qkv[..., 2 * d:]
    a = ops.attention_fwd(q, k, v, n_heads)
    o = ops.linear_fwd(a, p["attn_wo"], p["attn_bo"])
    x1 = x + g1 * o
    _, xh2, rs2 = ops.layernorm_fwd(x1, None, None, eps)
    h2 = xh2 * (1.0 + sc2) + sh2
    f1 = ops.linear_fwd(h2, p["fc1_w"], p["fc1_b"])
    f = act(f1)
    f2 = ops.linear_fwd(f, p["fc2_w"], p["fc2_b"])
    y = x1 + g2 * f2
    c.update(sc_in=sc_in, m=m, xh1=xh1, rs1=rs1, h1=h1, q=q, k=k, v=v, a=a, o=o,
             xh2=xh2, rs2=rs2, h2=h2, f1=f1, f=f, f2=f2)
    return y, c


def dit_block_bwd(p, c, dy, n_heads):
    """Returns (dx, dcond, grads dict)."""
    d = c["x"].shape[-1]
    gr = {}
    m = c["m"]
    sh1, sc1, g1, sh2, sc2, g2 = (m[:, None, i * d:(i + 1) * d] for i in range(6))
    act_grad = ops.gelu_tanh_grad if c["gelu_tanh"] else ops.gelu_erf_grad
    # MLP branch
    dg2 = (dy * c["f2"]).sum(axis=1)
    df2 = dy * g2
    df, gr["fc2_w"], gr["fc2_b"] = ops.linear_bwd(df2, c["f"], p["fc2_w"])
    df1 = df * act_grad(c["f1"])
    dh2, gr["fc1_w"], gr["fc1_b"] = ops.linear_bwd(df1, c["h2"], p["fc1_w"])
    dsc2 = (dh2 * c["xh2"]).sum(axis=1)
    dsh2 = dh2.sum(axis=1)
    dx1n, _, _ = ops.layernorm_bwd(dh2 * (1.0 + sc2), c["xh2"], c["rs2"], None)
    dx1 = dy + dx1n
    # attention branch
    dg1 = (dx1 * c["o"]).sum(axis=1)
    do = dx1 * g1
    da, gr["attn_wo"], gr["attn_bo"] = ops.linear_bwd(do, c["a"], p["attn_wo"])
    dq, dk, dv = ops.attention_bwd(da, c["q"], c["k"], c["v"], n_heads)
    dh1, gr["attn_wqkv"], gr["attn_bqkv"] = ops.linear_bwd(
        np.concatenate([dq, dk, dv], axis=-1), c["h1"], p["attn_wqkv"])
    dsc1 = (dh1 * c["xh1"]).sum(axis=1)
    dsh1 = dh1.sum(axis=1)
    dxn, _, _ = ops.layernorm_bwd(dh1 * (1.0 + sc1), c["xh1"], c["rs1"], None)
    dx = dx1 + dxn
    # conditioning path
    dm = np.concatenate([dsh1, dsc1, dg1, dsh2, dsc2, dg2], axis=-1)   # [B, 6d]
    dsc_in, gr["ada_w"], gr["ada_b"] = ops.linear_bwd(dm, c["sc_in"], p["ada_w"])
    dcond = dsc_in * ops.silu_grad(c["cond"])
    return dx, dcond, gr


# =================================================== stage = contiguous blocks
def _block_params(params, b):
    pre = f"block{b}."
    return {k[len(pre):]: v for k, v in params.items() if k.startswith(pre)}


def stage_fwd(kind, params, x, ctx_or_cond, n_blocks, n_heads, eps, gelu_tanh=True):
    """Forward of the stage's blocks in order.  Returns (y, caches)."""
    caches = []
    for b in range(n_blocks):
        p = _block_params(params, b)
        if kind == "unet_xattn_geglu":
            x, c = unet_block_fwd(p, x, ctx_or_cond, n_heads, eps)
        elif kind == "dit_adaln_zero":
            x, c = dit_block_fwd(p, x, ctx_or_cond, n_heads, eps, gelu_tanh)
        else:
            raise ValueError(kind)
        caches.append(c)
    return x, caches


def stage_bwd(kind, params, caches, dy, n_heads):
    """Backward through the blocks in reverse.  Returns (dx, dcond or None, grads)
    with grads keyed like params; dcond is summed over the blocks."""
    grads, dcond = {}, None
    for b in reversed(range(len(caches))):
        p = _block_params(params, b)
        if kind == "unet_xattn_geglu":
            dy, gr = unet_block_bwd(p, caches[b], dy, n_heads)
        else:
            dy, dc, gr = dit_block_bwd(p, caches[b], dy, n_heads)
            dcond = dc if dcond is None else dcond + dc
        for k, v in gr.items():
            grads[f"block{b}.{k}"] = v
    return dy, dcond, grads


def stage_self_conditioned(kind, params, x_sc, x, ctx_or_cond, dy, n_blocks, n_heads, eps, gelu_tanh=True):
    """Self-conditioning seen from one stage (Sec. 4.3): one additional forward
    pass with the same parameters on the same device, nothing kept from it,
    followed by the ordinary forward and backward.  Returns
    (y_sc, y, dx, dcond, grads)."""
    y_sc, _ = stage_fwd(kind, params, x_sc, ctx_or_cond, n_blocks, n_heads, eps, gelu_tanh)
    y, caches = stage_fwd(kind, params, x, ctx_or_cond, n_blocks, n_heads, eps, gelu_tanh)
    dx, dcond, grads = stage_bwd(kind, params, caches, dy, n_heads)
    return y_sc, y, dx, dcond, grads
