"""Elementary operations of the oracle, float64 numpy (test infrastructure only).

Each function is the plain definition of the operation named in the hot-path
list (LayerNorm, linear projection, softmax attention, GELU variants, SiLU);
the paper (Sec. 2.1, Sec. 4.1) only names the backbones, so these follow the
public definitions of those architectures.
"""
from __future__ import annotations

import math

import numpy as np

try:  # vectorised erf; math.erf is used as an independent check in the tests
    from scipy.special import erf as _erf
except Exception:  # pragma: no cover
    _erf = np.vectorize(math.erf)


# ---------------------------------------------------------------- LayerNorm
def layernorm_fwd(x, gamma=None, beta=None, eps=1e-5):
    """y = (x - mean) / sqrt(var + eps) * gamma + beta over the last axis,
    biased variance.  gamma/beta None = non-affine.  Returns (y, xhat, rstd)."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = xc * rstd
    y = xhat
    if gamma is not None:
        y = y * gamma
    if beta is not None:
        y = y + beta
    return y, xhat, rstd


def layernorm_bwd(dy, xhat, rstd, gamma=None):
    """Returns (dx, dgamma, dbeta); dgamma/dbeta are sums over all rows."""
    dxhat = dy * gamma if gamma is not None else dy
    m1 = dxhat.mean(axis=-1, keepdims=True)
    m2 = (dxhat * xhat).mean(axis=-1, keepdims=True)
    dx = rstd * (dxhat - m1 - xhat * m2)
    red = tuple(range(dy.ndim - 1))
    dgamma = (dy * xhat).sum(axis=red)
    dbeta = dy.sum(axis=red)
    return dx, dgamma, dbeta


# ------------------------------------------------------------------- linear
def linear_fwd(x, w, b=None):
    """y = x @ w.T (+ b); w is [out, in]."""
    y = x @ w.T
    if b is not None:
        y = y + b
    return y


def linear_bwd(dy, x, w):
    """Returns (dx, dw, db) for y = x @ w.T + b."""
    dx = dy @ w
    dy2 = dy.reshape(-1, dy.shape[-1])
    x2 = x.reshape(-1, x.shape[-1])
    dw = dy2.T @ x2
    db = dy2.sum(axis=0)
    return dx, dw, db


# -------------------------------------------------------------- activations
def gelu_erf(z):
    return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))


def gelu_erf_grad(z):
    return 0.5 * (1.0 + _erf(z / math.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)


_A = math.sqrt(2.0 / math.pi)
_C = 0.044715


def gelu_tanh(z):
    return 0.5 * z * (1.0 + np.tanh(_A * (z + _C * z ** 3)))


def gelu_tanh_grad(z):
    t = np.tanh(_A * (z + _C * z ** 3))
    return 0.5 * (1.0 + t) + 0.5 * z * (1.0 - t * t) * _A * (1.0 + 3.0 * _C * z * z)


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def quick_gelu(z):
    return z * sigmoid(1.702 * z)


def silu(z):
    return z * sigmoid(z)


def silu_grad(z):
    s = sigmoid(z)
    return s * (1.0 + z * (1.0 - s))


# ---------------------------------------------------------------- attention
def softmax_rows(s):
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def _split_heads(t, n_heads):
    B, N, D = t.shape
    return t.reshape(B, N, n_heads, D // n_heads)


def attention_probs(q, k, n_heads, causal=False):
    """Generator over (b, h, P) with P = softmax(q k^T / sqrt(dh)) [Nq, Nk]."""
    qh, kh = _split_heads(q, n_heads), _split_heads(k, n_heads)
    B, Nq, H, dh = qh.shape
    Nk = kh.shape[1]
    scale = 1.0 / math.sqrt(dh)
    for b in range(B):
        for h in range(H):
            s = (qh[b, :, h, :] @ kh[b, :, h, :].T) * scale
            if causal:
                s = np.where(np.arange(Nk)[None, :] > np.arange(Nq)[:, None], -np.inf, s)
            yield b, h, softmax_rows(s)


def attention_fwd(q, k, v, n_heads, causal=False):
    """q [B,Nq,d], k,v [B,Nk,d] -> o [B,Nq,d]; per (batch, head) softmax(q k^T/sqrt(dh)) v."""
    vh = _split_heads(v, n_heads)
    B, Nq, d = q.shape
    o = np.empty((B, Nq, n_heads, d // n_heads))
    for b, h, p in attention_probs(q, k, n_heads, causal):
        o[b, :, h, :] = p @ vh[b, :, h, :]
    return o.reshape(B, Nq, d)


def attention_bwd(do, q, k, v, n_heads, causal=False):
    """Returns (dq, dk, dv).  P is recomputed from q, k (same definition)."""
    qh, kh, vh = (_split_heads(t, n_heads) for t in (q, k, v))
    doh = _split_heads(do, n_heads)
    dh = qh.shape[-1]
    scale = 1.0 / math.sqrt(dh)
    dq, dk, dv = np.zeros_like(qh), np.zeros_like(kh), np.zeros_like(vh)
    for b, h, p in attention_probs(q, k, n_heads, causal):
        dob = doh[b, :, h, :]
        dp = dob @ vh[b, :, h, :].T
        ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
        dq[b, :, h, :] = (ds @ kh[b, :, h, :]) * scale
        dk[b, :, h, :] = (ds.T @ qh[b, :, h, :]) * scale
        dv[b, :, h, :] = p.T @ dob
    return dq.reshape(q.shape), dk.reshape(k.shape), dv.reshape(v.shape)
