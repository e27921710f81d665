"""Arithmetic operators of the chains, float64, plain definitions.

The paper names these operators (Table 3: MatMul, LayerNorm, Softmax, Unary,
Add) without defining them; the definitions are the public mathematical ones.
Weights are stored [out_features, in_features]; linear() computes x . W^T + b.
"""
import numpy as np
from scipy.special import erf as _erf


def linear(x, W, b=None):
    y = x @ W.T            # library matmul as one step
    if b is not None:
        y = y + b
    return y


def layer_norm(x, g, b, eps=1e-5):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)     # biased
    return (x - mu) / np.sqrt(var + eps) * g + b


def rms_norm(x, g, eps=1e-5):
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def group_norm_nchw(x, G, g, b, eps=1e-6):
    B, C, H, W = x.shape
    xg = x.reshape(B, G, (C // G) * H * W)
    mu = xg.mean(axis=-1, keepdims=True)
    var = ((xg - mu) ** 2).mean(axis=-1, keepdims=True)    # biased
    y = ((xg - mu) / np.sqrt(var + eps)).reshape(B, C, H, W)
    return y * g.reshape(1, C, 1, 1) + b.reshape(1, C, 1, 1)


def gelu(x):
    return 0.5 * x * (1.0 + _erf(x / np.sqrt(2.0)))


def silu(x):
    return x / (1.0 + np.exp(-x))


def softmax(s):
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def rope_half_split(x, base=10000.0):
    """x [..., S, D]; pairs (i, i + D/2); position p = index along S."""
    S, D = x.shape[-2], x.shape[-1]
    half = D // 2
    i = np.arange(half, dtype=np.float64)
    theta = base ** (-2.0 * i / D)
    ang = np.arange(S, dtype=np.float64)[:, None] * theta[None, :]
    c, s = np.cos(ang), np.sin(ang)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def attention(q, k, v, scale, add=None, causal=False):
    """q [..., Nq, d], k,v [..., Nk, d]; add broadcastable to [..., Nq, Nk]."""
    s = (q * scale) @ np.swapaxes(k, -1, -2)
    if add is not None:
        s = s + add
    if causal:
        Nq, Nk = s.shape[-2], s.shape[-1]
        i = np.arange(Nq)[:, None]
        j = np.arange(Nk)[None, :]
        s = np.where(j <= i, s, -np.inf)
    p = softmax(s)
    return p @ v, p
