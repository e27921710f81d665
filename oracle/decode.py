"""GPT-NeoX / Pythia-style layer at a decode step: one new token per sequence against a key / value cache (the paper
evaluates Pythia, Table 7; at one token per step every Linear is a matrix-vector product and the layer is bound by
memory traffic, so a materialised layout operator costs relatively most).  TEST INFRASTRUCTURE ONLY: plain numpy
float64, every layout operator materialised.

Readings (the paper gives no layer definition; this is the public GPT-NeoX one): LayerNorm eps 1e-5 with bias; the
fused query-key-value Linear has 3E outputs ordered [head][q | k | v][d] (view [B, 1, h, 3d], then three Slices and a
Permute to [B, h, 1, d]); rotary embedding on the first `rot` features of q and k only, half-split pairing
(i, i + rot/2), theta_i = base^(-2i/rot), at position L = number of cached tokens; the new key / value are Concat-ed
behind the cache along the token axis; softmax scale d^-1/2, no mask (every cached token is in the past); parallel
residual y = x + dense(attention(LN1 x)) + MLP(LN2 x), MLP = W2 gelu(W1 . + b1) + b2 with the exact (erf) GELU.
"""
import numpy as np
from . import views as V
from . import ops as O


def rope_partial(x, pos, rot, base=10000.0):
    """x [..., d] at token position pos: features [0, rot) rotated in pairs (i, i + rot/2), the rest untouched."""
    half = rot // 2
    theta = base ** (-2.0 * np.arange(half, dtype=np.float64) / rot)
    c, s = np.cos(pos * theta), np.sin(pos * theta)
    a, b = x[..., :half], x[..., half:rot]
    return np.concatenate([a * c - b * s, b * c + a * s, x[..., rot:]], axis=-1)


def neox_decode_step(x, p, k_cache, v_cache, h, rot, base=10000.0, want_all=False):
    """x [B, E] (the new token's hidden state), k_cache / v_cache [B, h, L, d] (keys already rotated).
    Returns y [B, E] and the caches grown by one token, [B, h, L + 1, d]."""
    B, E = x.shape
    d = E // h
    L = k_cache.shape[2]
    n1 = O.layer_norm(x, p["ln1_g"], p["ln1_b"])
    qkv = V.reshape(O.linear(n1, p["wqkv"], p["bqkv"]), (B, 1, h, 3 * d))
    q = V.permute(V.slice_(qkv, 3, 0, d), (0, 2, 1, 3))                 # [B, h, 1, d]
    k = V.permute(V.slice_(qkv, 3, d, 2 * d), (0, 2, 1, 3))
    v = V.permute(V.slice_(qkv, 3, 2 * d, 3 * d), (0, 2, 1, 3))
    q = rope_partial(q, L, rot, base)
    k = rope_partial(k, L, rot, base)
    K = V.concat([k_cache, k], 2)
    Vv = V.concat([v_cache, v], 2)
    o, _ = O.attention(q, K, Vv, d ** -0.5)                             # [B, h, 1, d]
    o = V.reshape(V.permute(o, (0, 2, 1, 3)), (B, E))
    a = O.linear(o, p["wdense"], p["bdense"])
    n2 = O.layer_norm(x, p["ln2_g"], p["ln2_b"])
    hid = O.gelu(O.linear(n2, p["w1"], p["b1"]))
    m = O.linear(hid, p["w2"], p["b2"])
    y = x + a + m
    if want_all:
        return {"qkv": qkv.reshape(B, 3 * E), "q": q, "k": k, "v": v, "o": o, "attn": x + a, "hid": hid, "y": y, "K": K, "V": Vv}
    return y, K, Vv
