"""Diffusion-UNet spatial-transformer block (the paper's SD-UNet row, Table 7,
names the model; the block definition is the public one).

Readings: GroupNorm eps 1e-6, biased variance; proj_in / proj_out are 1x1
convolutions = per-pixel Linear with bias; LayerNorm eps 1e-5; attention q/k/v
projections without bias, output projection with bias; GEGLU(z) = a * GELU(b)
with [a | b] = z W1^T + b1 (value first, gate second); residuals as written.
The NCHW <-> token rearrangements and the head split / merge are materialised.
"""
from . import views as V
from . import ops as O


def _mha(xq, xkv, wq, wk, wv, wo, bo, h):
    B, Sq, E = xq.shape
    Sk = xkv.shape[1]
    d = E // h
    q = V.apply_chain(O.linear(xq, wq), V.head_split_chain(B, Sq, h, d))
    k = V.apply_chain(O.linear(xkv, wk), V.head_split_chain(B, Sk, h, d))
    v = V.apply_chain(O.linear(xkv, wv), V.head_split_chain(B, Sk, h, d))
    o, _ = O.attention(q, k, v, d ** -0.5)
    o = V.apply_chain(o, V.head_merge_chain(B, Sq, h, d))
    return O.linear(o, wo, bo)


def spatial_transformer(x, ctx, p, G, h, want_all=False):
    """x NCHW [B,C,H,W]; ctx [B, Sc, Dc] -> y NCHW."""
    B, C, H, W = x.shape
    g = O.group_norm_nchw(x, G, p["gn_g"], p["gn_b"])
    t = V.apply_chain(g, V.nchw_to_tokens_chain(B, C, H, W))     # [B, HW, C]
    t = O.linear(t, p["win"], p["bin"])
    t0 = t
    n = O.layer_norm(t, p["ln1_g"], p["ln1_b"])
    t = t + _mha(n, n, p["a1_wq"], p["a1_wk"], p["a1_wv"], p["a1_wo"], p["a1_bo"], h)
    t1 = t
    n = O.layer_norm(t, p["ln2_g"], p["ln2_b"])
    t = t + _mha(n, ctx, p["a2_wq"], p["a2_wk"], p["a2_wv"], p["a2_wo"], p["a2_bo"], h)
    t2 = t
    n = O.layer_norm(t, p["ln3_g"], p["ln3_b"])
    z = O.linear(n, p["ff_w1"], p["ff_b1"])
    F = z.shape[-1] // 2
    t = t + O.linear(z[..., :F] * O.gelu(z[..., F:]), p["ff_w2"], p["ff_b2"])
    t3 = t
    u = O.linear(t, p["wout"], p["bout"])                        # [B, HW, C]
    y = V.apply_chain(u, V.tokens_to_nchw_chain(B, C, H, W)) + x
    if want_all:
        return {"t0": t0, "t1": t1, "t2": t2, "t3": t3, "y": y}
    return y
