"""ViT encoder block (the paper's ViT row, Tables 1 and 7, names the model; the block definition is the public
pre-norm one).  TEST INFRASTRUCTURE ONLY.

Readings: LayerNorm eps 1e-5, biased variance; one fused q|k|v projection with bias, output projection with bias;
full (global) softmax attention over all S tokens (class token included: it is just a token), scale D^-1/2; MLP with
exact (erf) GELU; residuals as written.  The [B,S,3,H,D] -> [3,B,H,S,D] split and the head merge are materialised.
"""
from . import views as V
from . import ops as O


def vit_block(x, p, h, want_all=False):
    """x [B, S, E] -> y [B, S, E]."""
    B, S, E = x.shape
    d = E // h
    n1 = O.layer_norm(x, p["ln1_g"], p["ln1_b"])
    qkv = O.linear(n1, p["wqkv"], p["bqkv"])                              # [B, S, 3E]
    t = V.apply_chain(qkv, V.qkv_split_chain(B, S, h, d))                  # [3, B, h, S, d]
    o, P = O.attention(t[0].copy(), t[1].copy(), t[2].copy(), d ** -0.5)
    o = V.apply_chain(o, V.head_merge_chain(B, S, h, d))                   # [B, S, E]
    x1 = x + O.linear(o, p["wo"], p["bo"])
    n2 = O.layer_norm(x1, p["ln2_g"], p["ln2_b"])
    hid = O.gelu(O.linear(n2, p["w1"], p["b1"]))
    y = x1 + O.linear(hid, p["w2"], p["b2"])
    if want_all:
        return {"qkv": qkv, "P": P, "o": o, "x1": x1, "hid": hid, "y": y}
    return y
