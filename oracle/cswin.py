"""Cross-shaped window self-attention of the CSwin Transformer (one of the transformer models whose Reshape /
Transpose count the paper reports, Table 1, and evaluates, Table 7).  TEST INFRASTRUCTURE ONLY: plain numpy float64,
every layout operator materialised.

Readings (the paper gives no definition of the operator; this is the public CSwin one): the input
is what the query-key-value Linear leaves, [B, H*W, 3C] with columns [q | k | v], each of C = heads * d features; the
first half of the channels (heads [0, heads/2)) attends inside vertical stripes of H x sw grid positions, the second
half inside horizontal stripes of sw x W; softmax scale d^-1/2, no bias and no mask; the two halves are Concat-ed
along the channel axis into [B, H*W, C].  Locally-enhanced positional encoding (optional): each half adds, before its
heads are merged, a depth-wise 3 x 3 convolution (weights [C/2, 3, 3], bias [C/2], cross-correlation as in every deep
learning library) of its values laid out as the stripe's Hs x Ws image, zero-padded at the border of the STRIPE (not of
the image): a token's encoding only sees its neighbours inside its own stripe.
"""
import numpy as np
from . import views as V
from . import ops as O


def stripe_shape(H, W, sw, branch):
    """(rows, columns) of one stripe: branch 0 vertical, branch 1 horizontal."""
    return (H, sw) if branch == 0 else (sw, W)


def lepe(v, B, H, W, heads_b, Hs, Ws, w, b):
    """v [B, H*W, Cb] -> [nwin, heads_b, Hs*Ws, d]: the values as stripe images [nwin, Cb, Hs, Ws], a depth-wise 3 x 3
    convolution with zero padding, back to the attention output's layout."""
    Cb = v.shape[-1]
    d = Cb // heads_b
    nwin = B * (H // Hs) * (W // Ws)
    img = V.apply_chain(v, [("permute", (0, 2, 1)), ("reshape", (B, Cb, H // Hs, Hs, W // Ws, Ws)),
                            ("permute", (0, 2, 4, 1, 3, 5)), ("reshape", (nwin, Cb, Hs, Ws))])
    pad = np.zeros((nwin, Cb, Hs + 2, Ws + 2))
    pad[:, :, 1:-1, 1:-1] = img
    out = np.zeros_like(img)
    for dy in range(3):
        for dx in range(3):
            out += pad[:, :, dy:dy + Hs, dx:dx + Ws] * w[None, :, dy, dx, None, None]
    out += b[None, :, None, None]
    return V.apply_chain(out, [("reshape", (nwin, heads_b, d, Hs * Ws)), ("permute", (0, 1, 3, 2))])


def branch_attention(q, k, v, B, H, W, heads_b, Hs, Ws, lepe_w=None, lepe_b=None):
    """q, k, v [B, H*W, Cb] (one half of the channels) -> [B, H*W, Cb]: partition into Hs x Ws stripes, split the heads,
    attend inside each stripe (plus the positional encoding of the values, when given), merge heads and stripes again."""
    Cb = q.shape[-1]
    d = Cb // heads_b
    nwin, S = B * (H // Hs) * (W // Ws), Hs * Ws
    part = []
    for t in (q, k, v):
        t = V.apply_chain(t, V.stripe_partition_chain(B, H, W, Cb, Hs, Ws))
        part.append(V.apply_chain(t, V.head_split_chain(nwin, S, heads_b, d)))
    o, _ = O.attention(part[0], part[1], part[2], d ** -0.5)
    if lepe_w is not None:
        o = o + lepe(v, B, H, W, heads_b, Hs, Ws, lepe_w, lepe_b)
    o = V.apply_chain(o, V.head_merge_chain(nwin, S, heads_b, d))
    return V.apply_chain(o, V.stripe_merge_chain(B, H, W, Cb, Hs, Ws))


def cross_window_attention(qkv, B, H, W, C, heads, sw, lepe_w=None, lepe_b=None):
    """qkv [B, H*W, 3C] -> [B, H*W, C]; lepe_w [C, 3, 3], lepe_b [C]: the two halves' convolutions, first half first."""
    t = V.reshape(qkv, (B, H * W, 3, C))
    q, k, v = [V.reshape(V.slice_(t, 2, i, i + 1), (B, H * W, C)) for i in range(3)]
    Cb = C // 2
    halves = []
    for branch in range(2):
        Hs, Ws = stripe_shape(H, W, sw, branch)
        sl = [V.slice_(x, 2, branch * Cb, (branch + 1) * Cb) for x in (q, k, v)]
        cs = slice(branch * Cb, (branch + 1) * Cb)
        halves.append(branch_attention(sl[0], sl[1], sl[2], B, H, W, heads // 2, Hs, Ws,
                                       None if lepe_w is None else lepe_w[cs], None if lepe_w is None else lepe_b[cs]))
    return V.concat(halves, 2)


def cswin_block(x, p, B, H, W, C, heads, sw, want_all=False):
    """One CSwin block, x [B, H*W, C] -> [B, H*W, C] (the public definition: LayerNorm eps 1e-5, fused q | k | v Linear
    with bias, cross-shaped window attention with its positional encoding, output Linear, residual, LayerNorm, MLP of
    width ratio * C with the exact GELU, residual).  p: ln1_g, ln1_b, wqkv [3C, C], bqkv, lepe_w [C, 3, 3], lepe_b,
    wproj, bproj, ln2_g, ln2_b, w1, b1, w2, b2."""
    n1 = O.layer_norm(x, p["ln1_g"], p["ln1_b"])
    qkv = O.linear(n1, p["wqkv"], p["bqkv"])
    a = cross_window_attention(qkv, B, H, W, C, heads, sw, p["lepe_w"], p["lepe_b"])
    x1 = x + O.linear(a, p["wproj"], p["bproj"])
    n2 = O.layer_norm(x1, p["ln2_g"], p["ln2_b"])
    hid = O.gelu(O.linear(n2, p["w1"], p["b1"]))
    y = x1 + O.linear(hid, p["w2"], p["b2"])
    if want_all:
        return {"qkv": qkv, "attn": a, "x1": x1, "y": y}
    return y
