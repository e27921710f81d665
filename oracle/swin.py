"""Swin block, patch merging, patch embedding, stage chain and full net,
written as the explicit operator chain: every Reshape / Permute / roll / window
partition / reverse / head split / merge is materialised through oracle.views.

The paper names Swin as a workload (Table 1, Table 7) but does not define it;
the block follows the public Swin definition with these readings:
  * LayerNorm eps 1e-5, biased variance; GELU is the erf form.
  * Forward cyclic shift rolls both spatial axes by -s, the reverse by +s.
  * Relative-position bias: table of (2w-1)^2 rows x h columns,
    bias[hh, i, j] = table[(yi - yj + w - 1) * (2w - 1) + (xi - xj + w - 1), hh].
  * Shift mask: regions on the shifted grid with boundaries H-w and H-s
    (same for W); pairs of tokens in different regions get -100 added.
  * Block k of a stage shifts by 0 (k even) or w//2 (k odd); a stage whose
    resolution equals the window never shifts.
  * Patch merging: 2x2 gather with channel block k = 2*dw + dh, LayerNorm(4C),
    Linear 4C -> 2C without bias.
  * Patch embedding: 4x4 stride-4 unfold with column order (c, py, px),
    Linear + bias, LayerNorm.
  * Head: LayerNorm, mean over tokens, Linear + bias.
"""
import numpy as np
from . import views as V
from . import ops as O


def rel_pos_index(w):
    """[N, N] int64 row index into the (2w-1)^2 table."""
    N = w * w
    idx = np.empty((N, N), dtype=np.int64)
    for i in range(N):
        yi, xi = divmod(i, w)
        for j in range(N):
            yj, xj = divmod(j, w)
            idx[i, j] = (yi - yj + w - 1) * (2 * w - 1) + (xi - xj + w - 1)
    return idx


def rel_pos_bias(table, w, h):
    """table [(2w-1)^2, h] -> bias [h, N, N] (Gather, Reshape, Permute materialised)."""
    N = w * w
    g = table[rel_pos_index(w).reshape(-1)]          # gather rows: [N*N, h]
    g = V.reshape(g, (N, N, h))
    return V.permute(g, (2, 0, 1))


def shift_mask(H, W, w, s):
    """[nW, N, N] additive mask for shifted windows (0 or -100)."""
    nW = (H // w) * (W // w)
    N = w * w
    if s == 0:
        return np.zeros((nW, N, N))
    region = np.zeros((1, H, W, 1))
    cnt = 0
    for ys in (slice(0, H - w), slice(H - w, H - s), slice(H - s, H)):
        for xs in (slice(0, W - w), slice(W - w, W - s), slice(W - s, W)):
            region[:, ys, xs, :] = cnt
            cnt += 1
    rw = V.apply_chain(region, V.window_partition_chain(1, H, W, 1, w, 0)).reshape(nW, N)
    diff = rw[:, :, None] != rw[:, None, :]
    return np.where(diff, -100.0, 0.0)


def window_attention(u_win, p, w, h, mask):
    """u_win [B_, N, C] -> dict with qkv, P, o ([B_, N, C] after head merge)."""
    B_, N, C = u_win.shape
    d = C // h
    qkv = O.linear(u_win, p["wqkv"], p["bqkv"])                  # [B_, N, 3C]
    t = V.apply_chain(qkv, V.qkv_split_chain(B_, N, h, d))       # [3, B_, h, N, d]
    q, k, v = t[0].copy(), t[1].copy(), t[2].copy()
    add = rel_pos_bias(p["rpb_table"], w, h)[None]               # [1, h, N, N]
    if mask is not None:
        nW = mask.shape[0]
        add = add + np.tile(mask, (B_ // nW, 1, 1))[:, None]     # window index mod nW
    o, P = O.attention(q, k, v, d ** -0.5, add=add)              # [B_, h, N, d]
    o = V.apply_chain(o, V.head_merge_chain(B_, N, h, d))        # [B_, N, C]
    return {"qkv": qkv, "P": P, "o": o}


def swin_block(x, p, H, W, w, h, s, want_all=False):
    """x [B, L, C] -> y [B, L, C]."""
    B, L, C = x.shape
    assert L == H * W and H % w == 0 and W % w == 0
    u = O.layer_norm(x, p["ln1_g"], p["ln1_b"])
    u = V.reshape(u, (B, H, W, C))
    u_win = V.apply_chain(u, V.window_partition_chain(B, H, W, C, w, s))
    mask = shift_mask(H, W, w, s) if s else None
    a = window_attention(u_win, p, w, h, mask)
    pr = O.linear(a["o"], p["wproj"], p["bproj"])                # [B_, N, C]
    pr = V.apply_chain(pr, V.window_reverse_chain(B, H, W, C, w, s))
    x1 = x + V.reshape(pr, (B, L, C))
    n2 = O.layer_norm(x1, p["ln2_g"], p["ln2_b"])
    hid = O.gelu(O.linear(n2, p["w1"], p["b1"]))
    y = x1 + O.linear(hid, p["w2"], p["b2"])
    if want_all:
        return {"u_win": u_win, "qkv": a["qkv"], "P": a["P"], "o": a["o"],
                "x1": x1, "hid": hid, "y": y}
    return y


def patch_merge(x, p, H, W):
    """x [B, H*W, C] -> [B, H*W/4, 2C]."""
    B, L, C = x.shape
    g = V.apply_chain(V.reshape(x, (B, H, W, C)), V.patch_merge_chain(B, H, W, C))
    g = V.reshape(g, (B, L // 4, 4 * C))
    g = O.layer_norm(g, p["ln_g"], p["ln_b"])
    return O.linear(g, p["w"], None)


def patch_embed(img, p, patch):
    """img NCHW -> [B, (H/p)*(W/p), E]."""
    B, Cin, H, W = img.shape
    a = V.apply_chain(img, V.patch_embed_chain(B, Cin, H, W, patch))
    t = O.linear(a, p["w"], p["b"])
    return O.layer_norm(t, p["ln_g"], p["ln_b"])


def block_shift(k, res, w):
    return 0 if (k % 2 == 0 or res <= w) else w // 2


def swin_stage(x, blocks, H, W, w, h):
    for k, p in enumerate(blocks):
        x = swin_block(x, p, H, W, w, h, block_shift(k, min(H, W), w))
    return x


def swin_net(img, net, patch, w, heads):
    """net: {"embed", "stages": [[block params]...], "merges": [...], "head"}.
    Returns (feature map before pooling [B, L_last, C_last], logits)."""
    B, _, Hi, Wi = img.shape
    H, W = Hi // patch, Wi // patch
    x = patch_embed(img, net["embed"], patch)
    for si, blocks in enumerate(net["stages"]):
        x = swin_stage(x, blocks, H, W, w, heads[si])
        if si + 1 < len(net["stages"]):
            x = patch_merge(x, net["merges"][si], H, W)
            H, W = H // 2, W // 2
    hp = net["head"]
    f = O.layer_norm(x, hp["ln_g"], hp["ln_b"])
    pooled = f.mean(axis=1)
    return f, O.linear(pooled, hp["w"], hp["b"])
