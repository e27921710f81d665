"""View primitives, each materialised (Sec. 2.2, Sec. 3.2.1 of the paper).

A "view op" is one of
    ("reshape", new_shape)            same linear order, new dimensions
    ("permute", perm)                 output axis k is input axis perm[k]
    ("roll", axis, r)                 out[i] = in[(i - r) mod n] along axis
    ("slice", axis, start, stop, step)
Reading of the garbled Transpose formula in Sec. 3.2.1: output axis k takes
input axis perm[k] (the numpy / ONNX convention).

index_map() applies a chain to an iota tensor, so that the result holds, for
every output element, the linear offset of the source element it copies.  That
array is the definition the composed index maps of the library are compared
with, element for element.
"""
import numpy as np


def reshape(a, shape):
    shape = tuple(int(s) for s in shape)
    return np.ascontiguousarray(a).reshape(shape).copy()


def permute(a, perm):
    perm = tuple(int(p) for p in perm)
    assert sorted(perm) == list(range(a.ndim))
    return np.ascontiguousarray(np.transpose(a, perm))


def roll(a, axis, r):
    n = a.shape[axis]
    out = np.empty_like(a)
    for i in range(n):
        src = (i - r) % n
        dst_ix = [slice(None)] * a.ndim
        src_ix = [slice(None)] * a.ndim
        dst_ix[axis] = i
        src_ix[axis] = src
        out[tuple(dst_ix)] = a[tuple(src_ix)]
    return out


def slice_(a, axis, start, stop, step=1):
    ix = [slice(None)] * a.ndim
    ix[axis] = slice(start, stop, step)
    return np.ascontiguousarray(a[tuple(ix)])


def concat(parts, axis):
    return np.ascontiguousarray(np.concatenate(parts, axis=axis))


def apply_chain(a, chain):
    for op in chain:
        kind = op[0]
        if kind == "reshape":
            a = reshape(a, op[1])
        elif kind == "permute":
            a = permute(a, op[1])
        elif kind == "roll":
            a = roll(a, op[1], op[2])
        elif kind == "slice":
            a = slice_(a, op[1], op[2], op[3], op[4] if len(op) > 4 else 1)
        else:
            raise ValueError(kind)
    return a


def index_map(src_shape, chain):
    n = int(np.prod(src_shape))
    iota = np.arange(n, dtype=np.int64).reshape(tuple(src_shape))
    return apply_chain(iota, chain)


# ---- the named rearrangements of the five chains, as chains of primitives ----

def window_partition_chain(B, H, W, C, w, s):
    """[B,H,W,C] -> [B*nW, w*w, C]; cyclic shift by -s on both axes first."""
    chain = []
    if s:
        chain += [("roll", 1, -s), ("roll", 2, -s)]
    chain += [("reshape", (B, H // w, w, W // w, w, C)),
              ("permute", (0, 1, 3, 2, 4, 5)),
              ("reshape", (B * (H // w) * (W // w), w * w, C))]
    return chain


def window_reverse_chain(B, H, W, C, w, s):
    """[B*nW, w*w, C] -> [B,H,W,C]; cyclic shift by +s afterwards."""
    chain = [("reshape", (B, H // w, W // w, w, w, C)),
             ("permute", (0, 1, 3, 2, 4, 5)),
             ("reshape", (B, H, W, C))]
    if s:
        chain += [("roll", 1, s), ("roll", 2, s)]
    return chain


def qkv_split_chain(B_, N, h, d):
    """[B_, N, 3*h*d] -> [3, B_, h, N, d]."""
    return [("reshape", (B_, N, 3, h, d)), ("permute", (2, 0, 3, 1, 4))]


def head_split_chain(B, S, h, d):
    """[B, S, h*d] -> [B, h, S, d]."""
    return [("reshape", (B, S, h, d)), ("permute", (0, 2, 1, 3))]


def head_merge_chain(B, S, h, d):
    """[B, h, S, d] -> [B, S, h*d]."""
    return [("permute", (0, 2, 1, 3)), ("reshape", (B, S, h * d))]


def patch_merge_chain(B, H, W, C):
    """[B,H,W,C] -> [B, H/2, W/2, 4C], channel block k = 2*dw + dh holds
    X[b, 2*y2+dh, 2*x2+dw, :] (four strided slices concatenated = SpaceToDepth)."""
    return [("reshape", (B, H // 2, 2, W // 2, 2, C)),
            ("permute", (0, 1, 3, 4, 2, 5)),
            ("reshape", (B, H // 2, W // 2, 4 * C))]


def patch_embed_chain(B, Cin, H, W, p):
    """NCHW image -> [B, (H/p)*(W/p), Cin*p*p], column order (c, py, px)."""
    return [("reshape", (B, Cin, H // p, p, W // p, p)),
            ("permute", (0, 2, 4, 1, 3, 5)),
            ("reshape", (B, (H // p) * (W // p), Cin * p * p))]


def nchw_to_tokens_chain(B, C, H, W):
    return [("reshape", (B, C, H * W)), ("permute", (0, 2, 1))]


def tokens_to_nchw_chain(B, C, H, W):
    return [("permute", (0, 2, 1)), ("reshape", (B, C, H, W))]


def stripe_partition_chain(B, H, W, C, Hs, Ws):
    """Tokens [B, H*W, C] -> stripes [B*(H/Hs)*(W/Ws), Hs*Ws, C] of Hs x Ws grid positions, as the public CSwin model
    writes it: channels first, the grid split on both axes, the two stripe axes moved next to each other."""
    return [("permute", (0, 2, 1)),
            ("reshape", (B, C, H // Hs, Hs, W // Ws, Ws)),
            ("permute", (0, 2, 4, 3, 5, 1)),
            ("reshape", (B * (H // Hs) * (W // Ws), Hs * Ws, C))]


def stripe_merge_chain(B, H, W, C, Hs, Ws):
    """Stripes [B*(H/Hs)*(W/Ws), Hs*Ws, C] -> tokens [B, H*W, C]."""
    return [("reshape", (B, H // Hs, W // Ws, Hs, Ws, C)),
            ("permute", (0, 1, 3, 2, 4, 5)),
            ("reshape", (B, H * W, C))]
