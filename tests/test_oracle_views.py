"""Pins for oracle.views: library routines (torch.roll / permute), brute-force
loops, the paper's 5x5x5 example (Sec. 2.2) and the identities the method
relies on (layout transformations are pure data movement)."""
import itertools
import os
import numpy as np
import pytest
import torch
from oracle import views as V

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_roll_matches_library_and_definition():
    a = np.arange(2 * 5 * 7).reshape(2, 5, 7).astype(np.float64)
    for axis, r in [(1, 2), (1, -2), (2, 3), (2, -10), (0, 1)]:
        got = V.roll(a, axis, r)
        assert np.array_equal(got, torch.roll(torch.from_numpy(a), r, axis).numpy())
        n = a.shape[axis]
        for i in range(n):        # out[i] = in[(i - r) mod n]
            assert np.array_equal(np.take(got, i, axis), np.take(a, (i - r) % n, axis))


def test_permute_brute_force():
    a = np.random.default_rng(0).standard_normal((2, 3, 4, 5))
    for perm in [(0, 2, 1, 3), (3, 0, 2, 1), (1, 0, 3, 2)]:
        got = V.permute(a, perm)
        assert got.shape == tuple(a.shape[p] for p in perm)
        for idx in itertools.product(*[range(s) for s in got.shape]):
            src = [0] * 4
            for k, p in enumerate(perm):
                src[p] = idx[k]
            assert got[idx] == a[tuple(src)]
        assert np.array_equal(got, torch.from_numpy(a).permute(*perm).contiguous().numpy())


def test_paper_reshape_transpose_example():
    lines = [l.split() for l in open(os.path.join(GOLD, "reshape_transpose_example.txt"))
             if l.strip() and not l.startswith("#")]
    spec = {l[0]: tuple(int(v) for v in l[1:]) for l in lines}
    m = V.index_map(spec["src_shape"], [("reshape", spec["reshape"]), ("permute", spec["permute"])])
    assert m.shape == (25, 5)
    for j in range(25):
        for i in range(5):
            assert m[j, i] == (i * 5 + j // 5) * 5 + j % 5


def test_pure_reshape_chain_is_identity_map():
    m = V.index_map((4, 6, 10), [("reshape", (24, 10)), ("reshape", (2, 12, 10)), ("reshape", (240,))])
    assert np.array_equal(m, np.arange(240))


@pytest.mark.parametrize("s", [0, 3])
def test_partition_then_reverse_is_identity(s):
    B, H, W, C, w = 2, 14, 21, 3, 7
    x = np.random.default_rng(1).standard_normal((B, H, W, C))
    win = V.apply_chain(x, V.window_partition_chain(B, H, W, C, w, s))
    assert win.shape == (B * 2 * 3, 49, C)
    back = V.apply_chain(win, V.window_reverse_chain(B, H, W, C, w, s))
    assert np.array_equal(back, x)
    m = V.index_map((B, H, W, C), V.window_partition_chain(B, H, W, C, w, s))
    assert np.array_equal(np.sort(m.reshape(-1)), np.arange(B * H * W * C))   # a permutation


def test_window_map_closed_form():
    B, H, W, C, w, s = 2, 14, 14, 4, 7, 3
    m = V.index_map((B, H, W, C), V.window_partition_chain(B, H, W, C, w, s))
    nWy, nWx = H // w, W // w
    for bw in range(B * nWy * nWx):
        b, r = divmod(bw, nWy * nWx)
        wy, wx = divmod(r, nWx)
        for n in range(w * w):
            iy, ix = divmod(n, w)
            y, x = (wy * w + iy + s) % H, (wx * w + ix + s) % W
            assert m[bw, n, 0] == ((b * H + y) * W + x) * C


def test_roll_unroll_identity_and_head_split_merge():
    x = np.random.default_rng(2).standard_normal((2, 6, 8, 5))
    assert np.array_equal(V.roll(V.roll(x, 1, -3), 1, 3), x)
    B, S, h, d = 2, 9, 4, 6
    t = np.random.default_rng(3).standard_normal((B, S, h * d))
    sp = V.apply_chain(t, V.head_split_chain(B, S, h, d))
    assert sp.shape == (B, h, S, d)
    assert sp[1, 2, 3, 4] == t[1, 3, 2 * d + 4]
    assert np.array_equal(V.apply_chain(sp, V.head_merge_chain(B, S, h, d)), t)


def test_qkv_split_picks_columns():
    B_, N, h, d = 3, 5, 2, 4
    t = np.random.default_rng(4).standard_normal((B_, N, 3 * h * d))
    q = V.apply_chain(t, V.qkv_split_chain(B_, N, h, d))
    for k in range(3):
        for hh in range(h):
            assert np.array_equal(q[k, :, hh], t[:, :, (k * h + hh) * d:(k * h + hh + 1) * d])


def test_patch_merge_is_four_strided_slices():
    B, H, W, C = 2, 6, 8, 3
    x = np.random.default_rng(5).standard_normal((B, H, W, C))
    got = V.apply_chain(x, V.patch_merge_chain(B, H, W, C))
    parts = [x[:, 0::2, 0::2], x[:, 1::2, 0::2], x[:, 0::2, 1::2], x[:, 1::2, 1::2]]  # k = 2*dw + dh
    assert np.array_equal(got, np.concatenate(parts, axis=-1))
    m = V.index_map((B, H, W, C), V.patch_merge_chain(B, H, W, C))
    assert np.array_equal(np.sort(m.reshape(-1)), np.arange(x.size))


def test_patch_embed_unfold_and_nchw_tokens():
    B, Cin, H, W, p = 2, 3, 8, 12, 4
    img = np.random.default_rng(6).standard_normal((B, Cin, H, W))
    a = V.apply_chain(img, V.patch_embed_chain(B, Cin, H, W, p))
    un = torch.nn.functional.unfold(torch.from_numpy(img), kernel_size=p, stride=p)   # [B, Cin*p*p, L]
    assert np.array_equal(a, un.transpose(1, 2).contiguous().numpy())
    t = V.apply_chain(img, V.nchw_to_tokens_chain(B, Cin, H, W))
    assert t[1, 5, 2] == img[1, 2, 5 // W, 5 % W]
    assert np.array_equal(V.apply_chain(t, V.tokens_to_nchw_chain(B, Cin, H, W)), img)


def test_slice_brute_force_and_library():
    a = np.random.default_rng(1).standard_normal((3, 7, 5))
    for axis, start, stop, step in [(0, 1, 3, 1), (1, 0, 7, 2), (1, 2, 6, 3), (2, 4, 5, 1), (2, 0, 5, 1)]:
        got = V.slice_(a, axis, start, stop, step)
        n = len(range(start, stop, step))
        assert got.shape == tuple(n if k == axis else s for k, s in enumerate(a.shape))
        for idx in itertools.product(*[range(s) for s in got.shape]):      # out[.., i, ..] = in[.., start + i*step, ..]
            src = list(idx)
            src[axis] = start + idx[axis] * step
            assert got[idx] == a[tuple(src)]
        lib = torch.index_select(torch.from_numpy(a), axis, torch.arange(start, stop, step)).numpy()
        assert np.array_equal(got, lib)
    # through a chain: the q / k / v split is a slice of the permuted QKV tensor
    iota = V.index_map((2, 4, 12), [("reshape", (2, 4, 3, 2, 2)), ("permute", (2, 0, 3, 1, 4)), ("slice", 0, 1, 2, 1)])
    assert iota.shape == (1, 2, 2, 4, 2)
    assert iota[0, 1, 1, 3, 1] == ((1 * 4 + 3) * 12) + (1 * 2 + 1) * 2 + 1


def test_concat_brute_force_and_library():
    rng = np.random.default_rng(2)
    parts = [rng.standard_normal((2, k, 3)) for k in (1, 4, 2)]
    got = V.concat(parts, 1)
    assert got.shape == (2, 7, 3)
    at = 0
    for p in parts:                     # every part lands, in order, at its running offset along the axis
        for idx in itertools.product(*[range(s) for s in p.shape]):
            assert got[idx[0], at + idx[1], idx[2]] == p[idx]
        at += p.shape[1]
    assert np.array_equal(got, torch.cat([torch.from_numpy(p) for p in parts], 1).numpy())
    # slice then concat along the same axis is the identity; a roll is a concat of two slices (Table 3: Slice,
    # Gather are the ILI & Fixed operators a cyclic shift is exported as)
    a = rng.standard_normal((3, 6))
    assert np.array_equal(V.concat([V.slice_(a, 1, 0, 2), V.slice_(a, 1, 2, 6)], 1), a)
    assert np.array_equal(V.concat([V.slice_(a, 1, 2, 6), V.slice_(a, 1, 0, 2)], 1), V.roll(a, 1, -2))
