"""Host side of sm_cswin_attention without a GPU: the operator's graph (Slices, stripe partition, head split, head merge
and stripe merge around two attentions) plans down to the two attentions with load / store maps that are strided in
the factored index, for vertical and horizontal stripes of several widths; unsupported shapes are refused."""
import ctypes as C
import pytest
from paper_2404_13528_amd import binding as sm


def cfg(B=2, H=14, W=14, Cc=256, heads=8, sw=7):
    return sm.CswinCfg(sm.SM_BF16, B, H, W, Cc, heads, sw)


@pytest.mark.parametrize("shape", [dict(H=56, W=56, Cc=64, heads=2, sw=1), dict(H=28, W=28, Cc=128, heads=4, sw=2),
                                   dict(), dict(H=7, W=7, Cc=512, heads=16, sw=7), dict(H=8, W=12, Cc=96, heads=4, sw=4)])
def test_the_operator_plans_down_to_two_attentions(shape):
    lib = sm.lib()
    c = cfg(**shape)
    el = lib.sm_cswin_attention_workspace_bytes(C.byref(c), sm.SM_ELIDED)
    ex = lib.sm_cswin_attention_workspace_bytes(C.byref(c), sm.SM_EXPLICIT)
    assert el > 0, lib.sm_last_error()
    # explicit: per half of the channels, the three partitioned operands, the attention result and the merged result,
    # and for the positional encoding the values as stripe images and the encoding itself
    tokens = c.B * c.H * c.W
    assert ex >= 7 * tokens * c.C * 2 and ex < 7 * tokens * c.C * 2 + (1 << 20) + 64 * tokens


def test_refusals():
    lib = sm.lib()
    bad = [cfg(heads=3), cfg(heads=7), cfg(Cc=512, heads=8), cfg(sw=4), cfg(B=0), cfg(Cc=72, heads=6), cfg(heads=0)]
    for c in bad:
        assert lib.sm_cswin_attention_workspace_bytes(C.byref(c), sm.SM_ELIDED) == 0
        assert len(lib.sm_last_error()) > 0
    assert lib.sm_cswin_attention_workspace_bytes(C.byref(cfg()), 5) == 0
    assert lib.sm_cswin_attention(C.byref(cfg()), None, None, None, None, None, C.c_size_t(0), sm.SM_ELIDED, None) < 0
    f32 = cfg(); f32.dtype = sm.SM_F32
    assert lib.sm_cswin_attention_workspace_bytes(C.byref(f32), sm.SM_ELIDED) == 0


@pytest.mark.parametrize("B,H,W,Cc,heads,sw", [(2, 6, 6, 32, 4, 2), (1, 8, 12, 48, 2, 4), (2, 4, 4, 16, 2, 1)])
def test_operand_maps_are_strided_in_the_factored_index(B, H, W, Cc, heads, sw):
    """The chain of a q / k / v operand, composed by the library and looked at as (image, stripe, head, run, token in
    run, feature), has the strides the attention kernel is given, and equals the oracle's materialised chain."""
    import numpy as np
    from oracle import views as V
    L, Cb, hb, d = H * W, Cc // 2, heads // 2, Cc // heads
    for branch in range(2):
        Hs, Ws = (H, sw) if branch == 0 else (sw, W)
        S, stripes = Hs * Ws, (H // Hs) * (W // Ws)
        run = sw if branch == 0 else S
        nwin = B * stripes
        for k in range(3):
            chain = [("reshape", (B, L, 3, Cc)), ("slice", 2, k, k + 1), ("reshape", (B, L, Cc)), ("slice", 2, branch * Cb, (branch + 1) * Cb)]
            chain += V.stripe_partition_chain(B, H, W, Cb, Hs, Ws) + V.head_split_chain(nwin, S, hb, d)
            m = sm.Map.create((B, L, 3 * Cc), chain + [("reshape", (B, stripes, hb, S // run, run, d))])
            got = m.eval_host()
            want = V.index_map((B, L, 3 * Cc), chain).reshape(got.shape)
            assert np.array_equal(got, want)
            base, st = m.affine()
            expect = (L * 3 * Cc, (sw if branch == 0 else S) * 3 * Cc, d, W * 3 * Cc, 3 * Cc, 1)
            assert base == k * Cc + branch * Cb
            for axis, n in enumerate(got.shape):
                assert n == 1 or st[axis] == expect[axis], (axis, st, expect)      # an axis of one entry has no stride


def test_block_workspace_and_refusals():
    lib = sm.lib()

    def bcfg(B=2, H=14, W=14, Cc=256, heads=8, sw=7, ratio=4, eps=1e-5):
        return sm.CswinBlockCfg(sm.SM_BF16, B, H, W, Cc, heads, sw, ratio, eps)
    el = lib.sm_cswin_block_workspace_bytes(C.byref(bcfg()), sm.SM_ELIDED)
    ex = lib.sm_cswin_block_workspace_bytes(C.byref(bcfg()), sm.SM_EXPLICIT)
    tokens = 2 * 14 * 14 * 256 * 2
    assert 10 * tokens <= el < 11 * tokens and ex > el + 7 * tokens          # q|k|v, attention output, x1, a norm, the hidden tensor
    for bad in (bcfg(ratio=0), bcfg(eps=0.0), bcfg(heads=3), bcfg(sw=4), bcfg(Cc=24, heads=2)):
        assert lib.sm_cswin_block_workspace_bytes(C.byref(bad), sm.SM_ELIDED) == 0
    w = sm.CswinWeights()
    assert lib.sm_cswin_block(C.byref(bcfg()), C.byref(w), None, None, None, C.c_size_t(0), sm.SM_ELIDED, None) < 0
