"""sm_cswin_attention (cross-shaped window attention) and the stripe kind of sm_attention against oracle/cswin.py: both
modes, the stripe widths and grids of the four stages of CSwin-T, a non-square grid, and the full batch bench-sized case."""
import numpy as np
import pytest
import torch

from oracle import cswin as CS
from oracle import ops as O
from paper_2404_13528_amd import binding as sm, workloads as Wl
from util import assert_bf16_close, np_params, to_np

pytestmark = pytest.mark.gpu

CASES = [
    (2, 56, 56, 64, 2, 1),       # stage 1: stripes one token wide (runs of one token)
    (2, 28, 28, 128, 4, 2),      # stage 2
    (3, 14, 14, 256, 8, 7),      # stage 3: 98 tokens per stripe
    (2, 7, 7, 512, 16, 7),       # stage 4: the stripe is the whole image
    (2, 8, 12, 96, 4, 4),        # non-square grid, head size 24, stripes of 32 and 48 tokens
    (1, 48, 48, 32, 2, 3),       # 144 tokens per stripe: two query tiles and three key tiles with ragged tails
    (2, 6, 10, 32, 4, 2),        # head size 8, stripes of 12 and 20 tokens: less than one key tile
    (1, 5, 5, 16, 2, 5),         # a single stripe of 25 tokens per half, one head per half
]


def run_case(B, H, W, Cc, heads, sw, mode, seed=0, lepe=False):
    qkv = Wl.cswin_qkv_case(B, H, W, Cc, seed=seed, bf16=True)
    pe = Wl.cswin_lepe_params(Cc, seed=seed, bf16=True) if lepe else None
    want = CS.cross_window_attention(to_np(qkv), B, H, W, Cc, heads, sw, *([to_np(t) for t in pe] if lepe else []))
    op = sm.CswinAttention(B, H, W, Cc, heads, sw, mode)
    dev = qkv.to(torch.bfloat16).cuda()
    before = dev.clone()
    out = torch.full((B, H * W, Cc), float("nan"), dtype=torch.bfloat16, device="cuda")      # nothing of it may survive
    out = op(dev, out=out, lepe=[t.to(torch.bfloat16).cuda() for t in pe] if lepe else None)
    torch.cuda.synchronize()
    # elided: the two attentions are one launch when both halves have one shape (square grid), and so are the two
    # convolutions; explicit: one kernel per operator and per half, and the copies
    n_att = 1 if H == W else 2
    if lepe:
        assert sm.launch_counts() == ((n_att + 1, 0) if mode == sm.SM_ELIDED else (4, 9))
    else:
        assert sm.launch_counts() == ((n_att, 0) if mode == sm.SM_ELIDED else (2, 5))
    assert torch.equal(dev, before)
    assert_bf16_close(out.reshape(B * H * W, Cc), want.reshape(B * H * W, Cc), what="cross-window attention")
    return out


@pytest.mark.parametrize("mode", [sm.SM_ELIDED, sm.SM_EXPLICIT])
@pytest.mark.parametrize("B,H,W,Cc,heads,sw", CASES)
def test_matches_the_oracle(B, H, W, Cc, heads, sw, mode):
    run_case(B, H, W, Cc, heads, sw, mode, seed=H + sw)


@pytest.mark.parametrize("mode", [sm.SM_ELIDED, sm.SM_EXPLICIT])
@pytest.mark.parametrize("B,H,W,Cc,heads,sw", CASES)
def test_with_positional_encoding_matches_the_oracle(B, H, W, Cc, heads, sw, mode):
    run_case(B, H, W, Cc, heads, sw, mode, seed=H + sw + 1, lepe=True)


def test_positional_encoding_is_visible_and_its_planted_mistake_shows():
    B, H, W, Cc, heads, sw = 2, 14, 14, 64, 2, 7
    out = run_case(B, H, W, Cc, heads, sw, sm.SM_ELIDED, seed=4, lepe=True)
    qkv = to_np(Wl.cswin_qkv_case(B, H, W, Cc, seed=4, bf16=True))
    w, b = [to_np(t) for t in Wl.cswin_lepe_params(Cc, seed=4, bf16=True)]
    for wrong in (CS.cross_window_attention(qkv, B, H, W, Cc, heads, sw),                              # encoding dropped
                  CS.cross_window_attention(qkv, B, H, W, Cc, heads, sw, w[:, ::-1, ::-1].copy(), b)):     # kernel flipped
        with pytest.raises(AssertionError):
            assert_bf16_close(out.reshape(B * H * W, Cc), wrong.reshape(B * H * W, Cc), what="planted mistake")


def test_attention_accumulates_into_its_output():
    nb, h, n, d = 3, 2, 150, 32
    g = torch.Generator().manual_seed(2)
    q, k, v, o0 = [torch.randn(nb, h, n, d, generator=g).to(torch.bfloat16) for _ in range(4)]
    want, _ = O.attention(to_np(q), to_np(k), to_np(v), d ** -0.5, causal=True)
    out = o0.cuda().clone()
    sm.attention(q.cuda(), k.cuda(), v.cuda(), kind="causal", out=out, accumulate=True)
    torch.cuda.synchronize()
    assert_bf16_close(out.reshape(nb * h * n, d), (want + to_np(o0)).reshape(nb * h * n, d), what="accumulating attention")
    with pytest.raises(sm.SmError):        # the window kernels have no accumulating form
        t = torch.zeros(169, 2, dtype=torch.bfloat16, device="cuda")
        w = torch.zeros(1, 2, 49, 32, dtype=torch.bfloat16, device="cuda")
        sm.attention(w, w, w, kind="window", rpb_table=t, window=7, H=7, W=7, accumulate=True)


def test_modes_agree_and_repeat():
    B, H, W, Cc, heads, sw = 4, 14, 14, 256, 8, 7
    a = run_case(B, H, W, Cc, heads, sw, sm.SM_ELIDED, seed=5)
    b = run_case(B, H, W, Cc, heads, sw, sm.SM_EXPLICIT, seed=5)
    # same kernel arithmetic on the same values, only the addresses differ
    assert torch.equal(a, b)
    assert torch.equal(a, run_case(B, H, W, Cc, heads, sw, sm.SM_ELIDED, seed=5))


def test_full_batch_stage3():
    # the size bench-style runs use: 64 images of 14 x 14 tokens, 256 channels, stripes 7 wide
    run_case(64, 14, 14, 256, 8, 7, sm.SM_ELIDED, seed=9)


def test_a_planted_mistake_in_the_oracle_shows():
    B, H, W, Cc, heads, sw = 2, 14, 14, 64, 2, 7
    qkv = Wl.cswin_qkv_case(B, H, W, Cc, seed=3, bf16=True)
    out = sm.CswinAttention(B, H, W, Cc, heads, sw)(qkv.to(torch.bfloat16).cuda())
    # horizontal stripes for the first half of the heads and vertical for the second (the halves exchanged)
    x = to_np(qkv).reshape(B, H, W, 3, Cc).transpose(0, 2, 1, 3, 4).reshape(B, H * W, 3 * Cc)
    wrong = CS.cross_window_attention(np.ascontiguousarray(x), B, W, H, Cc, heads, sw)
    wrong = wrong.reshape(B, W, H, Cc).transpose(0, 2, 1, 3).reshape(B * H * W, Cc)
    with pytest.raises(AssertionError):
        assert_bf16_close(out.reshape(B * H * W, Cc), wrong, what="exchanged halves")


def test_stripe_kind_of_the_attention_operator():
    # one tensor [B, H, W, heads, d] read as vertical stripes of width 2 (runs of 2 tokens, a grid row apart) and
    # written back in place order; against the oracle's attention on gathered stripes
    B, H, W, h, d, sw = 2, 6, 8, 3, 16, 2
    g = torch.Generator().manual_seed(1)
    q, k, v = [torch.randn(B, H, W, h, d, generator=g).to(torch.bfloat16) for _ in range(3)]
    ns, S = W // sw, H * sw
    tok = h * d
    strides = dict(q_stride=(H * W * tok, d, tok), k_stride=(H * W * tok, d, tok), v_stride=(H * W * tok, d, tok), o_stride=(H * W * tok, d, tok))
    stripe = (sw * tok, W * tok)
    out = torch.zeros(B, H, W, h, d, dtype=torch.bfloat16, device="cuda")
    sm.attention(q.cuda(), k.cuda(), v.cuda(), kind="stripe", out=out, shape=(B * ns, h, S, S, d), stripes=ns, run=sw,
                 q_stripe=stripe, k_stripe=stripe, v_stripe=stripe, o_stripe=stripe, **strides)
    torch.cuda.synchronize()

    def gather(t):          # [B, H, W, h, d] -> [B, ns, h, H * sw, d]
        return to_np(t).reshape(B, H, ns, sw, h, d).transpose(0, 2, 4, 1, 3, 5).reshape(B, ns, h, S, d)
    want, _ = O.attention(gather(q), gather(k), gather(v), d ** -0.5)
    want = want.reshape(B, ns, h, H, sw, d).transpose(0, 3, 1, 4, 2, 5).reshape(B * H * W, h * d)
    assert_bf16_close(out.reshape(B * H * W, h * d), want, what="stripe attention")


def test_refusals_on_device():
    q = torch.zeros(2, 2, 8, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sm.SmError):        # head size 64 has no stripe variant
        sm.attention(q, q, q, kind="stripe", stripes=1, run=8)
    q = torch.zeros(3, 2, 8, 32, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sm.SmError):        # three batch entries are not whole images of two stripes
        sm.attention(q, q, q, kind="stripe", stripes=2, run=8)
    with pytest.raises(sm.SmError):        # a stripe of 8 tokens is not whole runs of 3
        sm.attention(q, q, q, kind="stripe", stripes=1, run=3)


BLOCKS = [
    (2, 56, 56, 64, 2, 1),       # stage 1 of CSwin-T: no fused kernel at 64 channels, one kernel per Linear
    (2, 28, 28, 128, 4, 2),      # stage 2: packed-weight LayerNorm + QKV, projection + MLP as one kernel
    (3, 14, 14, 256, 8, 7),      # stage 3
    (2, 7, 7, 512, 16, 7),       # stage 4: the 64-token fused kernel
    (2, 8, 12, 96, 4, 4),        # CSwin-B's first width: head size 24, no fused kernel
]


def run_block(B, H, W, Cc, heads, sw, mode, seed=0, std=0.02, fuse=True):
    x, p = Wl.cswin_block_case(B, H, W, Cc, seed=seed, bf16=True, std=std)
    want = CS.cswin_block(to_np(x), np_params(p), B, H, W, Cc, heads, sw)
    dev = {k: v.to(torch.bfloat16).cuda() for k, v in p.items()}
    blk = sm.CswinBlock(B, H, W, Cc, heads, sw, dev, mode, fuse=fuse)
    xd = x.to(torch.bfloat16).cuda()
    y = blk(xd)
    torch.cuda.synchronize()
    n_compute, n_copy = sm.launch_counts()
    assert n_copy == (0 if mode == sm.SM_ELIDED else 9)
    assert_bf16_close(y.reshape(B * H * W, Cc), want.reshape(B * H * W, Cc), x=to_np(x), what="CSwin block")
    # kernels of the attention operator: convolution + attention(s) elided, 2 + 2 explicit
    n_attention_op = (2 if H == W else 3) if mode == sm.SM_ELIDED else 4
    return y, n_compute - n_attention_op


@pytest.mark.parametrize("mode", [sm.SM_ELIDED, sm.SM_EXPLICIT])
@pytest.mark.parametrize("B,H,W,Cc,heads,sw", BLOCKS)
def test_block_matches_the_oracle(B, H, W, Cc, heads, sw, mode):
    # weights of std 0.02 leave a branch delta y - x of about 0.05 here (the attention averages 50 to 100 values under a
    # nearly uniform softmax), of which the bf16 rounding of y alone (magnitude 1) is already 3 %: wider weights, so
    # that the delta check sees the arithmetic and not that rounding
    _, n = run_block(B, H, W, Cc, heads, sw, mode, seed=H, std=0.06)
    # around the attention operator: LayerNorm + QKV, then projection + MLP in one kernel or the Linears one by one
    fused = Cc in (128, 256, 512)
    assert n == (2 if fused else 4)


# kernels without fusion: at 256 channels both LayerNorms are kernels of their own (their Linears have too many column
# tiles to repeat the norm in each), at 128 they are folded into the Linear's load
@pytest.mark.parametrize("B,H,W,Cc,heads,sw,n_per_op", [(2, 14, 14, 256, 8, 7, 6), (1, 28, 28, 128, 4, 2, 4)])
def test_block_on_the_stress_distribution_and_without_fusion(B, H, W, Cc, heads, sw, n_per_op):
    a, _ = run_block(B, H, W, Cc, heads, sw, sm.SM_ELIDED, seed=7, std=0.1)
    b, n = run_block(B, H, W, Cc, heads, sw, sm.SM_ELIDED, seed=7, std=0.1, fuse=False)
    assert n == n_per_op
    assert_bf16_close(a.reshape(-1, Cc), to_np(b).reshape(-1, Cc), what="fused against kernel per operator")


def test_block_full_batch_stage3_both_modes():
    # the size bench.py times: 64 images of 14 x 14 tokens, 256 channels
    a, _ = run_block(64, 14, 14, 256, 8, 7, sm.SM_ELIDED, seed=12, std=0.06)
    b, _ = run_block(64, 14, 14, 256, 8, 7, sm.SM_EXPLICIT, seed=12, std=0.06)
    assert torch.equal(a, b)          # the same kernels on the same values: only the addresses differ
