"""GPU parity of sm_attn_block against the oracle: a Llama-style decoder layer
(configuration 4 at full size and a small stress case) and the diffusion
spatial-transformer block (configuration 5 at full size and a small stress
case), elided and explicit modes, with the branch delta compared as well."""
import numpy as np
import pytest
import torch
from oracle import llama, sd
from paper_2404_13528_amd import binding as sm, workloads as Wl
from util import to_np, np_params, dev, dev_params, rel_l2, assert_bf16_close

pytestmark = pytest.mark.gpu
MODES = [sm.SM_ELIDED, sm.SM_EXPLICIT]
BF = torch.bfloat16


def run_llama(B, S, E, h, F, mode, std=0.02, in_std=1.0, seed=0):
    x, p = Wl.llama_case(B, S, E, F, seed=seed, std=std, in_std=in_std)
    blk = sm.AttnBlock("llama", dev_params(p, BF), BF, mode, B=B, S=S, E=E, heads=h, F=F)
    y = blk(dev(x, BF))
    torch.cuda.synchronize()
    return to_np(y), llama.llama_layer(to_np(x), np_params(p), h), to_np(x), sm.launch_counts()


@pytest.mark.parametrize("mode", MODES)
def test_llama_small_stress(mode):
    # weights std 0.1 with E = 256: O(1) logits, branches comparable to the residual; ragged S
    got, want, x, counts = run_llama(2, 150, 256, 2, 352, mode, std=0.1)
    assert_bf16_close(got, want, "block output", x=x)
    assert counts == ((7, 0) if mode == sm.SM_ELIDED else (7, 2))


def test_llama_wrong_rope_pairing_is_detected():
    x, p = Wl.llama_case(2, 150, 256, 352, std=0.1)
    good = llama.llama_layer(to_np(x), np_params(p), 2)
    from oracle import ops as O
    orig = O.rope_half_split

    def interleaved(t, base=10000.0):        # the other common pairing (2i, 2i+1)
        S, D = t.shape[-2], t.shape[-1]
        th = base ** (-2.0 * np.arange(D // 2) / D)
        ang = np.arange(S)[:, None] * th[None]
        out = t.copy()
        out[..., 0::2] = t[..., 0::2] * np.cos(ang) - t[..., 1::2] * np.sin(ang)
        out[..., 1::2] = t[..., 1::2] * np.cos(ang) + t[..., 0::2] * np.sin(ang)
        return out
    O.rope_half_split = interleaved
    try:
        bad = llama.llama_layer(to_np(x), np_params(p), 2)
    finally:
        O.rope_half_split = orig
    assert rel_l2(bad - to_np(x), good - to_np(x)) > 3e-2


@pytest.mark.parametrize("mode", MODES)
def test_config4_llama_layer_full_size(mode):
    got, want, x, _ = run_llama(1, 2048, 4096, 32, 11008, mode)
    assert_bf16_close(got, want, "block output", x=x)


def run_sd(B, C, H, W, Sc, Dc, F, G, h, mode, std=0.02, seed=0):
    x, ctx, p = Wl.sd_case(B, C, H, W, Sc, Dc, F, seed=seed, std=std)
    blk = sm.AttnBlock("sd", dev_params(p, BF), BF, mode, B=B, E=C, heads=h, F=F, Hs=H, Ws=W, groups=G, Sc=Sc, Dc=Dc)
    y = blk(dev(x, BF), dev(ctx, BF))
    torch.cuda.synchronize()
    return to_np(y), sd.spatial_transformer(to_np(x), to_np(ctx), np_params(p), G, h), to_np(x), sm.launch_counts()


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("H,W", [(9, 7), (8, 12)])
def test_sd_small_stress(mode, H, W):
    got, want, x, counts = run_sd(2, 64, H, W, 13, 24, 96, 8, 2, mode, std=0.12)
    assert_bf16_close(got, want, "block output", x=x)
    # GroupNorm is two launches (statistics, apply) where H W is a multiple of the 16-byte vector, else one
    n = 15 + (1 if (H * W) % 8 == 0 else 0)
    assert counts == ((n, 0) if mode == sm.SM_ELIDED else (n, 7))


@pytest.mark.parametrize("mode", MODES)
def test_config5_sd_block_full_size(mode):
    got, want, x, _ = run_sd(2, 320, 64, 64, 77, 768, 1280, 32, 8, mode)
    assert_bf16_close(got, want, "block output", x=x)


def run_vit(B, S, E, h, F, mode, std=0.02, seed=0):
    from oracle import vit
    x, p = Wl.vit_case(B, S, E, h, F, seed=seed, std=std)
    blk = sm.AttnBlock("vit", dev_params(p, BF), BF, mode, B=B, S=S, E=E, heads=h, F=F)
    y = blk(dev(x, BF))
    torch.cuda.synchronize()
    return to_np(y), vit.vit_block(to_np(x), np_params(p), h), to_np(x), sm.launch_counts()


@pytest.mark.parametrize("mode", MODES)
def test_vit_small_stress(mode):
    # 197 tokens (14 x 14 patches + class token: ragged against every tile), O(1) logits
    got, want, x, counts = run_vit(2, 197, 128, 2, 256, mode, std=0.1, seed=4)
    assert_bf16_close(got, want, "ViT block", x=x)
    assert counts == ((7, 0) if mode == sm.SM_ELIDED else (7, 2))


@pytest.mark.parametrize("mode", MODES)
def test_vit_b16_block_full_size(mode):
    # ViT-B/16 at 224 x 224 (the paper's ViT row, Table 7): 197 tokens, 768 wide, 12 heads, MLP 3072; B = 32
    got, want, x, _ = run_vit(32, 197, 768, 12, 3072, mode)
    assert_bf16_close(got, want, "ViT-B block", x=x)
