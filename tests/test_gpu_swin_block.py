"""GPU parity of sm_swin_block (both modes) against the oracle: configuration 1
(fp32, B=1, 56x56, C=96, 3 heads, window 7, shift 3) at full size, small bf16
blocks, and stress-distribution weights so that bias / mask / shift errors
exceed the tolerance.  The branch delta y - x is compared as well, because the
residual stream dominates y."""
import numpy as np
import pytest
import torch
from oracle import swin
from paper_2404_13528_amd import binding as sm, workloads as Wl
from util import to_np, np_params, dev, dev_params, assert_close, rel_l2, assert_bf16_close

pytestmark = pytest.mark.gpu
MODES = [sm.SM_ELIDED, sm.SM_EXPLICIT]


def n_compute(C, mlp=4, fused=False, mode=None):
    """Compute kernels of a block: seven, minus a LayerNorm for each Linear narrow enough (N <= 512) to take it folded;
    with the fused MLP kernel LayerNorm-2, FC1 and FC2 are one ("mlp"); True: in elided mode the output projection
    joins them and LayerNorm-1 + QKV are one packed-weight Linear."""
    if fused is True and mode == sm.SM_ELIDED:
        return 3          # LayerNorm-1 + QKV (packed-weight Linear), attention, projection + MLP
    if fused:
        return 5 - (3 * C <= 512)
    return 7 - (3 * C <= 512) - (mlp * C <= 512)


def run_block(B, H, W, C, h, w, s, dtype, mode, seed=0, std=0.02, fuse_mlp=True):
    x, p = Wl.swin_block_case(B, H, W, C, h, w, seed=seed, bf16=(dtype == torch.bfloat16), std=std)
    blk = sm.SwinBlock(B, H, W, C, h, w, s, dev_params(p, dtype), dtype, mode, fuse_mlp=fuse_mlp)
    y = blk(dev(x, dtype))
    torch.cuda.synchronize()
    want = swin.swin_block(to_np(x), np_params(p), H, W, w, h, s)
    return to_np(y), want, to_np(x), sm.launch_counts()


@pytest.mark.parametrize("mode", MODES)
def test_config1_fp32_full_size(mode):
    got, want, x, counts = run_block(1, 56, 56, 96, 3, 7, 3, torch.float32, mode)
    e = np.abs(got - want).max()
    assert e <= 1e-4, "max-abs %.3e" % e
    assert rel_l2(got - x, want - x) <= 1e-4            # branch delta
    assert counts == ((n_compute(96), 0) if mode == sm.SM_ELIDED else (n_compute(96), 6))


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("s", [0, 3])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_small_block_stress_weights(dtype, s, mode):
    # weights with std 0.15: logits and biases are O(1), the branches are as large as the residual
    got, want, x, counts = run_block(2, 14, 21, 96, 3, 7, s, dtype, mode, seed=5, std=0.15)
    if dtype == torch.float32:
        assert np.abs(got - want).max() <= 1e-4 * max(1.0, np.abs(want).max())
    else:
        assert_bf16_close(got, want, "stress block", x=x)
    assert counts == (n_compute(96), 0 if mode == sm.SM_ELIDED else (6 if s else 4))


def test_wrong_shift_or_bias_is_detected_by_the_tolerance():
    # the oracle with a planted mistake (no shift / zero bias table) must violate the tolerance
    x, p = Wl.swin_block_case(2, 14, 21, 96, 3, 7, seed=5, std=0.15)
    good = swin.swin_block(to_np(x), np_params(p), 14, 21, 7, 3, 3)
    bad_shift = swin.swin_block(to_np(x), np_params(p), 14, 21, 7, 3, 0)
    pz = np_params(p); pz["rpb_table"] = np.zeros_like(pz["rpb_table"])
    bad_bias = swin.swin_block(to_np(x), pz, 14, 21, 7, 3, 3)
    assert rel_l2(bad_shift, good) > 2e-2 and rel_l2(bad_bias, good) > 2e-2


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("fuse_mlp", [True, "mlp", False])
def test_config2_block_bf16_full_size(mode, fuse_mlp):
    got, want, x, counts = run_block(32, 14, 14, 384, 12, 7, 3, torch.bfloat16, mode, fuse_mlp=fuse_mlp)
    assert_bf16_close(got, want, "config-2 block", x=x)
    assert counts == (n_compute(384, fused=fuse_mlp, mode=mode), 0 if mode == sm.SM_ELIDED else 6)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("fuse_mlp", [True, "mlp", False])
@pytest.mark.parametrize("C,h", [(128, 4), (256, 8)])
def test_small_block_stress_weights_fused_mlp_shapes(C, h, fuse_mlp, mode):
    # widths the fused MLP kernel covers, with and without it; a token count (2 * 14 * 21 = 588) that ends inside
    # a 32-token tile
    got, want, x, counts = run_block(2, 14, 21, C, h, 7, 3, torch.bfloat16, mode, seed=6, std=0.1, fuse_mlp=fuse_mlp)
    assert_bf16_close(got, want, "stress block", x=x)
    assert counts == (n_compute(C, fused=fuse_mlp, mode=mode), 0 if mode == sm.SM_ELIDED else 6)


@pytest.mark.parametrize("s", [0, 3])
@pytest.mark.parametrize("std", [0.02, 0.15])
def test_intermediates_of_the_elided_block(s, std):
    # one kernel per surviving operator (fuse_mlp=False): qkv, attention output, x1 and the hidden activation are
    # stored tensors, each compared with the oracle's own intermediate in the layout the plan gave it
    B, H, W, C, h, w = 3, 14, 21, 384, 12, 7
    dtype = torch.bfloat16
    x, p = Wl.swin_block_case(B, H, W, C, h, w, seed=7, bf16=True, std=std)
    blk = sm.SwinBlock(B, H, W, C, h, w, s, dev_params(p, dtype), dtype, sm.SM_ELIDED, fuse_mlp=False)
    y = blk(dev(x, dtype))
    torch.cuda.synchronize()
    got = {k: to_np(v) for k, v in sm.swin_block_intermediates(blk).items()}
    want = swin.swin_block(to_np(x), np_params(p), H, W, w, h, s, want_all=True)
    for name in ("qkv", "o", "x1", "hid"):
        assert_bf16_close(got[name], want[name], name)
    assert_bf16_close(to_np(y), want["y"], "y", x=to_np(x))
    # the softmax itself: every row of P the oracle formed sums to 1, and o is P . v of the stored qkv
    assert np.abs(want["P"].sum(-1) - 1).max() < 1e-9


def test_errors_before_launch():
    x, p = Wl.swin_block_case(1, 14, 14, 32, 2, 7)
    with pytest.raises(sm.SmError):
        sm.SwinBlock(1, 15, 14, 32, 2, 7, 0, dev_params(p, torch.float32), torch.float32)     # 15 % 7
    blk = sm.SwinBlock(1, 14, 14, 32, 2, 7, 0, dev_params(p, torch.float32), torch.float32)
    blk.ws = blk.ws[:1024]
    with pytest.raises(sm.SmError, match="workspace"):
        blk(dev(x, torch.float32))
