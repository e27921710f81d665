"""sm_swin_block_static (the entry point for callers that cannot allocate) against sm_swin_block: same kernels on the
library's static workspace, so the outputs must be identical; two calls in a row, the second with a smaller input
(the static buffer keeps the first call's contents)."""
import pytest
import torch
from paper_2404_13528_amd import binding as sm, workloads as Wl
from util import dev, dev_params

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", [sm.SM_ELIDED, sm.SM_EXPLICIT])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_static_workspace_matches_callers_workspace(mode, dtype):
    bf = dtype == torch.bfloat16
    for (B, H, W, C, h, s) in ((4, 28, 28, 128, 4, 3), (1, 14, 14, 96, 3, 0)):      # the second call is the smaller one
        x, p = Wl.swin_block_case(B, H, W, C, h, 7, seed=B, bf16=bf)
        blk = sm.SwinBlock(B, H, W, C, h, 7, s, dev_params(p, dtype), dtype, mode)
        assert blk.ws.numel() <= sm.lib().sm_swin_block_static_max_bytes()
        xd = dev(x, dtype)
        want = blk(xd)
        got = sm.swin_block_static(blk, xd)
        torch.cuda.synchronize()
        assert torch.equal(got, want)


def test_static_workspace_refuses_a_block_that_does_not_fit():
    dtype = torch.bfloat16
    B, H, W, C, h = 64, 56, 56, 128, 4                  # 51 MB per activation: far beyond the static buffer
    x, p = Wl.swin_block_case(1, 7, 7, C, h, 7, seed=0, bf16=True)
    blk = sm.SwinBlock(1, 7, 7, C, h, 7, 0, dev_params(p, dtype), dtype, sm.SM_ELIDED)
    blk.cfg.B, blk.cfg.H, blk.cfg.W = B, H, W
    with pytest.raises(sm.SmError, match="static buffer"):
        sm.swin_block_static(blk, dev(x, dtype))
