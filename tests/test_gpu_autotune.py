"""The Linear tuner (Sec. 3.3: tile shapes chosen by search): every variant gives the same result as the built-in
choice, the remembered variant is the one later launches use, and it is never slower than the default it measured."""
import numpy as np
import pytest
import torch
from oracle import ops as O
from paper_2404_13528_amd import binding as sm
from util import to_np, assert_bf16_close

pytestmark = pytest.mark.gpu


def test_autotune_keeps_results_and_never_loses():
    dt = torch.bfloat16
    M, N, K = 3000, 640, 512                      # ragged in M, several tiles in both directions
    g = torch.Generator().manual_seed(3)
    A = (torch.randn(M, K, generator=g)).to(dt)
    W = (torch.randn(N, K, generator=g) * K ** -0.5).to(dt)
    b = (torch.randn(N, generator=g) * 0.1).to(dt)
    want = O.gelu(O.linear(to_np(A), to_np(W), to_np(b)))
    sm.lib().sm_linear_autotune_clear()
    base = sm.linear(A.cuda(), W.cuda(), bias=b.cuda(), act="gelu")
    torch.cuda.synchronize()
    assert_bf16_close(base, want, "default tile")
    for rows in (64, 128, 256):                   # every tile height through the sweep hook: identical outputs
        for stages in (2, 3, 4):
            sm.gemm_tuning(rows, stages)
            try:
                got = sm.linear(A.cuda(), W.cuda(), bias=b.cuda(), act="gelu")
                torch.cuda.synchronize()
            finally:
                sm.gemm_tuning(0, 0)
            assert torch.equal(got, base), (rows, stages)
    r = sm.linear_autotune(M, N, K, act="gelu", iters=10)
    assert r["tile_rows"] in (0, 64, 128, 256) and r["stages"] in (0, 2, 3, 4)
    assert r["best_us"] <= r["default_us"] * 1.0001
    tuned = sm.linear(A.cuda(), W.cuda(), bias=b.cuda(), act="gelu")      # now through the remembered variant
    torch.cuda.synchronize()
    assert torch.equal(tuned, base)
    sm.lib().sm_linear_autotune_clear()


def test_autotune_shape_without_variants_and_bad_arguments():
    r = sm.linear_autotune(100, 96, 40, dtype=torch.float32, iters=3)     # fp32: one variant
    assert r["tile_rows"] == 0 and r["stages"] == 0
    with pytest.raises(sm.SmError):
        sm.linear_autotune(64, 64, 64, iters=0)
