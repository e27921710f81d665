"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch


def to_np(t):
    return t.detach().double().cpu().numpy()


def np_params(p):
    return {k: to_np(v) for k, v in p.items()}


def dev(t, dtype):
    return t.to(dtype).cuda().contiguous()


def dev_params(p, dtype):
    return {k: dev(v, dtype) for k, v in p.items()}


def rel_l2(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30))


def max_abs(got, want):
    return float(np.abs(np.asarray(got, np.float64) - np.asarray(want, np.float64)).max())


# tolerances of the build: fp32 kernels max-abs 1e-4, bf16 kernels relative L2 2e-2
def assert_close(got, want, dtype, what="", scale_abs=1.0):
    got = to_np(got) if isinstance(got, torch.Tensor) else got
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.isfinite(got).all(), what + ": non-finite output"
    if dtype == torch.float32:
        e = max_abs(got, want)
        assert e <= 1e-4 * scale_abs, "%s: max-abs %.3e" % (what, e)
    else:
        e = rel_l2(got, want)
        assert e <= 2e-2, "%s: relative L2 %.3e" % (what, e)
    return e
