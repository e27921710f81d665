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


def row_rel_l2(got, want):
    """Relative L2 error of every row (last axis) on its own; the denominator of a row is floored at a hundredth of
    the mean row norm so that a near-zero row cannot blow the ratio up."""
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    got, want = got.reshape(-1, got.shape[-1]), want.reshape(-1, want.shape[-1])
    wn = np.linalg.norm(want, axis=1)
    return np.linalg.norm(got - want, axis=1) / np.maximum(wn, 1e-2 * wn.mean() + 1e-30)


# bf16 bounds beside the benchmark spec's global relative L2 of 2e-2.  Every stored tensor is rounded to bf16 (relative
# spacing 2^-8, so up to 2^-9 = 2e-3 per element and rounding) and a block passes through 4 - 6 roundings plus fp32
# accumulation: a correct row stays below about 1e-2, and a row that is wrong (swapped, unshifted, unmasked) is off
# by the size of its branch, 1e-1 or more.  The global norm alone cannot see a few wrong rows among thousands.
ROW_TOL = 5e-2          # every row: relative L2
ABS_TOL = 4e-2          # every element: |error| <= ABS_TOL * max|want|
DELTA_TOL = 3e-2        # branch delta y - x, global relative L2 (the final rounding of y alone gives about 1e-2)
DELTA_ROW_TOL = 2.5e-1  # branch delta, every row


def assert_bf16_close(got, want, what="", x=None):
    """Global relative L2 (2e-2), per-row relative L2, max-abs scaled by |want|max and, given the block input x, the
    same on the branch delta y - x."""
    got = to_np(got) if isinstance(got, torch.Tensor) else np.asarray(got, np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.isfinite(got).all(), what + ": non-finite output"
    e = rel_l2(got, want)
    assert e <= 2e-2, "%s: relative L2 %.3e" % (what, e)
    r = row_rel_l2(got, want)
    assert r.max() <= ROW_TOL, "%s: row %d has relative L2 %.3e" % (what, int(r.argmax()), r.max())
    a = max_abs(got, want)
    assert a <= ABS_TOL * np.abs(want).max(), "%s: max-abs %.3e against |want|max %.3e" % (what, a, np.abs(want).max())
    if x is not None:
        x = to_np(x) if isinstance(x, torch.Tensor) else np.asarray(x, np.float64)
        x = x.reshape(want.shape)
        d = rel_l2(got - x, want - x)
        assert d <= DELTA_TOL, "%s: branch delta relative L2 %.3e" % (what, d)
        dr = row_rel_l2(got - x, want - x)
        assert dr.max() <= DELTA_ROW_TOL, "%s: branch delta of row %d has relative L2 %.3e" % (what, int(dr.argmax()), dr.max())
    return e
