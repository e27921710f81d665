"""GPU parity of the single operators against the oracle, through the C ABI,
on stress distributions (O(1) logits, O(1) biases) so that a wrong index, sign
or pairing cannot hide inside the tolerances."""
import numpy as np
import pytest
import torch
from oracle import ops as O, views as V, swin
from paper_2404_13528_amd import binding as sm
from util import to_np, dev, assert_close

pytestmark = pytest.mark.gpu
DT = [torch.float32, torch.bfloat16]


def draw(shape, seed, dtype, std=1.0, mean=0.0):
    g = torch.Generator().manual_seed(seed)
    t = torch.randn(shape, generator=g) * std + mean
    return t.to(dtype).float()          # values both sides consume


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("rows,C", [(37, 96), (200, 384), (5, 1024), (3, 4096), (1003, 128), (45, 64), (70, 256), (9, 32)])
def test_layernorm_and_rmsnorm(dtype, rows, C):
    if dtype == torch.float32 and C > 2048:
        pytest.skip("fp32 rows are limited to 2048 columns")
    x = draw((rows, C), 1, dtype, 2.0, 0.5)
    g = draw((C,), 2, dtype, 0.2, 1.0)
    b = draw((C,), 3, dtype, 0.2)
    y = sm.norm(dev(x, dtype), dev(g, dtype), dev(b, dtype))
    assert_close(y, O.layer_norm(to_np(x), to_np(g), to_np(b)), dtype, "layernorm", 4.0)
    y = sm.norm(dev(x, dtype), dev(g, dtype), None, rms=True)
    assert_close(y, O.rms_norm(to_np(x), to_np(g)), dtype, "rmsnorm", 4.0)


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("s", [0, 3])
def test_layernorm_store_through_window_map(dtype, s):
    B, H, W, C, w = 2, 14, 21, 96, 7
    x = draw((B, H * W, C), 4, dtype)
    g = draw((C,), 5, dtype, 0.2, 1.0)
    b = draw((C,), 6, dtype, 0.2)
    # natural output index -> position in the window-major tensor = map of the inverse chain
    inv = sm.Map.create((B * (H // w) * (W // w), w * w, C), V.window_reverse_chain(B, H, W, C, w, s))
    y = sm.norm(dev(x, dtype), dev(g, dtype), dev(b, dtype), store_map=inv)
    ln = O.layer_norm(to_np(x), to_np(g), to_np(b)).reshape(B, H, W, C)
    want = V.apply_chain(ln, V.window_partition_chain(B, H, W, C, w, s))
    assert_close(y.reshape(want.shape), want, dtype, "layernorm -> windows", 4.0)


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("tokens_out", [False, True])
@pytest.mark.parametrize("split", [False, True])
@pytest.mark.parametrize("B,C,H,W,G", [(2, 64, 9, 7, 8), (2, 320, 8, 12, 32), (1, 40, 16, 13, 4)])
def test_groupnorm(dtype, tokens_out, split, B, C, H, W, G):
    # the second and third shapes take the two-kernel path when split is set (H W a multiple of the vector width),
    # with token tiles of 64 that end ragged (96 and 208 tokens)
    x = draw((B, C, H, W), 7, dtype, 2.0, -0.5)
    g = draw((C,), 8, dtype, 0.2, 1.0)
    b = draw((C,), 9, dtype, 0.2)
    y = sm.groupnorm(dev(x, dtype), dev(g, dtype), dev(b, dtype), G, tokens_out=tokens_out, split=split)
    want = O.group_norm_nchw(to_np(x), G, to_np(g), to_np(b))
    if tokens_out:
        want = V.apply_chain(want, V.nchw_to_tokens_chain(B, C, H, W))
    assert_close(y, want, dtype, "groupnorm", 4.0)


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("M,N,K", [(70, 96, 96), (300, 288, 96), (129, 130, 200), (1000, 384, 1536), (9000, 256, 64)])
def test_linear_plain_bias_gelu_residual(dtype, M, N, K):
    if dtype == torch.bfloat16 and N % 2:
        pytest.skip("odd N")
    A = draw((M, K), 10, dtype)
    W = draw((N, K), 11, dtype, K ** -0.5)
    b = draw((N,), 12, dtype)
    R = draw((M, N), 13, dtype)
    want = O.linear(to_np(A), to_np(W))
    scale = float(np.abs(want).max()) + 1.0
    assert_close(sm.linear(dev(A, dtype), dev(W, dtype)), want, dtype, "A W^T", scale)
    want = O.gelu(O.linear(to_np(A), to_np(W), to_np(b)))
    assert_close(sm.linear(dev(A, dtype), dev(W, dtype), dev(b, dtype), act="gelu"), want, dtype, "gelu(A W^T + b)", scale)
    want = O.linear(to_np(A), to_np(W), to_np(b)) + to_np(R)
    assert_close(sm.linear(dev(A, dtype), dev(W, dtype), dev(b, dtype), residual=dev(R, dtype)), want, dtype, "+residual", scale)


@pytest.mark.parametrize("dtype", DT)
def test_linear_row_maps(dtype):
    # A rows gathered through the window map; C rows (and the residual) scattered back
    B, H, W, C, w, s, N = 2, 14, 14, 64, 7, 3, 96
    x = draw((B, H, W, C), 14, dtype)
    Wt = draw((N, C), 15, dtype, C ** -0.5)
    part = V.window_partition_chain(B, H, W, C, w, s)
    a_map = sm.Map.create((B, H, W, C), part)
    got = sm.linear(dev(x, dtype), dev(Wt, dtype), a_map=a_map, M=B * H * W)
    want = O.linear(V.apply_chain(to_np(x), part).reshape(-1, C), to_np(Wt))
    assert_close(got, want, dtype, "gathered A", 4.0)
    # scatter: natural row (window-major) -> position in the [B,H,W,N] tensor
    R = draw((B, H, W, N), 16, dtype)
    xw = draw((B * H * W, C), 17, dtype)
    c_map = sm.Map.create((B, H, W, N), V.window_partition_chain(B, H, W, N, w, s))
    got = sm.linear(dev(xw, dtype), dev(Wt, dtype), residual=dev(R, dtype), c_map=c_map)
    y = O.linear(to_np(xw), to_np(Wt)).reshape(-1, w * w, N)
    want = V.apply_chain(y, V.window_reverse_chain(B, H, W, N, w, s)) + to_np(R)
    assert_close(got.reshape(want.shape), want, dtype, "scattered C + residual", 4.0)


@pytest.mark.parametrize("act", ["swiglu", "geglu"])
def test_linear_gated(act):
    dtype = torch.bfloat16
    M, K, F = 150, 128, 192
    A = draw((M, K), 18, dtype)
    W = draw((2 * F, K), 19, dtype, K ** -0.5)
    b = draw((2 * F,), 20, dtype, 0.5)
    z = O.linear(to_np(A), to_np(W), to_np(b))
    want = O.silu(z[:, :F]) * z[:, F:] if act == "swiglu" else z[:, :F] * O.gelu(z[:, F:])
    assert_close(sm.linear(dev(A, dtype), dev(W, dtype), dev(b, dtype), act=act), want, dtype, act)


def test_linear_rope_epilogue():
    dtype = torch.bfloat16
    Bn, S, E, h = 2, 80, 256, 2       # head size 128
    d = E // h
    A = draw((Bn * S, 64), 21, dtype)
    W = draw((3 * E, 64), 22, dtype, 0.125)
    got = to_np(sm.linear(dev(A, dtype), dev(W, dtype), rope=(2 * E, d, S, 10000.0)))
    z = O.linear(to_np(A), to_np(W)).reshape(Bn, S, 3, h, d)
    want = z.copy()
    for t in range(2):
        r = O.rope_half_split(np.transpose(z[:, :, t], (0, 2, 1, 3)))       # [B, h, S, d]
        want[:, :, t] = np.transpose(r, (0, 2, 1, 3))
    assert_close(got.reshape(want.shape), want, dtype, "rope(q), rope(k), v")
    # the rotation must matter at this tolerance
    assert np.linalg.norm(z - want) / np.linalg.norm(want) > 0.3


def test_linear_transposed_store():
    dtype = torch.bfloat16
    Bn, HW, K, N = 2, 72, 64, 40
    A = draw((Bn * HW, K), 23, dtype)
    W = draw((N, K), 24, dtype, 0.125)
    b = draw((N,), 25, dtype)
    R = draw((Bn, N, HW), 26, dtype)
    out = torch.empty((Bn, N, HW), dtype=dtype, device="cuda")
    sm.linear(dev(A, dtype), dev(W, dtype), dev(b, dtype), residual=dev(R, dtype), c_transposed_batch=HW, out=out)
    want = np.transpose(O.linear(to_np(A), to_np(W), to_np(b)).reshape(Bn, HW, N), (0, 2, 1)) + to_np(R)
    assert_close(out, want, dtype, "NCHW store")


# 7 x 7 windows below and above the wave count at which one wave takes both query blocks (interior, last-row,
# last-column and corner windows in each), and other window sizes (the general window kernel)
WINDOW_CASES = [(2, 14, 21, 96, 3, 7, 3), (43, 28, 28, 128, 4, 7, 3), (2, 8, 12, 64, 2, 4, 2), (1, 16, 24, 64, 2, 8, 4)]


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("shifted", [False, True])
@pytest.mark.parametrize("B,H,W,C,h,w,shift", WINDOW_CASES)
def test_window_attention_in_place_qkv(dtype, shifted, B, H, W, C, h, w, shift):
    if dtype == torch.float32 and B > 8:
        pytest.skip("the fp32 kernel does not depend on the wave count")
    s = shift if shifted else 0
    N, d = w * w, C // h
    B_ = B * (H // w) * (W // w)
    qkv = draw((B_, N, 3 * C), 27, dtype)               # O(1) logits
    table = draw(((2 * w - 1) ** 2, h), 28, dtype)      # O(1) bias
    dq, dt = dev(qkv, dtype), dev(table, dtype)
    out = torch.empty((B_, N, C), dtype=dtype, device="cuda")
    st = (N * 3 * C, d, 3 * C)
    sm.attention(dq, dq[..., C:], dq[..., 2 * C:], kind="window", rpb_table=dt, window=w, shift=s, H=H, W=W,
                 shape=(B_, h, N, N, d), q_stride=st, k_stride=st, v_stride=st, o_stride=(N * C, d, C), out=out)
    t = V.apply_chain(to_np(qkv), V.qkv_split_chain(B_, N, h, d))
    add = swin.rel_pos_bias(to_np(table), w, h)[None]
    if s:
        add = add + np.tile(swin.shift_mask(H, W, w, s), (B, 1, 1))[:, None]
    o, _ = O.attention(t[0], t[1], t[2], d ** -0.5, add=add)
    want = V.apply_chain(o, V.head_merge_chain(B_, N, h, d))
    assert_close(out, want, dtype, "window attention")
    o_nobias, _ = O.attention(t[0], t[1], t[2], d ** -0.5)
    assert np.abs(V.apply_chain(o_nobias, V.head_merge_chain(B_, N, h, d)) - want).max() > 0.1   # bias and mask matter


@pytest.mark.parametrize("kind,nq,nk,d,h", [("full", 100, 77, 40, 2), ("full", 257, 257, 40, 3), ("causal", 200, 200, 128, 2),
                                           ("causal", 64, 64, 64, 1), ("full", 33, 500, 32, 2)])
def test_global_attention_strided_heads(kind, nq, nk, d, h):
    dtype = torch.bfloat16
    Bn = 2
    q = draw((Bn, nq, h * d), 29, dtype)
    k = draw((Bn, nk, h * d), 30, dtype)
    v = draw((Bn, nk, h * d), 31, dtype)
    dq, dk, dv = dev(q, dtype), dev(k, dtype), dev(v, dtype)
    out = torch.empty((Bn, nq, h * d), dtype=dtype, device="cuda")
    sm.attention(dq, dk, dv, kind=kind, shape=(Bn, h, nq, nk, d), q_stride=(nq * h * d, d, h * d),
                 k_stride=(nk * h * d, d, h * d), v_stride=(nk * h * d, d, h * d), o_stride=(nq * h * d, d, h * d), out=out)
    sp = lambda t, n: V.apply_chain(to_np(t), V.head_split_chain(Bn, n, h, d))
    o, _ = O.attention(sp(q, nq), sp(k, nk), sp(v, nk), d ** -0.5, causal=(kind == "causal"))
    assert_close(out, V.apply_chain(o, V.head_merge_chain(Bn, nq, h, d)), dtype, kind + " attention")


def test_argument_errors():
    x = torch.zeros(4, 96, device="cuda")
    with pytest.raises(sm.SmError):
        sm.norm(x[:, :94].contiguous(), x[0, :94].contiguous())                 # C not a multiple of 4
    with pytest.raises(sm.SmError):
        sm.linear(x, torch.zeros(8, 95, device="cuda"), M=4)                  # K not a multiple of 4
    with pytest.raises(sm.SmError):
        q = torch.zeros(1, 1, 50, 32, device="cuda")
        sm.attention(q, q, q, kind="window", rpb_table=x, window=7, H=14, W=14)   # 50 != 49


def test_linear_store_splits_columns_into_heads():
    # the store absorbs a head split: natural [B, S, h*d] -> stored [B, h, S, d]
    dtype = torch.bfloat16
    Bn, S, h, d, K = 2, 45, 3, 40, 64
    A = draw((Bn * S, K), 40, dtype)
    W = draw((h * d, K), 41, dtype, 0.125)
    c_map = sm.Map.create((Bn, h, S, d), V.head_merge_chain(Bn, S, h, d))      # natural index -> stored offset
    got = sm.linear(dev(A, dtype), dev(W, dtype), c_map=c_map)
    want = V.apply_chain(O.linear(to_np(A), to_np(W)).reshape(Bn, S, h * d), V.head_split_chain(Bn, S, h, d))
    assert_close(got.reshape(want.shape), want, dtype, "head-major store")


@pytest.mark.parametrize("kind,nq,nk,d,h", [("full", 130, 64, 32, 1), ("full", 300, 1, 40, 2), ("causal", 129, 129, 96, 2),
                                           ("causal", 515, 515, 128, 1), ("full", 128, 191, 72, 1), ("full", 64, 130, 128, 2),
                                           ("causal", 1, 1, 64, 1)])
def test_global_attention_tile_edges(kind, nq, nk, d, h):
    # query tiles of 128 and key tiles of 64 with ragged ends, every head-size bucket (2, 3, 4, 6, 8 sixteenths),
    # a tile that lies entirely after the diagonal for some waves, a single key; contiguous [B, h, n, d] operands
    dtype = torch.bfloat16
    Bn = 2
    q = draw((Bn, h, nq, d), 50, dtype, 1.5)
    k = draw((Bn, h, nk, d), 51, dtype, 1.5)
    v = draw((Bn, h, nk, d), 52, dtype)
    out = sm.attention(dev(q, dtype), dev(k, dtype), dev(v, dtype), kind=kind)
    o, _ = O.attention(to_np(q), to_np(k), to_np(v), d ** -0.5, causal=(kind == "causal"))
    assert_close(out, o, dtype, "%s attention %dx%d d=%d" % (kind, nq, nk, d))


def test_global_attention_full_size_sampled_rows():
    # config-4 shape (32 heads, 2048 x 2048, d = 128, causal) in the bench's launch configuration: the oracle
    # computes sampled (head, query) rows one by one
    dtype = torch.bfloat16
    h, n, d = 32, 2048, 128
    q = draw((1, h, n, d), 53, dtype)
    k = draw((1, h, n, d), 54, dtype)
    v = draw((1, h, n, d), 55, dtype)
    out = to_np(sm.attention(dev(q, dtype), dev(k, dtype), dev(v, dtype), kind="causal").float().cpu())
    qn, kn, vn = to_np(q), to_np(k), to_np(v)
    rng = np.random.default_rng(7)
    for hh, i in [(0, 0), (31, 2047), (5, 127), (5, 128), (17, 1023)] + [(int(rng.integers(h)), int(rng.integers(n))) for _ in range(20)]:
        s = (kn[0, hh, : i + 1] @ qn[0, hh, i]) * d ** -0.5
        p = np.exp(s - s.max()); p /= p.sum()
        want = p @ vn[0, hh, : i + 1]
        assert np.linalg.norm(out[0, hh, i] - want) <= 2e-2 * np.linalg.norm(want) + 1e-3, (hh, i)


@pytest.mark.parametrize("M,N,K", [(70, 100, 64), (257, 1000, 128), (64, 36, 192), (500, 130, 64)])
def test_linear_ragged_columns_bf16(M, N, K):
    # N that cuts a 128-column tile, an 8-column store chunk and a 4-column bias run; bias, GELU and residual together
    dtype = torch.bfloat16
    A = draw((M, K), 60, dtype)
    W = draw((N, K), 61, dtype, K ** -0.5)
    b = draw((N,), 62, dtype)
    R = draw((M, N), 63, dtype)
    want = O.gelu(O.linear(to_np(A), to_np(W), to_np(b))) + to_np(R)
    got = sm.linear(dev(A, dtype), dev(W, dtype), dev(b, dtype), residual=dev(R, dtype), act="gelu")
    assert_close(got, want, dtype, "gelu(A W^T + b) + R, ragged N", float(np.abs(want).max()) + 1.0)


def test_linear_results_do_not_depend_on_tuning():
    dtype = torch.bfloat16
    M, N, K = 700, 384, 256
    A = draw((M, K), 64, dtype)
    W = draw((N, K), 65, dtype, K ** -0.5)
    b = draw((N,), 66, dtype)
    want = O.linear(to_np(A), to_np(W), to_np(b))
    ref = None
    try:
        for rows in (0, 64, 128, 256):
            for stages in (0, 2, 3, 4):
                sm.gemm_tuning(rows, stages)
                got = sm.linear(dev(A, dtype), dev(W, dtype), dev(b, dtype))
                assert_close(got, want, dtype, "tile %d stages %d" % (rows, stages), float(np.abs(want).max()) + 1.0)
                ref = got if ref is None else ref
                assert torch.equal(got, ref), "tile %d stages %d changed the result" % (rows, stages)
        with pytest.raises(sm.SmError):
            sm.gemm_tuning(96, 2)
        with pytest.raises(sm.SmError):
            sm.gemm_tuning(64, 7)
    finally:
        sm.gemm_tuning(0, 0)


def test_timing_calibration_labels():
    sm.timing_enable(True)
    try:
        sm.timing_calibrate(8)
        torch.cuda.synchronize()
        rep = sm.timing_report()
    finally:
        sm.timing_enable(False)
    assert rep["empty_kernel"][0] == 8 and rep["empty_pair"][0] == 8
    assert rep["empty_kernel"][1] > 0.0


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("kind", ["layer", "rms"])
@pytest.mark.parametrize("M,N,K", [(70, 96, 96), (300, 288, 384), (129, 130, 200), (1000, 384, 40)])
def test_linear_with_folded_norm(dtype, kind, M, N, K):
    # the norm that precedes a Linear, folded into its A-load: same result as norm then Linear (K that ends inside
    # a 64-wide tile and K below one tile included); with a row gather on A and GELU
    if dtype == torch.bfloat16 and (N % 2 or K % 8):
        pytest.skip("vector width")
    A = draw((M, K), 70, dtype, 2.0, 0.7)
    W = draw((N, K), 71, dtype, K ** -0.5)
    b = draw((N,), 72, dtype)
    g = draw((K,), 73, dtype, 0.2, 1.0)
    be = draw((K,), 74, dtype, 0.2)
    n = O.layer_norm(to_np(A), to_np(g), to_np(be)) if kind == "layer" else O.rms_norm(to_np(A), to_np(g))
    want = O.gelu(O.linear(n, to_np(W), to_np(b)))
    scale = float(np.abs(want).max()) + 1.0
    got = sm.linear(dev(A, dtype), dev(W, dtype), dev(b, dtype), act="gelu", norm=(kind, dev(g, dtype), dev(be, dtype) if kind == "layer" else None, 1e-5))
    assert_close(got, want, dtype, kind + " norm folded into the Linear", scale)


def test_empty_inputs_are_no_ops():
    # zero rows: success, nothing launched (the operand pointers of an empty tensor are null)
    dtype = torch.bfloat16
    g = torch.ones(96, dtype=dtype, device="cuda")
    x0 = torch.empty((0, 96), dtype=dtype, device="cuda")
    assert sm.norm(x0, g, g).shape == (0, 96)
    W = torch.ones((64, 96), dtype=dtype, device="cuda")
    assert sm.linear(x0, W, M=0).shape == (0, 64)
    x1 = torch.empty((0, 128), dtype=dtype, device="cuda")
    W1, W2 = torch.ones((256, 128), dtype=dtype, device="cuda"), torch.ones((128, 256), dtype=dtype, device="cuda")
    b1, b2 = torch.ones(256, dtype=dtype, device="cuda"), torch.ones(128, dtype=dtype, device="cuda")
    assert sm.mlp_fused(x1, sm.mlp_pack(W1, W2), b1, b2, M=0).shape == (0, 128)
    assert sm.linear(x1, sm.linear_pack(W1), b1, M=0, packed=True).shape == (0, 256)


@pytest.mark.parametrize("M,C,Hd", [(32, 128, 512), (70, 128, 96), (200, 256, 1024), (6272, 384, 1536), (45, 384, 160),
                                    (64, 512, 256), (130, 512, 1024), (12544, 512, 2048), (33, 512, 512),      # C = 512: the 64-token kernel
                                    (16400, 256, 1024), (16384, 384, 1536)])     # large grids: 64-token tiles from C = 256 up
@pytest.mark.parametrize("with_res,with_norm", [(True, False), (False, False), (True, True)])
def test_mlp_fused(M, C, Hd, with_res, with_norm):
    # (LayerNorm +) FC1 + GELU + FC2 (+ residual) in one kernel against the oracle's operators; row counts that end
    # inside a 32-token tile, hidden sizes that leave waves with unequal (or no) slices
    dtype = torch.bfloat16
    X = draw((M, C), 80, dtype, 2.0, 0.7)
    W1 = draw((Hd, C), 81, dtype, C ** -0.5)
    b1 = draw((Hd,), 82, dtype, 0.5)
    W2 = draw((C, Hd), 83, dtype, Hd ** -0.5)
    b2 = draw((C,), 84, dtype, 0.5)
    R = draw((M, C), 85, dtype, 1.0)
    g = draw((C,), 91, dtype, 0.2, 1.0)
    be = draw((C,), 92, dtype, 0.2)
    xin = O.layer_norm(to_np(X), to_np(g), to_np(be)) if with_norm else to_np(X)
    hid = O.gelu(O.linear(xin, to_np(W1), to_np(b1)))
    want = O.linear(hid, to_np(W2), to_np(b2)) + (to_np(R) if with_res else 0.0)
    assert sm.mlp_fused_supported(C, Hd, dtype)
    packed = sm.mlp_pack(dev(W1, dtype), dev(W2, dtype))
    got = sm.mlp_fused(dev(X, dtype), packed, dev(b1, dtype), dev(b2, dtype), dev(R, dtype) if with_res else None,
                       norm=(dev(g, dtype), dev(be, dtype), 1e-5) if with_norm else None)
    assert_close(got, want, dtype, "fused MLP", float(np.abs(want).max()) + 1.0)


def test_mlp_pack_is_a_permutation_of_the_weights():
    # bit-exact: the packed buffer holds every weight element exactly once (checked as sorted multisets of 16-byte
    # chunks' sums being equal is too weak: compare sorted raw values)
    dtype = torch.bfloat16
    W1, W2 = dev(draw((160, 128), 93, dtype), dtype), dev(draw((128, 160), 94, dtype), dtype)
    packed = sm.mlp_pack(W1, W2)
    n = W1.numel()
    a = torch.sort(packed[:n].view(torch.int16).cpu().flatten()).values
    b = torch.sort(W1.view(torch.int16).cpu().flatten()).values
    assert torch.equal(a, b)
    a = torch.sort(packed[n:].view(torch.int16).cpu().flatten()).values
    b = torch.sort(W2.view(torch.int16).cpu().flatten()).values
    assert torch.equal(a, b)


def test_mlp_fused_row_maps_and_unsupported_shapes():
    dtype = torch.bfloat16
    M, C, Hd = 4 * 49, 128, 256
    X = draw((M, C), 86, dtype)
    W1, b1 = draw((Hd, C), 87, dtype, C ** -0.5), draw((Hd,), 88, dtype, 0.3)
    W2, b2 = draw((C, Hd), 89, dtype, Hd ** -0.5), draw((C,), 90, dtype, 0.3)
    # X read through a window partition with roll
    chain_in = V.window_partition_chain(1, 14, 14, C, 7, 3)
    xm = sm.Map.create((1, 14, 14, C), chain_in)
    xin = V.apply_chain(to_np(X).reshape(1, 14, 14, C), chain_in).reshape(M, C)
    want = O.linear(O.gelu(O.linear(xin, to_np(W1), to_np(b1))), to_np(W2), to_np(b2))
    packed = sm.mlp_pack(dev(W1, dtype), dev(W2, dtype))
    got = sm.mlp_fused(dev(X, dtype), packed, dev(b1, dtype), dev(b2, dtype), x_map=xm)
    assert_close(got, want, dtype, "fused MLP with a mapped X", float(np.abs(want).max()) + 1.0)
    # the wide-row kernel (C = 512, 64-token tiles): X gathered and Y scattered through a window map, tile ends inside a window
    M, C, Hd = 3 * 49, 512, 512
    X, R = draw((M, C), 95, dtype), draw((M, C), 96, dtype)
    W1, b1 = draw((Hd, C), 97, dtype, C ** -0.5), draw((Hd,), 98, dtype, 0.3)
    W2, b2 = draw((C, Hd), 99, dtype, Hd ** -0.5), draw((C,), 100, dtype, 0.3)
    chain_in = V.window_partition_chain(3, 7, 7, C, 7, 0) + [("roll", 0, 1)]
    xm = sm.Map.create((3, 7, 7, C), chain_in)
    xin = V.apply_chain(to_np(X).reshape(3, 7, 7, C), chain_in).reshape(M, C)
    want = O.linear(O.gelu(O.linear(xin, to_np(W1), to_np(b1))), to_np(W2), to_np(b2))
    got = sm.mlp_fused(dev(X, dtype), sm.mlp_pack(dev(W1, dtype), dev(W2, dtype)), dev(b1, dtype), dev(b2, dtype), x_map=xm)
    assert_close(got, want, dtype, "wide fused MLP with a mapped X", float(np.abs(want).max()) + 1.0)
    assert not sm.mlp_fused_supported(512, 384, dtype)          # hidden must be whole rounds of 256
    assert not sm.mlp_fused_supported(96, 384, dtype)
    assert not sm.mlp_fused_supported(128, 100, dtype)
    assert not sm.mlp_fused_supported(128, 512, torch.float32)
    with pytest.raises(sm.SmError):
        sm.mlp_pack(dev(draw((384, 96), 2, dtype), dtype), dev(draw((96, 384), 4, dtype), dtype))


@pytest.mark.parametrize("M,N,K", [(32, 128, 128), (70, 96, 128), (200, 1152, 384), (6272, 384, 384), (45, 160, 256),
                                   (200, 1536, 512), (12544, 1536, 512), (45, 160, 512), (97, 96, 512)])      # K = 512: 64-token tiles
@pytest.mark.parametrize("variant", ["plain", "gelu", "res", "ln+res"])
def test_linear_with_packed_weight(M, N, K, variant):
    # the kernel that streams a packed weight into registers against the oracle: row counts that end inside a 32-row
    # tile, column counts that leave waves with unequal (or no) slices; bias, GELU, residual, folded LayerNorm
    dtype = torch.bfloat16
    A = draw((M, K), 100, dtype, 2.0, 0.7)
    W = draw((N, K), 101, dtype, K ** -0.5)
    b = draw((N,), 102, dtype, 0.5)
    R = draw((M, N), 103, dtype)
    g, be = draw((K,), 104, dtype, 0.2, 1.0), draw((K,), 105, dtype, 0.2)
    xin = O.layer_norm(to_np(A), to_np(g), to_np(be)) if "ln" in variant else to_np(A)
    want = O.linear(xin, to_np(W), to_np(b))
    if variant == "gelu":
        want = O.gelu(want)
    if "res" in variant:
        want = want + to_np(R)
    assert sm.linear_pack_supported(N, K, dtype)
    Wp = sm.linear_pack(dev(W, dtype))
    assert torch.equal(torch.sort(Wp.view(torch.int16).flatten()).values, torch.sort(dev(W, dtype).view(torch.int16).flatten()).values)
    got = sm.linear(dev(A, dtype), Wp, dev(b, dtype), residual=dev(R, dtype) if "res" in variant else None,
                    act="gelu" if variant == "gelu" else "none",
                    norm=("layer", dev(g, dtype), dev(be, dtype), 1e-5) if "ln" in variant else None, packed=True)
    assert_close(got, want, dtype, "packed-weight Linear " + variant, float(np.abs(want).max()) + 1.0)


def test_linear_with_packed_weight_row_maps_and_refusals():
    dtype = torch.bfloat16
    C = 128
    M = 4 * 49
    A = draw((M, C), 106, dtype)
    W, b = draw((96, C), 107, dtype, C ** -0.5), draw((96,), 108, dtype, 0.3)
    chain_in = V.window_partition_chain(1, 14, 14, C, 7, 3)
    am = sm.Map.create((1, 14, 14, C), chain_in)
    xin = V.apply_chain(to_np(A).reshape(1, 14, 14, C), chain_in).reshape(M, C)
    want = O.linear(xin, to_np(W), to_np(b))
    Wp = sm.linear_pack(dev(W, dtype))
    got = sm.linear(dev(A, dtype), Wp, dev(b, dtype), a_map=am, packed=True)
    assert_close(got, want, dtype, "packed-weight Linear with a gathered A", float(np.abs(want).max()) + 1.0)
    assert not sm.linear_pack_supported(96, 96, dtype)
    assert not sm.linear_pack_supported(100, 128, dtype)
    assert not sm.linear_pack_supported(128, 128, torch.float32)
    with pytest.raises(sm.SmError):
        sm.linear(dev(A, dtype), Wp, dev(b, dtype), act="swiglu", packed=True)


@pytest.mark.parametrize("M,C,Hd", [(70, 128, 96), (200, 256, 1024), (6272, 384, 1536), (130, 512, 1536), (12544, 512, 2048),
                                    (16400, 256, 1024), (16387, 384, 1536)])     # large grids: 64-token tiles
def test_mlp_fused_with_projection(M, C, Hd):
    # x1 = A . Wp^T + bp + x0, y = x1 + MLP(LayerNorm(x1)) in one kernel; x0 read and y written through a row map
    dtype = torch.bfloat16
    A = draw((M, C), 110, dtype, 1.0)
    Wp, bp = draw((C, C), 111, dtype, C ** -0.5), draw((C,), 112, dtype, 0.5)
    x0 = draw((M, C), 113, dtype, 1.0)
    W1, b1 = draw((Hd, C), 114, dtype, C ** -0.5), draw((Hd,), 115, dtype, 0.5)
    W2, b2 = draw((C, Hd), 116, dtype, Hd ** -0.5), draw((C,), 117, dtype, 0.5)
    g, be = draw((C,), 118, dtype, 0.2, 1.0), draw((C,), 119, dtype, 0.2)
    x1 = O.linear(to_np(A), to_np(Wp), to_np(bp)) + to_np(x0)
    hid = O.gelu(O.linear(O.layer_norm(x1, to_np(g), to_np(be)), to_np(W1), to_np(b1)))
    want = x1 + O.linear(hid, to_np(W2), to_np(b2))
    assert sm.lib().sm_mlp_proj_supported(C, Hd, sm.SM_BF16)
    got = sm.mlp_fused(dev(A, dtype), sm.mlp_pack(dev(W1, dtype), dev(W2, dtype)), dev(b1, dtype), dev(b2, dtype),
                       norm=(dev(g, dtype), dev(be, dtype), 1e-5),
                       proj=(sm.linear_pack(dev(Wp, dtype)), dev(bp, dtype), dev(x0, dtype)))
    assert_close(got, want, dtype, "projection + fused MLP", float(np.abs(want).max()) + 1.0)


def test_mlp_fused_with_projection_scattered_rows():
    # the window-reverse store (with roll) as the row map of the residual read and of the output
    dtype = torch.bfloat16
    C, Hd, M = 128, 256, 4 * 49
    A = draw((M, C), 120, dtype)
    Wp, bp = draw((C, C), 121, dtype, C ** -0.5), draw((C,), 122, dtype, 0.3)
    x0 = draw((M, C), 123, dtype)
    W1, b1 = draw((Hd, C), 124, dtype, C ** -0.5), draw((Hd,), 125, dtype, 0.3)
    W2, b2 = draw((C, Hd), 126, dtype, Hd ** -0.5), draw((C,), 127, dtype, 0.3)
    g, be = draw((C,), 128, dtype, 0.2, 1.0), draw((C,), 129, dtype, 0.2)
    rev = V.window_reverse_chain(1, 14, 14, C, 7, 3)
    # row r of the window-major result lands where the reverse chain puts it: as a gather, natural = reverse(window-major)
    x1_win = O.linear(to_np(A), to_np(Wp), to_np(bp))
    x1 = V.apply_chain(x1_win.reshape(4, 49, C), rev).reshape(M, C) + to_np(x0)
    hid = O.gelu(O.linear(O.layer_norm(x1, to_np(g), to_np(be)), to_np(W1), to_np(b1)))
    want = x1 + O.linear(hid, to_np(W2), to_np(b2))
    part = V.window_partition_chain(1, 14, 14, C, 7, 3)      # offset in the natural tensor of window-major row r
    ym = sm.Map.create((1, 14, 14, C), part)
    got = sm.mlp_fused(dev(A, dtype), sm.mlp_pack(dev(W1, dtype), dev(W2, dtype)), dev(b1, dtype), dev(b2, dtype),
                       norm=(dev(g, dtype), dev(be, dtype), 1e-5),
                       proj=(sm.linear_pack(dev(Wp, dtype)), dev(bp, dtype), dev(x0, dtype)), y_map=ym)
    assert_close(got, want, dtype, "projection + fused MLP through the window-reverse store", float(np.abs(want).max()) + 1.0)


def test_wide_mlp_with_projection_scattered_rows():
    # the same through the 64-token kernel (C = 512): tiles that straddle windows, a ragged last tile
    dtype = torch.bfloat16
    C, Hd, M = 512, 1536, 3 * 4 * 49
    A = draw((M, C), 140, dtype)
    Wp, bp = draw((C, C), 141, dtype, C ** -0.5), draw((C,), 142, dtype, 0.3)
    x0 = draw((M, C), 143, dtype)
    W1, b1 = draw((Hd, C), 144, dtype, C ** -0.5), draw((Hd,), 145, dtype, 0.3)
    W2, b2 = draw((C, Hd), 146, dtype, Hd ** -0.5), draw((C,), 147, dtype, 0.3)
    g, be = draw((C,), 148, dtype, 0.2, 1.0), draw((C,), 149, dtype, 0.2)
    rev = V.window_reverse_chain(3, 14, 14, C, 7, 3)
    x1_win = O.linear(to_np(A), to_np(Wp), to_np(bp))
    x1 = V.apply_chain(x1_win.reshape(12, 49, C), rev).reshape(M, C) + to_np(x0)
    hid = O.gelu(O.linear(O.layer_norm(x1, to_np(g), to_np(be)), to_np(W1), to_np(b1)))
    want = x1 + O.linear(hid, to_np(W2), to_np(b2))
    ym = sm.Map.create((3, 14, 14, C), V.window_partition_chain(3, 14, 14, C, 7, 3))
    got = sm.mlp_fused(dev(A, dtype), sm.mlp_pack(dev(W1, dtype), dev(W2, dtype)), dev(b1, dtype), dev(b2, dtype),
                       norm=(dev(g, dtype), dev(be, dtype), 1e-5),
                       proj=(sm.linear_pack(dev(Wp, dtype)), dev(bp, dtype), dev(x0, dtype)), y_map=ym)
    assert_close(got, want, dtype, "wide projection + fused MLP through the window-reverse store", float(np.abs(want).max()) + 1.0)


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("M,N,K", [(70, 96, 64), (300, 130, 200), (64, 64, 8)])
def test_linear_reads_a_transposed_operand_in_place(dtype, M, N, K):
    # A stored as [K, M] (K not contiguous at all): the transposition folded into the Linear's load, element by element
    if dtype == torch.bfloat16 and N % 2:
        pytest.skip("vector width")
    At = draw((K, M), 130, dtype)                  # the producer's layout
    W = draw((N, K), 131, dtype, K ** -0.5)
    b = draw((N,), 132, dtype, 0.5)
    want = O.linear(to_np(At).T, to_np(W), to_np(b))
    am = sm.Map.create((K, M), [("permute", (1, 0))])
    got = sm.linear(dev(At, dtype), dev(W, dtype), dev(b, dtype), a_map=am, M=M)
    assert_close(got, want, dtype, "Linear over a transposed A", float(np.abs(want).max()) + 1.0)
