"""Pins for oracle.ops: torch CPU library routines as an independent opinion,
closed forms, invariants and brute force."""
import math
import numpy as np
import torch
import torch.nn.functional as F
from oracle import ops as O

RNG = np.random.default_rng(7)


def T(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float64))


def test_linear_brute_force():
    x = RNG.standard_normal((5, 7)); W = RNG.standard_normal((4, 7)); b = RNG.standard_normal(4)
    got = O.linear(x, W, b)
    for i in range(5):
        for j in range(4):
            acc = b[j]
            for k in range(7):
                acc += x[i, k] * W[j, k]
            assert abs(got[i, j] - acc) < 1e-12


def test_norms_against_library_and_closed_form():
    x = RNG.standard_normal((3, 11, 32)) * 3 + 1
    g = RNG.standard_normal(32); b = RNG.standard_normal(32)
    ln = O.layer_norm(x, g, b)
    assert np.allclose(ln, F.layer_norm(T(x), (32,), T(g), T(b), 1e-5).numpy(), atol=1e-12)
    z = O.layer_norm(x, np.ones(32), np.zeros(32), eps=0.0)
    assert np.allclose(z.mean(-1), 0, atol=1e-12) and np.allclose(z.var(-1), 1, atol=1e-12)
    rn = O.rms_norm(x, g)
    assert np.allclose(rn, F.rms_norm(T(x), (32,), T(g), 1e-5).numpy(), atol=1e-12)
    xn = RNG.standard_normal((2, 8, 5, 6)) * 2 - 1
    gg = RNG.standard_normal(8); bb = RNG.standard_normal(8)
    gn = O.group_norm_nchw(xn, 4, gg, bb)
    assert np.allclose(gn, F.group_norm(T(xn), 4, T(gg), T(bb), 1e-6).numpy(), atol=1e-12)


def test_activations():
    x = np.linspace(-6, 6, 101)
    assert np.allclose(O.gelu(x), F.gelu(T(x)).numpy(), atol=1e-12)
    assert O.gelu(np.array([0.0]))[0] == 0.0 and abs(O.gelu(np.array([10.0]))[0] - 10.0) < 1e-12
    assert abs(O.gelu(np.array([1.0]))[0] - 0.5 * (1 + math.erf(1 / math.sqrt(2)))) < 1e-15
    assert np.allclose(O.silu(x), F.silu(T(x)).numpy(), atol=1e-12)


def test_softmax_rows_sum_to_one():
    s = RNG.standard_normal((4, 9, 13)) * 5
    s[0, 0, 3:] = -100.0
    p = O.softmax(s)
    assert np.allclose(p.sum(-1), 1.0, atol=1e-12)
    assert np.allclose(p, F.softmax(T(s), -1).numpy(), atol=1e-14)


def test_attention_against_library():
    q = RNG.standard_normal((2, 3, 10, 8)); k = RNG.standard_normal((2, 3, 12, 8)); v = RNG.standard_normal((2, 3, 12, 8))
    o, p = O.attention(q, k, v, 8 ** -0.5)
    assert np.allclose(o, F.scaled_dot_product_attention(T(q), T(k), T(v)).numpy(), atol=1e-12)
    k2, v2 = k[:, :, :10], v[:, :, :10]
    oc, pc = O.attention(q, k2, v2, 8 ** -0.5, causal=True)
    assert np.allclose(oc, F.scaled_dot_product_attention(T(q), T(k2), T(v2), is_causal=True).numpy(), atol=1e-12)
    assert np.all(np.triu(pc, 1) == 0) and np.allclose(pc.sum(-1), 1)
    add = RNG.standard_normal((1, 3, 10, 12))
    oa, _ = O.attention(q, k, v, 8 ** -0.5, add=add)
    assert np.allclose(oa, F.scaled_dot_product_attention(T(q), T(k), T(v), attn_mask=T(add)).numpy(), atol=1e-12)


def test_rope_properties():
    S, D = 9, 16
    q = RNG.standard_normal((2, S, D)); k = RNG.standard_normal((2, S, D))
    rq, rk = O.rope_half_split(q), O.rope_half_split(k)
    assert np.allclose(rq[:, 0], q[:, 0])                                   # position 0 is the identity
    h = D // 2
    assert np.allclose(rq[..., :h] ** 2 + rq[..., h:] ** 2, q[..., :h] ** 2 + q[..., h:] ** 2)   # per-pair norm
    # <R_p q, R_p' k> depends only on p - p': same vectors at shifted positions give equal scores
    qv, kv = RNG.standard_normal(D), RNG.standard_normal(D)
    Q = O.rope_half_split(np.tile(qv, (S, 1))); K = O.rope_half_split(np.tile(kv, (S, 1)))
    sc = Q @ K.T
    for dlt in range(-3, 4):
        diag = np.diagonal(sc, offset=dlt)
        assert np.allclose(diag, diag[0])
    # explicit pair (i, i + D/2) with theta_i = base^(-2i/D) at p = 5, i = 3
    th = 10000.0 ** (-2 * 3 / D)
    a, b = q[1, 5, 3], q[1, 5, 3 + h]
    assert abs(rq[1, 5, 3] - (a * math.cos(5 * th) - b * math.sin(5 * th))) < 1e-12
    assert abs(rq[1, 5, 3 + h] - (b * math.cos(5 * th) + a * math.sin(5 * th))) < 1e-12
