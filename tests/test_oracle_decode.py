"""Pins of oracle/decode.py (the GPT-NeoX-style decode step) against things other than itself: a full-sequence causal
forward assembled from torch CPU library routines with a complex-number rotary, closed forms and the invariants of the
rotary embedding."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import decode as D
from oracle import ops as O
from paper_2404_13528_amd import workloads as Wl
from util import np_params, to_np


def torch_neox_prefill(xs, p, h, rot, base=10000.0):
    """All tokens at once, xs [B, S, E]: library LayerNorm / linear / gelu / causal scaled-dot-product attention; the
    rotary embedding as a multiplication by e^{i pos theta} of the complex numbers (x_i + i x_{i + rot/2})."""
    B, S, E = xs.shape
    d = E // h
    t = {k: torch.from_numpy(v) for k, v in p.items()}
    x = torch.from_numpy(xs)
    n1 = F.layer_norm(x, (E,), t["ln1_g"], t["ln1_b"], 1e-5)
    qkv = F.linear(n1, t["wqkv"], t["bqkv"]).view(B, S, h, 3, d)
    q, k, v = [qkv[:, :, :, i].transpose(1, 2) for i in range(3)]                  # [B, h, S, d]
    half = rot // 2
    theta = base ** (-2.0 * torch.arange(half, dtype=torch.float64) / rot)
    ph = torch.polar(torch.ones(S, half, dtype=torch.float64), torch.arange(S, dtype=torch.float64)[:, None] * theta[None])
    def rotary(z):
        c = torch.complex(z[..., :half], z[..., half:rot]) * ph
        return torch.cat([c.real, c.imag, z[..., rot:]], -1)
    q, k = rotary(q), rotary(k)
    o = F.scaled_dot_product_attention(q, k, v, is_causal=True)
    o = o.transpose(1, 2).reshape(B, S, E)
    a = F.linear(o, t["wdense"], t["bdense"])
    n2 = F.layer_norm(x, (E,), t["ln2_g"], t["ln2_b"], 1e-5)
    m = F.linear(F.gelu(F.linear(n2, t["w1"], t["b1"])), t["w2"], t["b2"])
    return (x + a + m).numpy(), k.numpy(), v.numpy()


def test_decode_step_is_the_last_token_of_a_full_causal_forward():
    B, E, h, L, Fh, rot = 2, 64, 4, 9, 160, 8
    x, p, _, _ = Wl.neox_decode_case(B, E, h, L, Fh, seed=3, bf16=False, std=0.2)
    p = np_params(p)
    rng = np.random.default_rng(5)
    xs = rng.standard_normal((B, L + 1, E))
    y_full, k_all, v_all = torch_neox_prefill(xs, p, h, rot)
    # the caches are the keys / values of the first L tokens; the step processes token L
    y, K, Vv = D.neox_decode_step(xs[:, L], p, k_all[:, :, :L].copy(), v_all[:, :, :L].copy(), h, rot)
    assert np.abs(y - y_full[:, L]).max() < 1e-10
    assert np.abs(K - k_all).max() < 1e-12 and np.abs(Vv - v_all).max() < 1e-12       # grown caches = all keys / values
    # a wrong position, an un-rotated key or a dropped cache entry must show
    y_bad, _, _ = D.neox_decode_step(xs[:, L], p, k_all[:, :, 1:L].copy(), v_all[:, :, 1:L].copy(), h, rot)
    assert np.abs(y_bad - y_full[:, L]).max() > 1e-4


def test_empty_cache_closed_form():
    # with no cached token the softmax has one entry: the attention output is the new value itself
    B, E, h, Fh, rot = 3, 32, 2, 48, 8
    d = E // h
    x, p, kc, vc = Wl.neox_decode_case(B, E, h, 0, Fh, seed=4, bf16=False, std=0.3)
    x, p = to_np(x), np_params(p)
    y, K, Vv = D.neox_decode_step(x, p, to_np(kc), to_np(vc), h, rot)
    n1 = O.layer_norm(x, p["ln1_g"], p["ln1_b"])
    qkv = (n1 @ p["wqkv"].T + p["bqkv"]).reshape(B, h, 3, d)
    v = qkv[:, :, 2].reshape(B, E)
    n2 = O.layer_norm(x, p["ln2_g"], p["ln2_b"])
    want = x + v @ p["wdense"].T + p["bdense"] + O.gelu(n2 @ p["w1"].T + p["b1"]) @ p["w2"].T + p["b2"]
    assert np.abs(y - want).max() < 1e-12
    assert K.shape == (B, h, 1, d) and np.abs(Vv[:, :, 0] - qkv[:, :, 2]).max() < 1e-14


def test_rotary_invariants():
    rng = np.random.default_rng(0)
    d, rot = 16, 8
    q, k = rng.standard_normal((5, d)), rng.standard_normal((5, d))
    assert np.array_equal(D.rope_partial(q, 0, rot), q)                                # position 0: identity
    r = D.rope_partial(q, 7, rot)
    assert np.array_equal(r[..., rot:], q[..., rot:])                                  # features past rot untouched
    assert np.allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(q, axis=-1), atol=1e-13)      # a rotation
    # the score of a rotated pair depends on the distance of the positions only
    s1 = (D.rope_partial(q, 11, rot) * D.rope_partial(k, 4, rot)).sum(-1)
    s2 = (D.rope_partial(q, 107, rot) * D.rope_partial(k, 100, rot)).sum(-1)
    assert np.allclose(s1, s2, atol=1e-11)
    # one pair by hand: features (0, rot/2) turn by pos * theta_0 = pos
    e = np.zeros(d); e[0] = 1.0
    t = D.rope_partial(e, 0.5, rot)
    assert abs(t[0] - np.cos(0.5)) < 1e-15 and abs(t[rot // 2] - np.sin(0.5)) < 1e-15
