"""sm_decode_step (GPT-NeoX-style layer, one new token per sequence against a key / value cache) against
oracle/decode.py: both modes, several head sizes and rotary widths, ragged key counts, an empty cache, and the
Pythia-1B-shaped step bench.py times."""
import numpy as np
import pytest
import torch

from oracle import decode as D
from paper_2404_13528_amd import binding as sm, workloads as Wl
from util import assert_bf16_close, np_params, to_np

pytestmark = pytest.mark.gpu


def run_case(B, E, h, L, F, rot, mode, seed=0, std=0.02, pitch=None):
    d = E // h
    x, p, kc, vc = Wl.neox_decode_case(B, E, h, L, F, seed=seed, bf16=True, std=std)
    want = D.neox_decode_step(to_np(x), np_params(p), to_np(kc), to_np(vc), h, rot, want_all=True)
    dev = {k: v.to(torch.bfloat16).cuda() for k, v in p.items()}
    step = sm.DecodeStep(dev, B, E, h, F, rot, mode)
    pitch = L + 1 if pitch is None else pitch
    kbuf = torch.zeros(B, h, pitch, d, dtype=torch.bfloat16, device="cuda")
    vbuf = torch.zeros_like(kbuf)
    kbuf[:, :, :L] = kc.to(torch.bfloat16).cuda()
    vbuf[:, :, :L] = vc.to(torch.bfloat16).cuda()
    k_before, v_before = kbuf.clone(), vbuf.clone()
    xd = x.to(torch.bfloat16).cuda()
    out = step(xd, kbuf, vbuf, L)
    torch.cuda.synchronize()
    n_compute, n_copy = sm.launch_counts()
    if mode == sm.SM_ELIDED:
        y = out
        assert (n_compute, n_copy) == (3, 0)
        # the step touched row L of the caches and nothing else
        assert torch.equal(kbuf[:, :, :L], k_before[:, :, :L]) and torch.equal(vbuf[:, :, :L], v_before[:, :, :L])
        assert torch.equal(kbuf[:, :, L + 1:], k_before[:, :, L + 1:]) and torch.equal(vbuf[:, :, L + 1:], v_before[:, :, L + 1:])
        k_new, v_new = kbuf[:, :, L], vbuf[:, :, L]
    else:
        y, ko, vo = out
        assert (n_compute, n_copy) == (3, 6)
        assert torch.equal(kbuf, k_before) and torch.equal(vbuf, v_before)
        assert torch.equal(ko[:, :, :L], k_before[:, :, :L]) and torch.equal(vo[:, :, :L], v_before[:, :, :L])
        k_new, v_new = ko[:, :, L], vo[:, :, L]
    assert_bf16_close(k_new.reshape(B * h, d), want["k"].reshape(B * h, d), what="new key row")
    assert_bf16_close(v_new.reshape(B * h, d), want["v"].reshape(B * h, d), what="new value row")
    assert_bf16_close(y, want["y"], x=to_np(x), what="y")
    return y, k_new, v_new


@pytest.mark.parametrize("mode", [sm.SM_ELIDED, sm.SM_EXPLICIT])
@pytest.mark.parametrize("B,E,h,L,F,rot", [
    (1, 128, 2, 5, 256, 32),        # d = 64
    (3, 256, 2, 130, 512, 64),      # d = 128, keys over several splits with a ragged tail
    (8, 512, 2, 300, 1024, 64),     # d = 256
    (5, 256, 4, 0, 320, 0),         # empty cache, no rotary features
    (32, 128, 2, 77, 192, 32),      # the largest batch
    (3, 2560, 20, 70, 2560, 32),    # rows longer than 2048: the first kernel's long-row form
])
def test_decode_step_matches_the_oracle(B, E, h, L, F, rot, mode):
    run_case(B, E, h, L, F, rot, mode, seed=B + L, std=0.1)


def test_modes_agree_and_cache_room_is_respected():
    y0, k0, v0 = run_case(4, 256, 2, 200, 512, 64, sm.SM_ELIDED, seed=11, std=0.1, pitch=260)
    y1, k1, v1 = run_case(4, 256, 2, 200, 512, 64, sm.SM_EXPLICIT, seed=11, std=0.1, pitch=260)
    assert torch.equal(y0, y1) and torch.equal(k0, k1) and torch.equal(v0, v1)


def test_stress_distribution_and_planted_mistakes():
    # O(1) logits: the softmax is far from uniform, position and rotation matter
    B, E, h, L, F, rot = 2, 256, 2, 96, 512, 64
    x, p, kc, vc = Wl.neox_decode_case(B, E, h, L, F, seed=5, bf16=True, std=0.25)
    y, _, _ = run_case(B, E, h, L, F, rot, sm.SM_ELIDED, seed=5, std=0.25)
    xn, pn, kn, vn = to_np(x), np_params(p), to_np(kc), to_np(vc)
    good = D.neox_decode_step(xn, pn, kn, vn, h, rot)[0]
    got = y.double().cpu().numpy()
    rel = lambda a, b: np.linalg.norm(a - b) / np.linalg.norm(b)
    assert rel(got, good) < 2e-2
    # an oracle with the mistake planted must be out of tolerance: no rotation; half of the cached tokens dropped
    e_rot = rel(got - xn, D.neox_decode_step(xn, pn, kn, vn, h, 0)[0] - xn)
    e_drop = rel(got - xn, D.neox_decode_step(xn, pn, kn[:, :, L // 2:], vn[:, :, L // 2:], h, rot)[0] - xn)
    assert e_rot > 3e-2 and e_drop > 3e-2, (e_rot, e_drop)


def test_refusals():
    B, E, h, L, F, rot = 2, 128, 2, 4, 256, 32
    x, p, kc, vc = Wl.neox_decode_case(B, E, h, L, F, seed=1, bf16=True)
    dev = {k: v.to(torch.bfloat16).cuda() for k, v in p.items()}
    step = sm.DecodeStep(dev, B, E, h, F, rot, sm.SM_ELIDED)
    kbuf = kc.to(torch.bfloat16).cuda().contiguous()          # pitch == L: no room for the new row
    with pytest.raises(sm.SmError):
        step(x.to(torch.bfloat16).cuda(), kbuf, kbuf.clone(), L)
    with pytest.raises(sm.SmError):
        sm.DecodeStep(dev, 33, E, h, F, rot)(torch.zeros(33, E, dtype=torch.bfloat16, device="cuda"), kbuf, kbuf, 0)


def test_pythia_1b_shaped_step_full_size():
    # the step bench.py times: B = 8, E = 2048, 8 heads x 256, MLP 8192, 64 rotary features, 2047 cached tokens
    for mode in (sm.SM_ELIDED, sm.SM_EXPLICIT):
        run_case(8, 2048, 8, 2047, 8192, 64, mode, seed=0, pitch=2048)
