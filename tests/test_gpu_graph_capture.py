"""No entry point allocates, copies or synchronises: a call the library has never seen (its plan is built inside
the call) can be captured into a HIP graph, and every replay gives the eager result bit for bit."""
import pytest
import torch
from paper_2404_13528_amd import binding as sm, workloads as Wl
from util import dev, dev_params

pytestmark = pytest.mark.gpu


def _replays_match(run, eager, make_x, n=3):
    """run(x, out): the captured call; eager(x): the same call, eager, on another object."""
    x_static, y_static = make_x(0).clone(), None
    y_static = torch.empty_like(eager(x_static))
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run(x_static, y_static)
    for i in range(1, n + 1):
        x = make_x(i)
        x_static.copy_(x)
        g.replay()
        torch.cuda.synchronize()
        got = y_static.clone()
        want = eager(x)                      # the program's own eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(got, want), "replay %d differs from the eager call" % i


@pytest.mark.parametrize("mode", [sm.SM_ELIDED, sm.SM_EXPLICIT])
def test_swin_block_first_call_under_capture(mode):
    dtype = torch.bfloat16
    B, H, W, C, h, w = 3, 14, 21, 96, 3, 7
    x0, p = Wl.swin_block_case(B, H, W, C, h, w, seed=5, bf16=True)
    dp = dev_params(p, dtype)
    blk = sm.SwinBlock(B, H, W, C, h, w, 3, dp, dtype, mode)      # sizes the workspace (and plans shift 3)
    blk.cfg.shift = 2 + mode                                       # a configuration the library has not planned yet
    ref = sm.SwinBlock(B, H, W, C, h, w, 1, dp, dtype, mode)      # same workspace size, another object for the eager calls
    ref.cfg.shift = 2 + mode

    def make_x(i):
        return dev(Wl.swin_block_case(B, H, W, C, h, w, seed=10 + i, bf16=True)[0], dtype)

    # the captured call is the first with this configuration: `ref` has not run yet
    x_static = make_x(0).clone()
    y_static = torch.empty_like(x_static)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        blk(x_static, out=y_static)
    for i in range(1, 4):
        x = make_x(i)
        x_static.copy_(x)
        g.replay()
        torch.cuda.synchronize()
        got = y_static.clone()
        want = ref(x)
        torch.cuda.synchronize()
        assert torch.equal(got, want), "replay %d differs from the eager call" % i


def test_chain_and_attn_block_under_capture():
    dtype = torch.bfloat16
    B, H, W, C, h, w, depth = 2, 14, 14, 128, 4, 7, 3
    x0, blocks = Wl.swin_stage_case(B, H, W, C, h, w, depth, seed=3)
    net = {"stages": [[dev_params(p, dtype) for p in blocks]]}
    ch = sm.SwinChain(B, [(C, h, depth, H, W)], w, net, dtype, sm.SM_ELIDED)
    ref = sm.SwinChain(B, [(C, h, depth, H, W)], w, net, dtype, sm.SM_ELIDED)
    _replays_match(lambda x, out: ch(x, out=out), lambda x: ref(x),
                   lambda i: dev(Wl.swin_stage_case(B, H, W, C, h, w, 1, seed=20 + i)[0], dtype))
    Bq, S, E, hh, F = 1, 128, 256, 4, 512
    xq, pq = Wl.llama_case(Bq, S, E, F, seed=4)
    dq = dev_params(pq, dtype)
    blk = sm.AttnBlock("llama", dq, dtype, sm.SM_ELIDED, B=Bq, S=S, E=E, heads=hh, F=F)
    ref2 = sm.AttnBlock("llama", dq, dtype, sm.SM_ELIDED, B=Bq, S=S, E=E, heads=hh, F=F)
    _replays_match(lambda x, out: blk(x, out=out), lambda x: ref2(x),
                   lambda i: dev(Wl.llama_case(Bq, S, E, F, seed=30 + i)[0], dtype))


def test_decode_step_first_call_under_capture():
    # a decode step whose plan the library has not built yet, captured; every replay rewrites cache row L and must give
    # the eager result bit for bit (the arrival counters of its split reductions are zeroed by the step's first kernel)
    dtype = torch.bfloat16
    B, E, h, L, F, rot = 4, 256, 2, 333, 512, 64
    d = E // h
    x0, p, kc, vc = Wl.neox_decode_case(B, E, h, L, F, seed=9, bf16=True, std=0.1)
    dp = dev_params(p, dtype)
    step = sm.DecodeStep(dp, B, E, h, F, rot, sm.SM_ELIDED)
    ref = sm.DecodeStep(dp, B, E, h, F, rot, sm.SM_ELIDED)
    caches = []
    for _ in range(2):
        kb = torch.zeros(B, h, L + 5, d, dtype=dtype, device="cuda")
        vb = torch.zeros_like(kb)
        kb[:, :, :L], vb[:, :, :L] = dev(kc, dtype), dev(vc, dtype)
        caches.append((kb, vb))
    step.reserve(L, L + 5)
    x_static = dev(x0, dtype).clone()
    y_static = torch.empty_like(x_static)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(x_static, caches[0][0], caches[0][1], L, out=y_static)
    for i in range(1, 4):
        x = dev(Wl.neox_decode_case(B, E, h, L, F, seed=40 + i, bf16=True)[0], dtype)
        x_static.copy_(x)
        g.replay()
        torch.cuda.synchronize()
        got, k_got = y_static.clone(), caches[0][0][:, :, L].clone()
        want = ref(x, caches[1][0], caches[1][1], L)
        torch.cuda.synchronize()
        assert torch.equal(got, want) and torch.equal(k_got, caches[1][0][:, :, L]), "replay %d differs from the eager call" % i


@pytest.mark.parametrize("mode", [sm.SM_ELIDED, sm.SM_EXPLICIT])
def test_cswin_block_first_call_under_capture(mode):
    # a stripe width the library has not planned yet (the constructor planned another one; the workspace is the same
    # size): the plan is built inside the captured call, the explicit chain's row tables are filled by a kernel
    dtype = torch.bfloat16
    B, H, W, C, h = 2, 12, 12, 128, 4
    x0, p = Wl.cswin_block_case(B, H, W, C, seed=6, bf16=True, std=0.06)
    dp = dev_params(p, dtype)
    blk = sm.CswinBlock(B, H, W, C, h, 2, dp, mode)
    ref = sm.CswinBlock(B, H, W, C, h, 2, dp, mode)
    blk.cfg.sw = ref.cfg.sw = 3 + mode          # 3 or 4: never seen before this test
    x_static = dev(x0, dtype).clone()
    y_static = torch.empty_like(x_static)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        blk(x_static, out=y_static)
    for i in range(1, 4):
        x = dev(Wl.cswin_block_case(B, H, W, C, seed=50 + i, bf16=True)[0], dtype)
        x_static.copy_(x)
        g.replay()
        torch.cuda.synchronize()
        got = y_static.clone()
        want = ref(x)
        torch.cuda.synchronize()
        assert torch.equal(got, want), "replay %d differs from the eager call" % i
