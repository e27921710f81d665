"""Host side of sm_decode_step without a GPU: the step's operator graph plans down to its compute operators, the
workspace query answers, and shapes the kernels have no variant for are refused before anything is enqueued."""
import ctypes as C
from paper_2404_13528_amd import binding as sm


def cfg(B=8, E=2048, heads=8, F=8192, rot=64, L=2047, pitch=2048):
    return sm.DecodeCfg(sm.SM_BF16, B, E, heads, F, rot, L, pitch, 10000.0, 1e-5)


def test_workspace_query_plans_the_step():
    lib = sm.lib()
    el = lib.sm_decode_step_workspace_bytes(C.byref(cfg()), sm.SM_ELIDED)
    ex = lib.sm_decode_step_workspace_bytes(C.byref(cfg()), sm.SM_EXPLICIT)
    # activations of one token per sequence and the partial results of the split reductions: well under 16 MiB; the
    # explicit chain adds the sliced q / k / v, the unmerged attention output and the copies' row tables
    assert 0 < el < 16 << 20 and el < ex < 16 << 20
    # an empty cache and the smallest shapes plan too
    assert lib.sm_decode_step_workspace_bytes(C.byref(cfg(B=1, E=64, heads=1, F=64, rot=0, L=0, pitch=1)), sm.SM_ELIDED) > 0


def test_refusals():
    lib = sm.lib()
    bad = [cfg(B=33), cfg(B=0), cfg(E=2000), cfg(heads=5), cfg(E=2048, heads=64), cfg(F=100), cfg(rot=48), cfg(L=-1),
           cfg(L=10, pitch=5), cfg(B=32, E=4096, heads=32)]
    for c in bad:
        assert lib.sm_decode_step_workspace_bytes(C.byref(c), sm.SM_ELIDED) == 0
        assert len(lib.sm_last_error()) > 0
    assert lib.sm_decode_step_workspace_bytes(C.byref(cfg()), 7) == 0
    # null pointers and the elided mode's need for room behind the cached tokens are refused by the call itself
    w = sm.DecodeWeights()
    assert lib.sm_decode_step(C.byref(cfg()), C.byref(w), None, None, None, None, None, None, None, C.c_size_t(0), sm.SM_ELIDED, None) < 0
    assert lib.sm_decode_pack(None, 64, 64, sm.SM_BF16, None, None) < 0
    assert lib.sm_decode_pack(None, 48, 64, sm.SM_BF16, None, None) < 0          # N must be a multiple of 32
