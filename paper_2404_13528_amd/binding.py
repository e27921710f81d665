"""Thin ctypes binding of libsmartmem.so: argument marshalling only.

Every computation happens inside the library's HIP kernels (or, for the
host-side planner and index-map composer, its C++ host code).  There is no
Python or CPU fallback: if the library is missing, loading raises.
torch is used for device memory and streams only.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsmartmem.so")
_lib = None

SM_OK = 0
SM_F32, SM_BF16 = 0, 1
SM_ELIDED, SM_EXPLICIT = 0, 1
MAX_RANK = 8
GROUPS = ("ILD_VAR", "ILI_VAR", "ILD_FIX", "ILI_FIX")
ACTIONS = ("KEEP_BOTH", "TRY_FUSE", "ELIM_2ND", "ELIM_1ST", "ELIM_BOTH")
SEARCH = ("SEARCH_BOTH", "SEARCH_FUSED", "SEARCH_1ST", "SEARCH_2ND", "NO_SEARCH")
STATUS = ("kept", "fused", "eliminated_store", "eliminated_load", "materialised")
OP_KIND = {"CONV": 0, "MATMUL": 1, "LAYERNORM": 2, "SOFTMAX": 3, "GROUPNORM": 4, "RMSNORM": 5,
           "ATTENTION": 6, "REDUCE": 7, "RESHAPE": 16, "TRANSPOSE": 17, "DTOS": 18, "STOD": 19,
           "UNARY": 32, "ADD": 33, "MUL": 34, "BIAS": 35, "ROPE": 36,
           "GATHER": 48, "SLICE": 49, "ROLL": 50, "CONCAT": 51}
VIEW_KIND = {"reshape": 0, "permute": 1, "roll": 2, "slice": 3}
ACT = {"none": 0, "gelu": 1, "swiglu": 2, "geglu": 3}
ATT = {"full": 0, "causal": 1, "window": 2, "stripe": 3}


class TensorDesc(C.Structure):
    _fields_ = [("rank", C.c_int32), ("shape", C.c_int64 * MAX_RANK), ("dtype", C.c_int32)]


class OpDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n_in", C.c_int32), ("in_", C.c_int32 * 4), ("out", C.c_int32),
                ("n_attr", C.c_int32), ("attr", C.c_int64 * 16)]


class ViewOp(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n", C.c_int32), ("arg", C.c_int64 * MAX_RANK)]


class LinearDesc(C.Structure):
    _fields_ = [("M", C.c_int64), ("N", C.c_int32), ("K", C.c_int32), ("dtype", C.c_int32), ("act", C.c_int32),
                ("rope_cols", C.c_int32), ("rope_dim", C.c_int32), ("rope_seq", C.c_int32), ("rope_base", C.c_float),
                ("c_transposed", C.c_int32), ("c_batch_rows", C.c_int64),
                ("norm", C.c_int32), ("norm_eps", C.c_float), ("norm_gamma", C.c_void_p), ("norm_beta", C.c_void_p),
                ("w_packed", C.c_int32)]


class AttentionDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("dtype", C.c_int32), ("nb", C.c_int32), ("heads", C.c_int32),
                ("nq", C.c_int32), ("nk", C.c_int32), ("d", C.c_int32), ("scale", C.c_float),
                ("q_stride", C.c_int64 * 3), ("k_stride", C.c_int64 * 3), ("v_stride", C.c_int64 * 3),
                ("o_stride", C.c_int64 * 3),
                ("window", C.c_int32), ("shift", C.c_int32), ("H", C.c_int32), ("W", C.c_int32),
                ("stripes", C.c_int32), ("run", C.c_int32),
                ("q_stripe", C.c_int64 * 2), ("k_stripe", C.c_int64 * 2), ("v_stripe", C.c_int64 * 2),
                ("o_stripe", C.c_int64 * 2), ("accumulate", C.c_int32), ("reserved", C.c_int32)]


class CswinCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("dtype", "B", "H", "W", "C", "heads", "sw")]


class CswinBlockCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("dtype", "B", "H", "W", "C", "heads", "sw", "mlp_ratio")] + [("eps", C.c_float)]


CSWIN_WEIGHT_NAMES = ("ln1_g", "ln1_b", "wqkv", "bqkv", "lepe_w", "lepe_b", "wproj", "bproj",
                      "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


class CswinWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in CSWIN_WEIGHT_NAMES + ("mlp_packed", "proj_packed", "qkv_packed")]


class SwinCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "H", "W", "C", "heads", "window", "shift", "mlp_ratio", "dtype")] + \
               [("eps", C.c_float)]


SWIN_WEIGHT_NAMES = ("ln1_g", "ln1_b", "wqkv", "bqkv", "rpb_table", "wproj", "bproj",
                     "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


class SwinWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in SWIN_WEIGHT_NAMES + ("mlp_packed", "proj_packed", "qkv_packed")]


def _packed_mlp(p, Cc, mlp_ratio, dtype, fuse_mlp):
    """[MLP weights, projection weight, QKV weight] of a block in the fused kernels' order (new tensors), None where there is no
    such kernel.  fuse_mlp: False (none), "mlp" (the MLP only) or True (the output projection as well)."""
    import torch
    if not fuse_mlp or not mlp_fused_supported(Cc, mlp_ratio * Cc, dtype):
        return [None, None, None]
    code = SM_BF16 if dtype == torch.bfloat16 else SM_F32
    proj = fuse_mlp is True and bool(lib().sm_mlp_proj_supported(int(Cc), int(mlp_ratio * Cc), code))
    # (at C = 512 the packed-weight Linear exists but LayerNorm + tiled Linear is as fast for QKV: not packed)
    return [mlp_pack(p["w1"], p["w2"]), linear_pack(p["wproj"]) if proj else None, linear_pack(p["wqkv"]) if proj else None]


class AttnCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kind", "dtype", "B", "S", "E", "heads", "F", "Hs", "Ws", "groups", "Sc", "Dc")] + \
               [("rope_base", C.c_float), ("eps_norm", C.c_float), ("eps_gn", C.c_float)]


class StageDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("C", "heads", "depth", "H", "W")]


class ChainDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("dtype", C.c_int32), ("window", C.c_int32), ("mlp_ratio", C.c_int32),
                ("has_embed", C.c_int32), ("in_ch", C.c_int32), ("img", C.c_int32), ("patch", C.c_int32),
                ("n_stages", C.c_int32), ("stages", StageDesc * 4),
                ("has_head", C.c_int32), ("n_cls", C.c_int32), ("eps", C.c_float)]


def lib():
    """Loads the HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libsmartmem.so is missing: run `python -m paper_2404_13528_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH, mode=C.RTLD_GLOBAL)
        L.sm_last_error.restype = C.c_char_p
        L.sm_map_numel.restype = C.c_int64
        for f in ("sm_fanout_graph_workspace_bytes", "sm_swin_block_workspace_bytes", "sm_attn_block_workspace_bytes", "sm_run_chain_workspace_bytes",
                  "sm_swin_block_static_max_bytes", "sm_decode_step_workspace_bytes",
                  "sm_cswin_attention_workspace_bytes", "sm_cswin_block_workspace_bytes"):
            getattr(L, f).restype = C.c_size_t
        _lib = L
    return _lib


class SmError(RuntimeError):
    pass


def check(rc, what=""):
    if rc < 0:
        raise SmError("%s failed (%d): %s" % (what, rc, lib().sm_last_error().decode()))
    return rc


def _tdesc(shape, dtype=SM_F32):
    t = TensorDesc()
    t.rank = len(shape)
    for i, s in enumerate(shape):
        t.shape[i] = int(s)
    t.dtype = dtype
    return t


def _view_ops(chain):
    arr = (ViewOp * max(1, len(chain)))()
    for i, op in enumerate(chain):
        v = arr[i]
        v.kind = VIEW_KIND[op[0]]
        if op[0] in ("reshape", "permute"):
            v.n = len(op[1])
            for k, a in enumerate(op[1]):
                v.arg[k] = int(a)
        elif op[0] == "roll":
            v.n = 2
            v.arg[0], v.arg[1] = int(op[1]), int(op[2])
        else:
            v.n = 4
            v.arg[0], v.arg[1], v.arg[2] = int(op[1]), int(op[2]), int(op[3])
            v.arg[3] = int(op[4]) if len(op) > 4 else 1
    return arr


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _stream(stream=None):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _dt(t):
    import torch
    if t.dtype == torch.float32:
        return SM_F32
    if t.dtype == torch.bfloat16:
        return SM_BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


class Map:
    """Handle of a composed index map (sm_map)."""

    def __init__(self, handle, owned=True):
        self.h = handle
        self.owned = owned

    @classmethod
    def create(cls, src_shape, chain):
        h = C.c_void_p()
        src = _tdesc(src_shape)
        check(lib().sm_map_create(C.byref(src), _view_ops(chain), len(chain), C.byref(h)), "sm_map_create")
        return cls(h)

    def compose(self, outer):
        h = C.c_void_p()
        check(lib().sm_map_compose(self.h, outer.h, C.byref(h)), "sm_map_compose")
        return Map(h)

    @property
    def shape(self):
        r = lib().sm_map_rank(self.h)
        s = (C.c_int64 * MAX_RANK)()
        check(lib().sm_map_shape(self.h, s), "sm_map_shape")
        return tuple(s[i] for i in range(r))

    def numel(self):
        return lib().sm_map_numel(self.h)

    def cost(self):
        a, b = C.c_int(), C.c_int()
        check(lib().sm_map_cost(self.h, C.byref(a), C.byref(b)), "sm_map_cost")
        return a.value, b.value

    def eval_host(self):
        import numpy as np
        n = self.numel()
        out = np.empty(n, dtype=np.int64)
        check(lib().sm_map_eval_host(self.h, out.ctypes.data_as(C.POINTER(C.c_int64)), C.c_int64(n)), "sm_map_eval_host")
        return out.reshape(self.shape)

    def describe(self):
        buf = C.create_string_buffer(4096)
        check(lib().sm_map_describe(self.h, buf, 4096), "sm_map_describe")
        return buf.value.decode()

    def affine(self):
        base = C.c_int64()
        st = (C.c_int64 * MAX_RANK)()
        r = check(lib().sm_map_affine(self.h, C.byref(base), st), "sm_map_affine")
        return (base.value, tuple(st[i] for i in range(len(self.shape)))) if r == 1 else None

    def gather_host(self, src):
        """numpy in, numpy out, executed by the library's host path."""
        import numpy as np
        src = np.ascontiguousarray(src)
        dt = {4: SM_F32, 2: SM_BF16}[src.dtype.itemsize]
        dst = np.empty(self.shape, dtype=src.dtype)
        check(lib().sm_gather_mapped(self.h, src.ctypes.data_as(C.c_void_p), dst.ctypes.data_as(C.c_void_p),
                                     dt, 0, None), "sm_gather_mapped")
        return dst

    def gather(self, src, out=None, stream=None):
        """torch device tensor in, torch device tensor out (HIP kernel)."""
        import torch
        assert src.is_cuda and src.is_contiguous()
        dst = torch.empty(self.shape, dtype=src.dtype, device=src.device) if out is None else out
        check(lib().sm_gather_mapped(self.h, _ptr(src), _ptr(dst), _dt(src), 1, _stream(stream)), "sm_gather_mapped")
        return dst

    def __del__(self):
        if self.owned and self.h and _lib is not None:
            _lib.sm_map_destroy(self.h)
            self.h = None


# --------------------------------------------------------------------------
# single operators (device tensors in, device tensors out)
# --------------------------------------------------------------------------

def norm(x, gamma, beta=None, eps=1e-5, rms=False, store_map=None, out=None, stream=None):
    import torch
    C_ = x.shape[-1]
    rows = x.numel() // C_
    y = torch.empty_like(x) if out is None else out
    check(lib().sm_norm(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), C.c_int64(rows), C_, C.c_float(eps),
                        int(rms), _dt(x), store_map.h if store_map else None, _stream(stream)), "sm_norm")
    return y


def groupnorm(x, gamma, beta, G, eps=1e-6, tokens_out=False, split=False, stream=None):
    """split=True passes scratch for the statistics: two fully parallel kernels instead of one workgroup per group."""
    import torch
    B, Cc, H, W = x.shape
    y = torch.empty((B, H * W, Cc) if tokens_out else x.shape, dtype=x.dtype, device=x.device)
    stats = torch.empty(2 * B * G, dtype=torch.float32, device=x.device) if split else None
    check(lib().sm_groupnorm(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), B, Cc, H * W, G, C.c_float(eps),
                             int(tokens_out), _dt(x), _ptr(stats), _stream(stream)), "sm_groupnorm")
    return y


def linear_pack_supported(N, K, dtype):
    import torch
    code = dtype if isinstance(dtype, int) else (SM_BF16 if dtype == torch.bfloat16 else SM_F32)
    return bool(lib().sm_linear_pack_supported(int(N), int(K), code))


def linear_pack(W, stream=None):
    """W [N, K] in the operand order of the packed-weight Linear kernel (same shape, new tensor)."""
    import torch
    packed = torch.empty_like(W)
    check(lib().sm_linear_pack(_ptr(W), int(W.shape[0]), int(W.shape[1]), _dt(W), _ptr(packed), _stream(stream)), "sm_linear_pack")
    return packed


def linear(A, W, bias=None, residual=None, act="none", rope=None, a_map=None, c_map=None,
           c_transposed_batch=0, out=None, M=None, norm=None, packed=False, stream=None):
    """C = epilogue(A . W^T).  rope = (rope_cols, rope_dim, seq, base) or None.
    norm = ("layer" | "rms", gamma, beta or None, eps): that norm of A's rows folded into the load.
    packed: W is linear_pack(W)."""
    import torch
    N, K = W.shape
    if M is None:
        M = A.numel() // K
    n_out = N // 2 if act in ("swiglu", "geglu") else N
    d = LinearDesc()
    d.M, d.N, d.K, d.dtype, d.act = M, N, K, _dt(A), ACT[act]
    if rope:
        d.rope_cols, d.rope_dim, d.rope_seq, d.rope_base = rope
    if norm:
        d.norm = 1 if norm[0] == "layer" else 2
        d.norm_gamma, d.norm_beta, d.norm_eps = _ptr(norm[1]).value, _ptr(norm[2]).value, norm[3]
    d.c_transposed = 1 if c_transposed_batch else 0
    d.c_batch_rows = c_transposed_batch
    d.w_packed = 1 if packed else 0
    Cm = torch.empty((M, n_out), dtype=A.dtype, device=A.device) if out is None else out
    check(lib().sm_linear(C.byref(d), _ptr(A), _ptr(W), _ptr(bias), _ptr(residual), _ptr(Cm),
                          a_map.h if a_map else None, c_map.h if c_map else None, _stream(stream)), "sm_linear")
    return Cm


def mlp_fused_supported(C_, hidden, dtype):
    import torch
    code = dtype if isinstance(dtype, int) else (SM_BF16 if dtype == torch.bfloat16 else SM_F32)
    return bool(lib().sm_mlp_fused_supported(int(C_), int(hidden), code))


class MlpDesc(C.Structure):
    _fields_ = [("M", C.c_int64), ("C", C.c_int32), ("hidden", C.c_int32), ("dtype", C.c_int32),
                ("norm", C.c_int32), ("norm_eps", C.c_float), ("norm_gamma", C.c_void_p), ("norm_beta", C.c_void_p),
                ("proj_packed", C.c_void_p), ("proj_bias", C.c_void_p), ("proj_residual", C.c_void_p)]


def linear_autotune(M, N, K, act="none", residual=False, rope=None, dtype=None, iters=20, stream=None):
    """sm_linear_autotune on scratch operands of the given shape (values do not affect the timing): the fastest tile
    variant is remembered by the library for every later Linear of that shape.  Returns a dict."""
    import torch
    dt = torch.bfloat16 if dtype is None else dtype
    g = torch.Generator(device="cpu").manual_seed(1)
    A = (torch.randn(M, K, generator=g) * 0.5).to(dt).cuda()
    W = (torch.randn(N, K, generator=g) * K ** -0.5).to(dt).cuda()
    n_out = N // 2 if act in ("swiglu", "geglu") else N
    bias = torch.zeros(N, dtype=dt, device="cuda")
    R = torch.zeros(M, n_out, dtype=dt, device="cuda") if residual else None
    Cm = torch.empty(M, n_out, dtype=dt, device="cuda")
    d = LinearDesc()
    d.M, d.N, d.K, d.dtype, d.act = M, N, K, _dt(A), ACT[act]
    if rope:
        d.rope_cols, d.rope_dim, d.rope_seq, d.rope_base = rope
    rows, stages, best, default = C.c_int(), C.c_int(), C.c_float(), C.c_float()
    check(lib().sm_linear_autotune(C.byref(d), _ptr(A), _ptr(W), _ptr(bias), _ptr(R), _ptr(Cm), int(iters), _stream(stream),
                                   C.byref(rows), C.byref(stages), C.byref(best), C.byref(default)), "sm_linear_autotune")
    return {"shape": (M, N, K), "act": act, "residual": residual, "tile_rows": rows.value, "stages": stages.value,
            "best_us": round(best.value, 2), "default_us": round(default.value, 2)}


def autotune_from_labels(labels, iters=20):
    """Tunes every distinct tiled-Linear shape among the kernel labels of a timing report (sm.timing_report() keys:
    `gemm_bf16[M,N,K]+gelu+res...`): the way to tune a whole chain without knowing how its executor is built."""
    import re
    seen, out = set(), []
    for l in labels:
        m = re.match(r"gemm_bf16\[(\d+),(\d+),(\d+)\](.*)", l)
        if not m:
            continue
        M, N, K, tail = int(m.group(1)), int(m.group(2)), int(m.group(3)), m.group(4)
        key = (M, N, K, "+gelu" in tail, "+glu" in tail, "+res" in tail)
        if key in seen or K % 64:
            continue
        seen.add(key)
        act = "gelu" if "+gelu" in tail else ("swiglu" if "+glu" in tail else "none")
        out.append(linear_autotune(M, N, K, act=act, residual="+res" in tail, iters=iters))
    return out


def mlp_pack(W1, W2, out=None, stream=None):
    """W1 [hidden, C] and W2 [C, hidden] in the fused MLP kernel's operand order (one tensor of 2 * hidden * C)."""
    import torch
    hidden, Cc = W1.shape
    packed = torch.empty(2 * hidden * Cc, dtype=W1.dtype, device=W1.device) if out is None else out
    check(lib().sm_mlp_pack(_ptr(W1), _ptr(W2), int(Cc), int(hidden), _dt(W1), _ptr(packed), _stream(stream)), "sm_mlp_pack")
    return packed


def mlp_fused(X, packed, b1, b2, residual=None, norm=None, proj=None, x_map=None, y_map=None, out=None, M=None, stream=None):
    """Y = residual + gelu(norm(X) . W1^T + b1) . W2^T + b2 in one kernel (bf16); packed = mlp_pack(W1, W2);
    norm = (gamma, beta, eps): LayerNorm of X's rows folded in.
    proj = (linear_pack(Wproj), bias, residual0): x1 = X . Wproj^T + bias + residual0 first, the MLP works on x1."""
    import torch
    hidden, Cc = b1.numel(), b2.numel()
    if M is None:
        M = X.numel() // Cc
    d = MlpDesc()
    d.M, d.C, d.hidden, d.dtype = M, Cc, hidden, _dt(X)
    if norm:
        d.norm, d.norm_gamma, d.norm_beta, d.norm_eps = 1, _ptr(norm[0]).value, _ptr(norm[1]).value, norm[2]
    if proj:
        d.proj_packed, d.proj_bias, d.proj_residual = _ptr(proj[0]).value, _ptr(proj[1]).value, _ptr(proj[2]).value
    Y = torch.empty((M, Cc), dtype=X.dtype, device=X.device) if out is None else out
    check(lib().sm_mlp_fused(C.byref(d), _ptr(X), _ptr(packed), _ptr(b1), _ptr(b2), _ptr(residual), _ptr(Y),
                             x_map.h if x_map else None, y_map.h if y_map else None, _stream(stream)), "sm_mlp_fused")
    return Y


def attention(q, k, v, kind="full", scale=None, out=None, rpb_table=None, window=0, shift=0, H=0, W=0,
              shape=None, q_stride=None, k_stride=None, v_stride=None, o_stride=None, stream=None,
              stripes=0, run=0, q_stripe=(0, 0), k_stripe=(0, 0), v_stripe=(0, 0), o_stripe=(0, 0), accumulate=False):
    """q, k, v: 4-D tensors [nb, heads, n, d] (any strides with unit innermost stride), or raw
    buffers with explicit shape = (nb, heads, nq, nk, d) and element strides (batch, head, token);
    kind "stripe": also stripes per image, tokens per run and the (stripe, run) element strides.
    accumulate: out += the result."""
    import torch
    d = AttentionDesc()
    if shape is None:
        nb, heads, nq, dd = q.shape
        nk = k.shape[2]
        q_stride, k_stride, v_stride = q.stride()[:3], k.stride()[:3], v.stride()[:3]
        if out is None:
            out = torch.empty((nb, heads, nq, dd), dtype=q.dtype, device=q.device)
        o_stride = out.stride()[:3]
    else:
        nb, heads, nq, nk, dd = shape
    d.kind, d.dtype, d.nb, d.heads, d.nq, d.nk, d.d = ATT[kind], _dt(q), nb, heads, nq, nk, dd
    d.scale = dd ** -0.5 if scale is None else scale
    for i in range(3):
        d.q_stride[i], d.k_stride[i], d.v_stride[i], d.o_stride[i] = q_stride[i], k_stride[i], v_stride[i], o_stride[i]
    d.window, d.shift, d.H, d.W = window, shift, H, W
    d.stripes, d.run, d.accumulate = stripes, run, int(bool(accumulate))
    for i in range(2):
        d.q_stripe[i], d.k_stripe[i], d.v_stripe[i], d.o_stripe[i] = q_stripe[i], k_stripe[i], v_stripe[i], o_stripe[i]
    check(lib().sm_attention(C.byref(d), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(rpb_table), _stream(stream)),
          "sm_attention")
    return out


# --------------------------------------------------------------------------
# block and chain executors
# --------------------------------------------------------------------------

def launch_counts():
    a, b = C.c_int(), C.c_int()
    lib().sm_last_launch_counts(C.byref(a), C.byref(b))
    return a.value, b.value


class SwinBlock:
    """One Swin block; owns its workspace tensor (allocated through torch, once)."""

    def __init__(self, B, H, W, Cc, heads, window, shift, params, dtype, mode=SM_ELIDED, mlp_ratio=4, eps=1e-5,
                 fuse_mlp=True):
        import torch
        self.cfg = SwinCfg(B, H, W, Cc, heads, window, shift, mlp_ratio,
                           SM_F32 if dtype == torch.float32 else SM_BF16, eps)
        self.mode = mode
        self.params = params           # keeps the device tensors alive
        # the MLP weights are packed here, once: later in-place changes of w1 / w2 need a new SwinBlock
        self.packed = _packed_mlp(params, Cc, mlp_ratio, dtype, fuse_mlp)
        self.w = SwinWeights(*([params[n].data_ptr() for n in SWIN_WEIGHT_NAMES] +
                               [t.data_ptr() if t is not None else None for t in self.packed]))
        n = lib().sm_swin_block_workspace_bytes(C.byref(self.cfg), mode)
        if n == 0:
            raise SmError("sm_swin_block_workspace_bytes: " + lib().sm_last_error().decode())
        self.ws = torch.empty(n, dtype=torch.uint8, device="cuda")

    def __call__(self, x, out=None, stream=None):
        import torch
        y = torch.empty_like(x) if out is None else out
        check(lib().sm_swin_block(C.byref(self.cfg), C.byref(self.w), _ptr(x), _ptr(y), _ptr(self.ws),
                                  C.c_size_t(self.ws.numel()), self.mode, _stream(stream)), "sm_swin_block")
        return y


def swin_block_intermediates(block):
    """Diagnostic view of an elided SwinBlock's workspace after a call made with fuse_mlp=False (one kernel per
    surviving operator): the stored intermediates in the layouts the plan gave them.  qkv and o are window-major
    ([B*nW, N, 3C] / [B*nW, N, C]: LayerNorm-1's store absorbed roll + partition), x1 and hid are in token order."""
    c = block.cfg
    T, Cc, N = c.B * c.H * c.W, c.C, c.window * c.window
    es = 4 if c.dtype == SM_F32 else 2
    tc = (T * Cc * es + 255) // 256 * 256
    import torch
    dt = torch.float32 if c.dtype == SM_F32 else torch.bfloat16

    def view(off_units, shape):
        n = 1
        for e in shape:
            n *= e
        return block.ws[off_units * tc: off_units * tc + n * es].view(dt).view(*shape)
    return {"qkv": view(1, (T // N, N, 3 * Cc)), "o": view(4, (T // N, N, Cc)), "x1": view(5, (c.B, c.H * c.W, Cc)),
            "hid": view(6, (c.B, c.H * c.W, c.mlp_ratio * Cc))}


def swin_block_static(block, x, out=None, stream=None):
    """sm_swin_block_static: `block`'s call (a SwinBlock) on the library's static workspace instead of block.ws."""
    import torch
    y = torch.empty_like(x) if out is None else out
    check(lib().sm_swin_block_static(C.byref(block.cfg), C.byref(block.w), _ptr(x), _ptr(y), block.mode, _stream(stream)),
          "sm_swin_block_static")
    return y


class SwinChain:
    """sm_run_chain: optional patch embedding, stages of Swin blocks with patch merging between them,
    optional head.  `net` follows workloads.swin_net_case ({"embed", "stages", "merges", "head"}), with
    device tensors; for a bare stage pass {"stages": [[block params...]]}."""

    def __init__(self, B, stages, window, net, dtype, mode=SM_ELIDED, img=0, patch=4, in_ch=3, n_cls=0,
                 mlp_ratio=4, eps=1e-5, fuse_mlp=True):
        import torch
        d = ChainDesc()
        d.B, d.dtype, d.window, d.mlp_ratio, d.eps = B, (SM_F32 if dtype == torch.float32 else SM_BF16), window, mlp_ratio, eps
        d.has_embed = 1 if "embed" in net else 0
        d.in_ch, d.img, d.patch = in_ch, img, patch
        d.n_stages = len(stages)
        for i, (Cc, heads, depth, H, W) in enumerate(stages):
            d.stages[i] = StageDesc(Cc, heads, depth, H, W)
        d.has_head = 1 if "head" in net else 0
        d.n_cls = n_cls
        self.desc, self.mode, self.net, self.dtype = d, mode, net, dtype
        ptrs = []
        if d.has_embed:
            ptrs += [net["embed"][k] for k in ("w", "b", "ln_g", "ln_b")]
        for si, blocks in enumerate(net["stages"]):
            for p in blocks:
                # (MLP weights packed once, here: later in-place changes of w1 / w2 need a new SwinChain)
                ptrs += [p[k] for k in SWIN_WEIGHT_NAMES] + _packed_mlp(p, stages[si][0], mlp_ratio, dtype, fuse_mlp)
            if si + 1 < len(net["stages"]):
                ptrs += [net["merges"][si][k] for k in ("ln_g", "ln_b", "w")]
        if d.has_head:
            ptrs += [net["head"][k] for k in ("ln_g", "ln_b", "w", "b")]
        self._keep = ptrs
        self.wptr = (C.c_void_p * len(ptrs))(*[t.data_ptr() if t is not None else None for t in ptrs])
        n = lib().sm_run_chain_workspace_bytes(C.byref(d), mode)
        if n == 0:
            raise SmError("sm_run_chain_workspace_bytes: " + lib().sm_last_error().decode())
        self.ws = torch.empty(n, dtype=torch.uint8, device="cuda")
        Cl, _, _, Hl, Wl = stages[-1]
        self.out_shape = (B, n_cls) if d.has_head else (B, Hl * Wl, Cl)
        self.feat_shape = (B, Hl * Wl, Cl)

    def __call__(self, x, out=None, want_feat=False, stream=None):
        import torch
        y = torch.empty(self.out_shape, dtype=self.dtype, device="cuda") if out is None else out
        feat = torch.empty(self.feat_shape, dtype=self.dtype, device="cuda") if (want_feat and self.desc.has_head) else None
        check(lib().sm_run_chain(C.byref(self.desc), self.wptr, len(self._keep), _ptr(x), _ptr(y), _ptr(feat),
                                 _ptr(self.ws), C.c_size_t(self.ws.numel()), self.mode, _stream(stream)), "sm_run_chain")
        return (y, feat) if want_feat else y


def gemm_tuning(tile_rows=0, stages=0):
    """Overrides the bf16 Linear kernel's tile height (64 / 128 / 256) and LDS stage count (2..4); 0 = automatic."""
    check(lib().sm_gemm_tuning(int(tile_rows), int(stages)), "sm_gemm_tuning")


def timing_enable(on=True):
    check(lib().sm_timing_enable(1 if on else 0), "sm_timing_enable")


def timing_calibrate(n=64, stream=None):
    """Records n empty-kernel launches under the label "empty_kernel" (timing must be enabled)."""
    check(lib().sm_timing_calibrate(int(n), _stream(stream)), "sm_timing_calibrate")


def timing_sequence():
    """Labels of the recorded launches in launch order."""
    buf = C.create_string_buffer(1 << 22)
    check(lib().sm_timing_sequence(buf, len(buf)), "sm_timing_sequence")
    return [l for l in buf.value.decode().split("\n") if l]


def timing_report():
    """{label: (launches, total_ms)} of the launches since timing_enable(True), in first-launch order."""
    buf = C.create_string_buffer(1 << 16)
    check(lib().sm_timing_report(buf, len(buf)), "sm_timing_report")
    out = {}
    for line in buf.value.decode().splitlines():
        label, n, ms = line.split("\t")
        out[label] = (int(n), float(ms))
    return out


# --------------------------------------------------------------------------
# layout planner
# --------------------------------------------------------------------------

def op_group(kind):
    g = C.c_int()
    check(lib().sm_op_group(OP_KIND[kind], C.byref(g)), "sm_op_group")
    return GROUPS[g.value]


def pair_action(first, second):
    a = C.c_int()
    check(lib().sm_pair_action(GROUPS.index(first), GROUPS.index(second), C.byref(a)), "sm_pair_action")
    return ACTIONS[a.value]


def pair_outcome(first, second):
    r, s = C.c_int(), C.c_int()
    check(lib().sm_pair_outcome(GROUPS.index(first), GROUPS.index(second), C.byref(r), C.byref(s)), "sm_pair_outcome")
    return (None if r.value < 0 else GROUPS[r.value]), SEARCH[s.value]


class Plan:
    """sm_layout_plan over a graph given as (tensor shapes, op dicts) in the form of workloads.Graph."""

    def __init__(self, tensors, ops, k=1):
        self.n_ops, self.ranks = len(ops), [len(t) for t in tensors]
        td = (TensorDesc * len(tensors))(*[_tdesc(t) for t in tensors])
        od = (OpDesc * len(ops))()
        for i, o in enumerate(ops):
            d = od[i]
            d.kind, d.n_in, d.out = OP_KIND[o["kind"]], len(o["in"]), o["out"]
            for s, t in enumerate(o["in"]):
                d.in_[s] = t
            a = o.get("attr", {})
            vals = []
            if o["kind"] == "TRANSPOSE":
                vals = list(a["perm"])
            elif o["kind"] == "ROLL":
                vals = [a["axis"], a["shift"]]
            elif o["kind"] == "SLICE":
                vals = [a["axis"], a["start"], a["stop"], a.get("step", 1)]
            elif "red" in a:
                vals = [-1 if r is None else r for r in a["red"]]
            d.n_attr = len(vals)
            for j, v in enumerate(vals):
                d.attr[j] = int(v)
        self.h = C.c_void_p()
        check(lib().sm_layout_plan(td, len(tensors), od, len(ops), k, C.byref(self.h)), "sm_layout_plan")

    def op(self, i):
        g, a, s, by, ng = C.c_int(), C.c_int(), C.c_int(), C.c_int(), C.c_int()
        check(lib().sm_plan_op(self.h, i, C.byref(g), C.byref(a), C.byref(s), C.byref(by), C.byref(ng)), "sm_plan_op")
        return {"group": GROUPS[g.value], "action": ACTIONS[a.value] if a.value >= 0 else None, "status": STATUS[s.value],
                "absorbed_by": by.value, "node_group": GROUPS[ng.value]}

    def tensor(self, t):
        order = (C.c_int * MAX_RANK)()
        red = (C.c_int * MAX_RANK)()
        nr, nc = C.c_int(), C.c_int()
        rc = lib().sm_plan_tensor(self.h, t, order, red, C.byref(nr), C.byref(nc))
        if rc < 0:
            return None
        return {"dim_order": [order[i] for i in range(self.ranks[t])], "red_dims": [red[i] for i in range(nr.value)],
                "n_copies": nc.value}

    def load_map(self, consumer, operand):
        m, t = C.c_void_p(), C.c_int()
        check(lib().sm_plan_load_map(self.h, consumer, operand, C.byref(m), C.byref(t)), "sm_plan_load_map")
        return (Map(m, owned=False) if m.value else None), t.value

    def store_map(self, producer):
        m, t = C.c_void_p(), C.c_int()
        check(lib().sm_plan_store_map(self.h, producer, C.byref(m), C.byref(t)), "sm_plan_store_map")
        return (Map(m, owned=False) if m.value else None), t.value

    def __del__(self):
        if self.h and _lib is not None:
            _lib.sm_plan_destroy(self.h)
            self.h = None


class FanoutCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("dtype", "D1", "D2", "D3", "Kin", "Cout", "k")]


class FanoutGraph:
    """sm_fanout_graph: the Fig. 4 multi-consumer graph (MatMul -> Transpose -> Reshape -> Reduce, Reduce', Conv)."""

    def __init__(self, D1, D2, D3, Kin, Cout, dtype, mode=SM_ELIDED, k=1):
        import torch
        self.cfg = FanoutCfg(SM_F32 if dtype == torch.float32 else SM_BF16, D1, D2, D3, Kin, Cout, k)
        self.mode, self.dtype = mode, dtype
        n = lib().sm_fanout_graph_workspace_bytes(C.byref(self.cfg), mode)
        if n == 0:
            raise SmError("sm_fanout_graph_workspace_bytes: " + lib().sm_last_error().decode())
        self.ws = torch.empty(n, dtype=torch.uint8, device="cuda")
        nc, nr, cb = C.c_int(), C.c_int(), C.c_size_t()
        rd = (C.c_int * 2)()
        check(lib().sm_fanout_graph_plan(C.byref(self.cfg), C.byref(nc), rd, C.byref(nr), C.byref(cb)), "sm_fanout_graph_plan")
        self.plan = {"n_copies": nc.value, "red_dims": [rd[i] for i in range(nr.value)], "copy_bytes": cb.value,
                     "workspace_bytes": n}

    def __call__(self, a, w, wconv, stream=None):
        import torch
        c = self.cfg
        r = torch.empty(c.D1, c.D2, dtype=self.dtype, device="cuda")
        rp = torch.empty(c.D2, c.D3, dtype=self.dtype, device="cuda")
        cv = torch.empty(c.D1, c.D2, c.Cout, dtype=self.dtype, device="cuda")
        check(lib().sm_fanout_graph(C.byref(c), _ptr(a), _ptr(w), _ptr(wconv), _ptr(r), _ptr(rp), _ptr(cv), _ptr(self.ws),
                                    C.c_size_t(self.ws.numel()), self.mode, _stream(stream)), "sm_fanout_graph")
        return r, rp, cv


class DecodeCfg(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("B", C.c_int32), ("E", C.c_int32), ("heads", C.c_int32), ("F", C.c_int32),
                ("rot", C.c_int32), ("L", C.c_int32), ("cache_pitch", C.c_int32), ("rope_base", C.c_float), ("eps", C.c_float)]


class DecodeWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("ln1_g", "ln1_b", "wqkv_p", "bqkv", "wdense_p", "bdense", "ln2_g", "ln2_b",
                                          "w1_p", "b1", "w2_p", "b2")]


def decode_pack(W, stream=None):
    """W [N, K] in matrix-core fragment order (same shape, new tensor): the weight layout of sm_decode_step."""
    import torch
    packed = torch.empty_like(W)
    check(lib().sm_decode_pack(_ptr(W), int(W.shape[0]), int(W.shape[1]), _dt(W), _ptr(packed), _stream(stream)), "sm_decode_pack")
    return packed


class DecodeStep:
    """sm_decode_step.  params follow workloads.neox_decode_case (device tensors, bf16); the four matrices are packed
    here, once (an in-place change of a matrix afterwards needs a new object).  Elided: k_cache / v_cache
    [B, heads, cache_pitch, d] are appended to in place at token L.  Explicit: returns the grown caches as new tensors."""

    def __init__(self, params, B, E, heads, F, rot, mode=SM_ELIDED, rope_base=10000.0, eps=1e-5):
        import torch
        p = params
        self._keep = {k: (decode_pack(p[k]) if k in ("wqkv", "wdense", "w1", "w2") else p[k]) for k in
                      ("ln1_g", "ln1_b", "wqkv", "bqkv", "wdense", "bdense", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")}
        k = self._keep
        self.w = DecodeWeights(*[k[n].data_ptr() for n in ("ln1_g", "ln1_b", "wqkv", "bqkv", "wdense", "bdense", "ln2_g",
                                                            "ln2_b", "w1", "b1", "w2", "b2")])
        self.B, self.E, self.heads, self.F, self.rot, self.mode = B, E, heads, F, rot, mode
        self.rope_base, self.eps = rope_base, eps
        self.ws = None

    def _cfg(self, L, pitch):
        return DecodeCfg(SM_BF16, self.B, self.E, self.heads, self.F, self.rot, int(L), int(pitch), self.rope_base, self.eps)

    def reserve(self, L, pitch):
        """Sizes the workspace for a step with L cached tokens (so that a later call, e.g. under graph capture, allocates nothing)."""
        import torch
        n = lib().sm_decode_step_workspace_bytes(C.byref(self._cfg(L, pitch)), self.mode)
        if n == 0:
            raise SmError("sm_decode_step_workspace_bytes: " + lib().sm_last_error().decode())
        if self.ws is None or self.ws.numel() < n:
            self.ws = torch.empty(n, dtype=torch.uint8, device="cuda")

    def __call__(self, x, k_cache, v_cache, L, out=None, stream=None):
        import torch
        d = self.E // self.heads
        cfg = self._cfg(L, k_cache.shape[2])
        self.reserve(L, k_cache.shape[2])
        y = torch.empty_like(x) if out is None else out
        ko = vo = None
        if self.mode == SM_EXPLICIT:
            ko = torch.empty(self.B, self.heads, L + 1, d, dtype=x.dtype, device=x.device)
            vo = torch.empty_like(ko)
        check(lib().sm_decode_step(C.byref(cfg), C.byref(self.w), _ptr(x), _ptr(k_cache), _ptr(v_cache), _ptr(y), _ptr(ko),
                                   _ptr(vo), _ptr(self.ws), C.c_size_t(self.ws.numel()), self.mode, _stream(stream)),
              "sm_decode_step")
        return (y, ko, vo) if self.mode == SM_EXPLICIT else y


class CswinAttention:
    """sm_cswin_attention: qkv [B, H*W, 3C] (bf16, device) -> [B, H*W, C]; owns its workspace (explicit mode only).
    lepe = (weights [C, 3, 3], bias [C]) adds the locally-enhanced positional encoding."""

    def __init__(self, B, H, W, Cc, heads, sw, mode=SM_ELIDED):
        import torch
        self.cfg = CswinCfg(SM_BF16, B, H, W, Cc, heads, sw)
        self.mode = mode
        n = lib().sm_cswin_attention_workspace_bytes(C.byref(self.cfg), mode)
        if n == 0:
            raise SmError("sm_cswin_attention_workspace_bytes: " + lib().sm_last_error().decode())
        self.ws = torch.empty(n, dtype=torch.uint8, device="cuda")

    def __call__(self, qkv, out=None, lepe=None, stream=None):
        import torch
        c = self.cfg
        if out is None:
            out = torch.empty(c.B, c.H * c.W, c.C, dtype=qkv.dtype, device=qkv.device)
        w, b = (None, None) if lepe is None else lepe
        check(lib().sm_cswin_attention(C.byref(self.cfg), _ptr(qkv), _ptr(w), _ptr(b), _ptr(out), _ptr(self.ws),
                                       C.c_size_t(self.ws.numel()), self.mode, _stream(stream)), "sm_cswin_attention")
        return out


class CswinBlock:
    """sm_cswin_block; params follow workloads.cswin_block_case (device tensors, bf16).  The MLP, projection and QKV
    weights are packed here, once, where a fused kernel exists for the width (fuse=False: one kernel per Linear)."""

    def __init__(self, B, H, W, Cc, heads, sw, params, mode=SM_ELIDED, mlp_ratio=4, eps=1e-5, fuse=True):
        import torch
        self.cfg = CswinBlockCfg(SM_BF16, B, H, W, Cc, heads, sw, mlp_ratio, eps)
        self.mode = mode
        self.params = params
        self.packed = _packed_mlp(params, Cc, mlp_ratio, torch.bfloat16, fuse)
        self.w = CswinWeights(*([params[n].data_ptr() for n in CSWIN_WEIGHT_NAMES] +
                                [t.data_ptr() if t is not None else None for t in self.packed]))
        n = lib().sm_cswin_block_workspace_bytes(C.byref(self.cfg), mode)
        if n == 0:
            raise SmError("sm_cswin_block_workspace_bytes: " + lib().sm_last_error().decode())
        self.ws = torch.empty(n, dtype=torch.uint8, device="cuda")

    def __call__(self, x, out=None, stream=None):
        import torch
        y = torch.empty_like(x) if out is None else out
        check(lib().sm_cswin_block(C.byref(self.cfg), C.byref(self.w), _ptr(x), _ptr(y), _ptr(self.ws),
                                   C.c_size_t(self.ws.numel()), self.mode, _stream(stream)), "sm_cswin_block")
        return y


class AttnBlock:
    """sm_attn_block: kind "llama", "sd" or "vit".  params follow workloads.llama_case / sd_case (device tensors);
    the fused weight matrices the library takes (q|k|v, gate|up, k|v) are concatenated here, once."""

    def __init__(self, kind, params, dtype, mode=SM_ELIDED, B=1, S=0, E=0, heads=1, F=0, Hs=0, Ws=0, groups=32, Sc=0, Dc=0,
                 rope_base=10000.0, eps_norm=1e-5, eps_gn=1e-6):
        import torch
        p = params
        if kind == "llama":
            ws = [p["rms1_g"], torch.cat([p["wq"], p["wk"], p["wv"]], 0).contiguous(), p["wo"], p["rms2_g"],
                  torch.cat([p["wgate"], p["wup"]], 0).contiguous(), p["wdown"]]
            k = 0
        elif kind == "vit":
            ws = [p[n] for n in ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")]
            k = 2
        else:
            ws = [p["gn_g"], p["gn_b"], p["win"], p["bin"], p["ln1_g"], p["ln1_b"],
                  torch.cat([p["a1_wq"], p["a1_wk"], p["a1_wv"]], 0).contiguous(), p["a1_wo"], p["a1_bo"],
                  p["ln2_g"], p["ln2_b"], p["a2_wq"], torch.cat([p["a2_wk"], p["a2_wv"]], 0).contiguous(), p["a2_wo"], p["a2_bo"],
                  p["ln3_g"], p["ln3_b"], p["ff_w1"], p["ff_b1"], p["ff_w2"], p["ff_b2"], p["wout"], p["bout"]]
            k = 1
            S = Hs * Ws
        self.cfg = AttnCfg(k, SM_BF16 if dtype == torch.bfloat16 else SM_F32, B, S, E, heads, F, Hs, Ws, groups, Sc, Dc,
                           rope_base, eps_norm, eps_gn)
        self._keep = ws
        self.wptr = (C.c_void_p * len(ws))(*[t.data_ptr() for t in ws])
        self.mode = mode
        n = lib().sm_attn_block_workspace_bytes(C.byref(self.cfg), mode)
        if n == 0:
            raise SmError("sm_attn_block_workspace_bytes: " + lib().sm_last_error().decode())
        self.ws = torch.empty(n, dtype=torch.uint8, device="cuda")

    def __call__(self, x, context=None, out=None, stream=None):
        import torch
        y = torch.empty_like(x) if out is None else out
        check(lib().sm_attn_block(C.byref(self.cfg), self.wptr, _ptr(x), _ptr(context), _ptr(y), _ptr(self.ws),
                                  C.c_size_t(self.ws.numel()), self.mode, _stream(stream)), "sm_attn_block")
        return y
