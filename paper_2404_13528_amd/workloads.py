"""Seeded synthetic inputs and operator graphs of the five workloads.

This module holds no arithmetic of the method: it draws Gaussian tensors in a
fixed order from a seeded CPU generator and writes down operator graphs as
plain lists.  Both the tests of the CPU oracle and the tests / benchmark of the
HIP library take their inputs from here, so the two are fed identical data.

The paper measured pretrained models on ImageNet / MS-COCO inputs (Sec. 4.1)
and notes that the data does not affect latency; seeded Gaussians of the same
shapes stand in for them.  Recipe: inputs and the diffusion context ~ N(0,1);
every Linear weight, bias and the relative-position table ~ N(0, 0.02); norm
gains 1 + N(0, 0.02), norm shifts N(0, 0.02).  Tensors are drawn in the order
"input, then parameters in forward order".  For bf16 workloads every tensor is
rounded once to bf16 (round to nearest even) and both sides consume the
rounded values.  Linear weights are stored [out_features, in_features]: the
reduction dimension is contiguous, which is the layout the reduction-dimension
rule (Sec. 3.2.2) selects for a MatMul operand.
"""
import torch

STD = 0.02


class Draw:
    def __init__(self, seed=0, bf16=False, std=STD):
        self.g = torch.Generator(device="cpu").manual_seed(seed)
        self.bf16 = bf16
        self.std = std

    def _q(self, t):
        return t.to(torch.bfloat16).to(torch.float32) if self.bf16 else t

    def normal(self, *shape, std=1.0, mean=0.0):
        return self._q(torch.randn(*shape, generator=self.g, dtype=torch.float32) * std + mean)

    def weight(self, *shape):
        return self.normal(*shape, std=self.std)

    def gain(self, n):
        return self.normal(n, std=self.std, mean=1.0)


def swin_block_params(dr, C, h, w, mlp_ratio=4):
    p = {}
    p["ln1_g"], p["ln1_b"] = dr.gain(C), dr.weight(C)
    p["wqkv"], p["bqkv"] = dr.weight(3 * C, C), dr.weight(3 * C)
    p["rpb_table"] = dr.weight((2 * w - 1) ** 2, h)
    p["wproj"], p["bproj"] = dr.weight(C, C), dr.weight(C)
    p["ln2_g"], p["ln2_b"] = dr.gain(C), dr.weight(C)
    p["w1"], p["b1"] = dr.weight(mlp_ratio * C, C), dr.weight(mlp_ratio * C)
    p["w2"], p["b2"] = dr.weight(C, mlp_ratio * C), dr.weight(C)
    return p


def swin_block_case(B, H, W, C, h, w, seed=0, bf16=False, std=STD, in_std=1.0):
    dr = Draw(seed, bf16, std)
    x = dr.normal(B, H * W, C, std=in_std)
    return x, swin_block_params(dr, C, h, w)


def swin_stage_case(B, H, W, C, h, w, depth, seed=0, bf16=True):
    dr = Draw(seed, bf16)
    x = dr.normal(B, H * W, C)
    return x, [swin_block_params(dr, C, h, w) for _ in range(depth)]


def swin_net_case(B, img=224, patch=4, embed=128, depths=(2, 2, 18, 2), heads=(4, 8, 16, 32),
                  w=7, n_cls=1000, seed=0, bf16=True):
    dr = Draw(seed, bf16)
    image = dr.normal(B, 3, img, img)
    net = {"embed": {"w": dr.weight(embed, 3 * patch * patch), "b": dr.weight(embed),
                     "ln_g": dr.gain(embed), "ln_b": dr.weight(embed)},
           "stages": [], "merges": []}
    C = embed
    for si, (dep, h) in enumerate(zip(depths, heads)):
        net["stages"].append([swin_block_params(dr, C, h, w) for _ in range(dep)])
        if si + 1 < len(depths):
            net["merges"].append({"ln_g": dr.gain(4 * C), "ln_b": dr.weight(4 * C),
                                  "w": dr.weight(2 * C, 4 * C)})
            C *= 2
    net["head"] = {"ln_g": dr.gain(C), "ln_b": dr.weight(C),
                   "w": dr.weight(n_cls, C), "b": dr.weight(n_cls)}
    return image, net


def llama_case(B, S, E, F, seed=0, bf16=True, std=STD, in_std=1.0):
    dr = Draw(seed, bf16, std)
    x = dr.normal(B, S, E, std=in_std)
    p = {"rms1_g": dr.gain(E),
         "wq": dr.weight(E, E), "wk": dr.weight(E, E), "wv": dr.weight(E, E), "wo": dr.weight(E, E),
         "rms2_g": dr.gain(E),
         "wgate": dr.weight(F, E), "wup": dr.weight(F, E), "wdown": dr.weight(E, F)}
    return x, p


def vit_case(B, S, E, h, F, seed=0, bf16=True, std=STD, in_std=1.0):
    dr = Draw(seed, bf16, std)
    x = dr.normal(B, S, E, std=in_std)
    p = {"ln1_g": dr.gain(E), "ln1_b": dr.weight(E),
         "wqkv": dr.weight(3 * E, E), "bqkv": dr.weight(3 * E),
         "wo": dr.weight(E, E), "bo": dr.weight(E),
         "ln2_g": dr.gain(E), "ln2_b": dr.weight(E),
         "w1": dr.weight(F, E), "b1": dr.weight(F), "w2": dr.weight(E, F), "b2": dr.weight(E)}
    return x, p


def neox_decode_case(B, E, h, L, F, seed=0, bf16=True, std=STD, in_std=1.0):
    """One decode step of a GPT-NeoX / Pythia-style layer: the new token's hidden state x [B, E], the layer's
    parameters, and key / value caches [B, h, L, d] of L earlier tokens (O(1) entries, like projected activations)."""
    dr = Draw(seed, bf16, std)
    d = E // h
    x = dr.normal(B, E, std=in_std)
    p = {"ln1_g": dr.gain(E), "ln1_b": dr.weight(E),
         "wqkv": dr.weight(3 * E, E), "bqkv": dr.weight(3 * E),
         "wdense": dr.weight(E, E), "bdense": dr.weight(E),
         "ln2_g": dr.gain(E), "ln2_b": dr.weight(E),
         "w1": dr.weight(F, E), "b1": dr.weight(F), "w2": dr.weight(E, F), "b2": dr.weight(E)}
    k_cache = dr.normal(B, h, L, d, std=in_std)
    v_cache = dr.normal(B, h, L, d, std=in_std)
    return x, p, k_cache, v_cache


def cswin_qkv_case(B, H, W, C, seed=0, bf16=True, in_std=1.0):
    """Input of the cross-shaped window attention: the fused query-key-value projection of an image's tokens,
    [B, H*W, 3C], O(1) entries like any projected activation."""
    dr = Draw(seed, bf16)
    return dr.normal(B, H * W, 3 * C, std=in_std)


def cswin_lepe_params(C, seed=0, bf16=True, std=0.2):
    """Depth-wise 3 x 3 weights [C, 3, 3] and bias [C] of the locally-enhanced positional encoding (both halves of the
    channels, first half first); std 0.2 so that the encoding is a visible share of the attention output."""
    dr = Draw(seed + 1000, bf16, std)
    return dr.weight(C, 3, 3), dr.weight(C)


def cswin_block_case(B, H, W, C, mlp_ratio=4, seed=0, bf16=True, std=STD, in_std=1.0, lepe_std=0.2):
    """Input tokens [B, H*W, C] and the parameters of one CSwin block (the positional encoding's 3 x 3 weights drawn
    wider than the Linears', so that the encoding is a visible share of the attention branch)."""
    dr = Draw(seed, bf16, std)
    x = dr.normal(B, H * W, C, std=in_std)
    p = {"ln1_g": dr.gain(C), "ln1_b": dr.weight(C), "wqkv": dr.weight(3 * C, C), "bqkv": dr.weight(3 * C)}
    p["lepe_w"], p["lepe_b"] = dr.normal(C, 3, 3, std=lepe_std), dr.weight(C)
    p.update({"wproj": dr.weight(C, C), "bproj": dr.weight(C), "ln2_g": dr.gain(C), "ln2_b": dr.weight(C),
              "w1": dr.weight(mlp_ratio * C, C), "b1": dr.weight(mlp_ratio * C),
              "w2": dr.weight(C, mlp_ratio * C), "b2": dr.weight(C)})
    return x, p


def fanout_case(D1, D2, D3, Kin, Cout, seed=0, bf16=True):
    """Operands of the Fig. 4 graph: activations N(0,1), weights scaled so that every output is O(1)."""
    dr = Draw(seed, bf16)
    a = dr.normal(D2 * D3, Kin)
    w = dr.normal(D1, Kin, std=Kin ** -0.5)
    wc = dr.normal(Cout, D3, std=D3 ** -0.5)
    return a, w, wc


def sd_case(B, C, H, W, Sc, Dc, F, seed=0, bf16=True, std=STD, in_std=1.0):
    dr = Draw(seed, bf16, std)
    x = dr.normal(B, C, H, W, std=in_std)
    ctx = dr.normal(B, Sc, Dc)
    p = {"gn_g": dr.gain(C), "gn_b": dr.weight(C),
         "win": dr.weight(C, C), "bin": dr.weight(C),
         "ln1_g": dr.gain(C), "ln1_b": dr.weight(C),
         "a1_wq": dr.weight(C, C), "a1_wk": dr.weight(C, C), "a1_wv": dr.weight(C, C),
         "a1_wo": dr.weight(C, C), "a1_bo": dr.weight(C),
         "ln2_g": dr.gain(C), "ln2_b": dr.weight(C),
         "a2_wq": dr.weight(C, C), "a2_wk": dr.weight(C, Dc), "a2_wv": dr.weight(C, Dc),
         "a2_wo": dr.weight(C, C), "a2_bo": dr.weight(C),
         "ln3_g": dr.gain(C), "ln3_b": dr.weight(C),
         "ff_w1": dr.weight(2 * F, C), "ff_b1": dr.weight(2 * F),
         "ff_w2": dr.weight(C, F), "ff_b2": dr.weight(C),
         "wout": dr.weight(C, C), "bout": dr.weight(C)}
    return x, ctx, p


# ---------------------------------------------------------------------------
# Operator graphs (explicit form: every layout transformation is its own op).
# tensors: list of shapes; ops: {"kind", "in", "out", "attr"} in topological order.
# ---------------------------------------------------------------------------

class Graph:
    def __init__(self):
        self.tensors, self.ops, self.names = [], [], {}

    def tensor(self, shape, name=None):
        self.tensors.append(tuple(int(s) for s in shape))
        if name:
            self.names[name] = len(self.tensors) - 1
        return len(self.tensors) - 1

    def op(self, kind, ins, out_shape, name=None, **attr):
        out = self.tensor(out_shape)
        self.ops.append({"kind": kind, "in": list(ins), "out": out, "attr": attr, "name": name or kind})
        return out

    def find(self, name):
        return [i for i, o in enumerate(self.ops) if o["name"] == name][0]

    # layout ops
    def reshape(self, t, shape):
        return self.op("RESHAPE", [t], shape)

    def transpose(self, t, perm):
        s = self.tensors[t]
        return self.op("TRANSPOSE", [t], [s[p] for p in perm], perm=tuple(perm))

    def roll(self, t, axis, shift):
        return self.op("ROLL", [t], self.tensors[t], axis=axis, shift=shift)

    def slice(self, t, axis, start, stop):
        s = list(self.tensors[t])
        s[axis] = stop - start
        return self.op("SLICE", [t], s, axis=axis, start=start, stop=stop, step=1)

    def linear(self, t, n_out, name, bias=True):
        s = list(self.tensors[t])
        s[-1] = n_out
        y = self.op("MATMUL", [t], s, name=name, red=[len(s) - 1])
        if bias:
            y = self.op("BIAS", [y], s, name=name + ".bias")
        return y


def swin_block_graph(B, H, W, C, h, w, s):
    g = Graph()
    L, N, d = H * W, w * w, C // h
    nWy, nWx = H // w, W // w
    B_ = B * nWy * nWx
    x = g.tensor((B, L, C), "x")
    t = g.op("LAYERNORM", [x], (B, L, C), name="ln1", red=[2])
    t = g.reshape(t, (B, H, W, C))
    if s:
        t = g.roll(t, 1, -s)
        t = g.roll(t, 2, -s)
    t = g.reshape(t, (B, nWy, w, nWx, w, C))
    t = g.transpose(t, (0, 1, 3, 2, 4, 5))
    t = g.reshape(t, (B_, N, C))
    t = g.linear(t, 3 * C, "qkv")
    t = g.reshape(t, (B_, N, 3, h, d))
    t = g.transpose(t, (2, 0, 3, 1, 4))
    qkv = []
    for k in range(3):
        u = g.slice(t, 0, k, k + 1)
        qkv.append(g.reshape(u, (B_, h, N, d)))
    t = g.op("ATTENTION", qkv, (B_, h, N, d), name="attn", red=[3, 3, None])
    t = g.transpose(t, (0, 2, 1, 3))
    t = g.reshape(t, (B_, N, C))
    t = g.linear(t, C, "proj")
    t = g.reshape(t, (B, nWy, nWx, w, w, C))
    t = g.transpose(t, (0, 1, 3, 2, 4, 5))
    t = g.reshape(t, (B, H, W, C))
    if s:
        t = g.roll(t, 1, s)
        t = g.roll(t, 2, s)
    t = g.reshape(t, (B, L, C))
    x1 = g.op("ADD", [x, t], (B, L, C), name="res1")
    t = g.op("LAYERNORM", [x1], (B, L, C), name="ln2", red=[2])
    t = g.linear(t, 4 * C, "fc1")
    t = g.op("UNARY", [t], (B, L, 4 * C), name="gelu")
    t = g.linear(t, C, "fc2")
    g.op("ADD", [x1, t], (B, L, C), name="res2")
    return g


def llama_layer_graph(B, S, E, h, F):
    g = Graph()
    d = E // h
    x = g.tensor((B, S, E), "x")
    n1 = g.op("RMSNORM", [x], (B, S, E), name="rms1", red=[2])
    t = g.linear(n1, 3 * E, "qkv", bias=False)
    parts = []
    for k in range(3):
        u = g.slice(t, 2, k * E, (k + 1) * E)
        u = g.reshape(u, (B, S, h, d))
        u = g.transpose(u, (0, 2, 1, 3))
        if k < 2:
            u = g.op("ROPE", [u], (B, h, S, d), name="rope%d" % k)
        parts.append(u)
    t = g.op("ATTENTION", parts, (B, h, S, d), name="attn", red=[3, 3, None])
    t = g.transpose(t, (0, 2, 1, 3))
    t = g.reshape(t, (B, S, E))
    t = g.linear(t, E, "wo", bias=False)
    h1 = g.op("ADD", [x, t], (B, S, E), name="res1")
    n2 = g.op("RMSNORM", [h1], (B, S, E), name="rms2", red=[2])
    gu = g.linear(n2, 2 * F, "gate_up", bias=False)
    ga = g.op("UNARY", [g.slice(gu, 2, 0, F)], (B, S, F), name="silu")
    up = g.slice(gu, 2, F, 2 * F)
    act = g.op("MUL", [ga, up], (B, S, F), name="swiglu")
    t = g.linear(act, E, "down", bias=False)
    g.op("ADD", [h1, t], (B, S, E), name="res2")
    return g


def cswin_attention_graph(B, H, W, C, h, sw, lepe=True):
    """Cross-shaped window attention as an exporter writes it: q, k, v sliced out of the fused projection [B, H*W, 3C],
    per half of the channels the stripe partition (Transpose, Reshape, Transpose, Reshape) and the head split, the
    attention, head merge and stripe merge; with the positional encoding a depth-wise Conv of the values as stripe
    images (emitted before the attention) and an Add of its result.  The Concat of the two halves is left out: layout
    operators with several inputs are outside the planner."""
    g = Graph()
    L, Cb, hb, d = H * W, C // 2, h // 2, C // h
    qkv = g.tensor((B, L, 3 * C), "qkv")
    t4 = g.reshape(qkv, (B, L, 3, C))
    whole = [g.reshape(g.slice(t4, 2, k, k + 1), (B, L, C)) for k in range(3)]
    for i in range(2):
        Hs, Ws = (H, sw) if i == 0 else (sw, W)
        S, nwin = Hs * Ws, B * (H // Hs) * (W // Ws)
        part = []
        for k in range(3):
            t = g.slice(whole[k], 2, i * Cb, (i + 1) * Cb)
            t = g.transpose(t, (0, 2, 1))
            t = g.reshape(t, (B, Cb, H // Hs, Hs, W // Ws, Ws))
            t = g.transpose(t, (0, 2, 4, 3, 5, 1))
            t = g.reshape(t, (nwin, S, Cb))
            t = g.reshape(t, (nwin, S, hb, d))
            part.append(g.transpose(t, (0, 2, 1, 3)))
        pe = None
        if lepe:
            u = g.slice(whole[2], 2, i * Cb, (i + 1) * Cb)
            u = g.transpose(u, (0, 2, 1))
            u = g.reshape(u, (B, Cb, H // Hs, Hs, W // Ws, Ws))
            u = g.transpose(u, (0, 2, 4, 1, 3, 5))
            u = g.reshape(u, (nwin, Cb, Hs, Ws))
            u = g.op("CONV", [u], (nwin, Cb, Hs, Ws), name="lepe%d" % i)
            u = g.reshape(u, (nwin, hb, d, S))
            pe = g.transpose(u, (0, 1, 3, 2))
        t = g.op("ATTENTION", part, (nwin, hb, S, d), name="attn%d" % i, red=[3, 3, None])
        if lepe:
            t = g.op("ADD", [t, pe], (nwin, hb, S, d), name="add_pe%d" % i)
        t = g.transpose(t, (0, 2, 1, 3))
        t = g.reshape(t, (nwin, S, Cb))
        t = g.reshape(t, (B, H // Hs, W // Ws, Hs, Ws, Cb))
        t = g.transpose(t, (0, 1, 3, 2, 4, 5))
        g.reshape(t, (B, L, Cb))
    return g


def neox_decode_graph(B, E, h, L, F):
    """A GPT-NeoX-style layer at a decode step (one token per sequence): the fused projection viewed [B, 1, h, 3d],
    Slices and Permutes to [B, h, 1, d], rotary embedding on q and k, attention against the grown caches (graph inputs:
    the Concat that grows them has two inputs and is outside the planner), head merge, parallel residual."""
    g = Graph()
    d = E // h
    x = g.tensor((B, 1, E), "x")
    kfull = g.tensor((B, h, L + 1, d), "k_full")
    vfull = g.tensor((B, h, L + 1, d), "v_full")
    t = g.op("LAYERNORM", [x], (B, 1, E), name="ln1", red=[2])
    qkv = g.reshape(g.linear(t, 3 * E, "qkv"), (B, 1, h, 3 * d))
    part = []
    for k in range(3):
        u = g.transpose(g.slice(qkv, 3, k * d, (k + 1) * d), (0, 2, 1, 3))
        if k < 2:
            u = g.op("ROPE", [u], (B, h, 1, d), name="rope%d" % k)
        part.append(u)
    t = g.op("ATTENTION", [part[0], kfull, vfull], (B, h, 1, d), name="attn", red=[3, 3, None])
    t = g.reshape(g.transpose(t, (0, 2, 1, 3)), (B, 1, E))
    t = g.linear(t, E, "dense")
    r1 = g.op("ADD", [x, t], (B, 1, E), name="res1")
    t = g.op("LAYERNORM", [x], (B, 1, E), name="ln2", red=[2])
    t = g.linear(t, F, "fc1")
    t = g.op("UNARY", [t], (B, 1, F), name="gelu")
    t = g.linear(t, E, "fc2")
    g.op("ADD", [r1, t], (B, 1, E), name="res2")
    return g


def vit_block_graph(B, S, E, h, F):
    """A ViT encoder block: LayerNorm, fused q | k | v Linear with bias, Slices + head split, global attention, head
    merge, output Linear, residual, LayerNorm, GELU MLP, residual."""
    g = Graph()
    d = E // h
    x = g.tensor((B, S, E), "x")
    t = g.op("LAYERNORM", [x], (B, S, E), name="ln1", red=[2])
    qkv = g.linear(t, 3 * E, "qkv")
    parts = []
    for k in range(3):
        u = g.slice(qkv, 2, k * E, (k + 1) * E)
        u = g.reshape(u, (B, S, h, d))
        parts.append(g.transpose(u, (0, 2, 1, 3)))
    t = g.op("ATTENTION", parts, (B, h, S, d), name="attn", red=[3, 3, None])
    t = g.reshape(g.transpose(t, (0, 2, 1, 3)), (B, S, E))
    t = g.linear(t, E, "wo")
    h1 = g.op("ADD", [x, t], (B, S, E), name="res1")
    t = g.op("LAYERNORM", [h1], (B, S, E), name="ln2", red=[2])
    t = g.linear(t, F, "fc1")
    t = g.op("UNARY", [t], (B, S, F), name="gelu")
    t = g.linear(t, E, "fc2")
    g.op("ADD", [h1, t], (B, S, E), name="res2")
    return g


def fig4_graph(D1=6, D2=4, D3=8):
    """The simplified graph of the paper's layout-selection example (Sec. 3.2.2):
    MatMul -> Transpose -> Reshape -> {Reduce over D3, Reduce' over D1, Conv over D3}."""
    g = Graph()
    D0 = D2 * D3
    a = g.tensor((D0, 16), "a")
    t = g.op("MATMUL", [a], (D0, D1), name="matmul", red=[1])
    t = g.transpose(t, (1, 0))
    t = g.reshape(t, (D1, D2, D3))
    g.op("REDUCE", [t], (D1, D2), name="reduce", red=[2])
    g.op("REDUCE", [t], (D2, D3), name="reduce_p", red=[0])
    g.op("CONV", [t], (D1, D2, 4), name="conv", red=[2])
    return g


def random_graph(seed, max_ops=12):
    """A seeded random operator DAG over all four operator groups (planner tests): small static shapes,
    operators reading any earlier tensor, so producers with several consumers, runs of layout operators of
    any length, element-wise operators with one or two Variable producers and graph outputs behind layout
    runs all occur."""
    import random
    rnd = random.Random(seed)
    g = Graph()
    pool = [g.tensor(rnd.choice([(4, 6), (2, 3, 4), (6, 4), (2, 2, 6)])) for _ in range(rnd.randint(1, 2))]
    kinds = ["MATMUL", "LAYERNORM", "REDUCE", "UNARY", "BIAS", "ADD", "MUL",
             "RESHAPE", "TRANSPOSE", "ROLL", "SLICE", "RESHAPE", "TRANSPOSE", "GATHER"]
    for _ in range(rnd.randint(2, max_ops)):
        t = rnd.choice(pool[-4:]) if rnd.random() < 0.75 else rnd.choice(pool)
        s = g.tensors[t]
        kind = rnd.choice(kinds)
        if kind in ("ADD", "MUL"):
            same = [u for u in pool if u != t and g.tensors[u] == s]
            if not same:
                kind = "UNARY"
            else:
                pool.append(g.op(kind, [t, rnd.choice(same)], s))
                continue
        if kind == "MATMUL":
            pool.append(g.op("MATMUL", [t], s[:-1] + (rnd.choice([s[-1], 2, 5]),), red=[len(s) - 1]))
        elif kind == "LAYERNORM":
            pool.append(g.op("LAYERNORM", [t], s, red=[len(s) - 1]))
        elif kind == "REDUCE":
            ax = rnd.randrange(len(s))
            pool.append(g.op("REDUCE", [t], tuple(e if i != ax else 1 for i, e in enumerate(s)), red=[ax]))
        elif kind in ("UNARY", "BIAS", "GATHER"):
            pool.append(g.op(kind, [t], s))
        elif kind == "RESHAPE":
            n = 1
            for e in s:
                n *= e
            shapes = [sh for sh in [(n,), (2, n // 2), (n // 2, 2), (n // 4, 2, 2), (2, 2, n // 4), (3, n // 3), (n // 6, 2, 3)]
                      if all(isinstance(e, int) and e >= 1 for e in sh) and _prod(sh) == n]
            pool.append(g.reshape(t, rnd.choice(shapes)))
        elif kind == "TRANSPOSE":
            perm = list(range(len(s)))
            rnd.shuffle(perm)
            pool.append(g.transpose(t, perm))
        elif kind == "ROLL":
            ax = rnd.randrange(len(s))
            pool.append(g.roll(t, ax, rnd.randint(-s[ax], s[ax])))
        else:
            ax = rnd.randrange(len(s))
            a = rnd.randrange(s[ax])
            pool.append(g.slice(t, ax, a, rnd.randint(a + 1, s[ax])))
    return g


def _prod(sh):
    n = 1
    for e in sh:
        n *= e
    return n
