"""Llama-style decoder layer, prefill (the paper's Pythia/LLM rows name the
family, Table 7; the layer definition is the public one).

Readings: RMSNorm eps 1e-5; no biases; RoPE half-split pairing (i, i + D/2),
theta_i = base^(-2i/D), applied to q and k after the head split; causal
softmax with scale D^-1/2; SwiGLU = SiLU(gate) * up.  The [B,S,H,D] <->
[B,H,S,D] permutes are materialised.
"""
from . import views as V
from . import ops as O


def llama_layer(x, p, h, base=10000.0, want_all=False):
    B, S, E = x.shape
    d = E // h
    n1 = O.rms_norm(x, p["rms1_g"])
    q = V.apply_chain(O.linear(n1, p["wq"]), V.head_split_chain(B, S, h, d))
    k = V.apply_chain(O.linear(n1, p["wk"]), V.head_split_chain(B, S, h, d))
    v = V.apply_chain(O.linear(n1, p["wv"]), V.head_split_chain(B, S, h, d))
    q = O.rope_half_split(q, base)
    k = O.rope_half_split(k, base)
    o, _ = O.attention(q, k, v, d ** -0.5, causal=True)          # [B, h, S, d]
    o = V.apply_chain(o, V.head_merge_chain(B, S, h, d))         # [B, S, E]
    h1 = x + O.linear(o, p["wo"])
    n2 = O.rms_norm(h1, p["rms2_g"])
    act = O.silu(O.linear(n2, p["wgate"])) * O.linear(n2, p["wup"])
    y = h1 + O.linear(act, p["wdown"])
    if want_all:
        return {"q": q, "k": k, "v": v, "o": o, "h1": h1, "act": act, "y": y}
    return y
