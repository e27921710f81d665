"""Pins for oracle.planner: the paper's Tables 3, 5, 6 (golden text fixtures),
the Conv+Reshape example (Sec. 3.2), the fixpoint property (Sec. 3.2.2) and the
layout-selection example of Fig. 4."""
import os
import numpy as np
from oracle import planner as P, views as V
from paper_2404_13528_amd import workloads as Wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rows(name):
    return [l.split() for l in open(os.path.join(GOLD, name)) if l.strip() and not l.startswith("#")]


def test_table3_groups():
    for op, grp in rows("table3_groups.txt"):
        assert P.GROUP_OF[op] == grp


def test_table5_and_table6():
    t5 = rows("table5_action.txt")
    t6 = rows("table6_outcome.txt")
    assert len(t5) == 16 and len(t6) == 16
    for a, b, act in t5:
        assert P.pair_action(a, b) == act
    for a, b, res, search in t6:
        assert P.pair_outcome(a, b) == (None if res == "NA" else res, search)


def two_op_graph(k1, k2):
    g = Wl.Graph()
    x = g.tensor((4, 6))

    def add(kind, t):
        if kind == "TRANSPOSE":
            return g.transpose(t, (1, 0))
        if kind == "SLICE":
            return g.slice(t, 0, 0, g.tensors[t][0])
        if kind == "MATMUL":
            return g.op("MATMUL", [t], g.tensors[t], red=[1])
        return g.op(kind, [t], g.tensors[t])
    add(k2, add(k1, x))
    return g


def test_every_pair_of_groups_on_two_op_graphs():
    rep = {"ILD_VAR": "MATMUL", "ILI_VAR": "UNARY", "ILD_FIX": "TRANSPOSE", "ILI_FIX": "SLICE"}
    for a, b, act in rows("table5_action.txt"):
        g = two_op_graph(rep[a], rep[b])
        r = P.plan(g.tensors, g.ops)
        st = r["status"]
        if act == "KEEP_BOTH":
            assert st[0] == ("kept",) and st[1] == ("kept",)
        elif act == "TRY_FUSE":
            assert (st[0][0], st[1][0]).count("fused") == 1
            keep = 0 if st[1][0] == "fused" else 1
            assert r["node_group"][keep] == P.pair_outcome(a, b)[0]
        elif act == "ELIM_2ND":
            assert st[0] == ("kept",) and st[1] == ("eliminated", 0, "store") and r["action"][1] == act
        elif act == "ELIM_1ST":
            assert st[1] == ("kept",) and st[0] == ("eliminated", 1, "load") and r["action"][0] == act
        else:
            assert st[0] == ("materialised",) and st[1] == ("materialised",)
            assert r["action"][0] == r["action"][1] == "ELIM_BOTH"


def test_conv_reshape_example():
    g = Wl.Graph()
    x = g.tensor((2, 8, 5, 5))
    c = g.op("CONV", [x], (2, 8, 5, 5), red=[1])
    g.reshape(c, (2, 8, 25))
    r = P.plan(g.tensors, g.ops)
    assert r["status"][1] == ("eliminated", 0, "store") and r["node_group"][0] == "ILD_VAR"
    assert P.pair_outcome("ILD_VAR", "ILD_FIX") == ("ILD_VAR", "SEARCH_1ST")


def test_fixpoint_only_ild_var_survive():
    for g in (Wl.swin_block_graph(1, 14, 14, 32, 2, 7, 3), Wl.swin_block_graph(2, 14, 14, 32, 2, 7, 0),
              Wl.llama_layer_graph(1, 16, 64, 4, 96)):
        r = P.plan(g.tensors, g.ops)
        sv = P.surviving(r)
        assert sv and all(r["node_group"][i] == "ILD_VAR" for i in sv)
        assert all(P.GROUP_OF[g.ops[i]["kind"]] == "ILD_VAR" for i in sv)


def test_swin_block_plan_shape():
    g = Wl.swin_block_graph(1, 14, 14, 32, 2, 7, 3)
    r = P.plan(g.tensors, g.ops)
    assert [g.ops[i]["name"] for i in P.surviving(r)] == ["ln1", "qkv", "attn", "proj", "ln2", "fc1", "fc2"]
    n_layout = sum(1 for o in g.ops if P.GROUP_OF[o["kind"]] in ("ILD_FIX", "ILI_FIX"))
    assert 18 <= n_layout <= 24                       # Table 1: 242 transforms over 12 blocks
    assert all(r["status"][i][0] == "eliminated" for i, o in enumerate(g.ops)
               if P.GROUP_OF[o["kind"]] in ("ILD_FIX", "ILI_FIX"))
    ln1, attn, proj = g.find("ln1"), g.find("attn"), g.find("proj")
    assert set(r["store_chain"]) == {ln1, attn, proj}
    assert sorted(r["load_chain"]) == [(attn, 0), (attn, 1), (attn, 2)]
    # the write-side map of ln1 is the window map, that of proj its inverse
    fwd = V.index_map((1, 14, 14, 32), V.window_partition_chain(1, 14, 14, 32, 7, 3))
    got = V.index_map(g.tensors[g.ops[ln1]["out"]], r["store_chain"][ln1][0])
    assert np.array_equal(got.reshape(-1), fwd.reshape(-1))
    inv = V.index_map(g.tensors[r["store_chain"][ln1][2]], r["store_chain"][ln1][1])
    assert np.array_equal(got.reshape(-1)[inv.reshape(-1)], np.arange(got.size))
    assert all(l["n_copies"] == 1 and l["dim_order"] == list(range(len(l["dim_order"])))
               for l in r["layouts"].values())


def test_fig4_example():
    spec = {l[0]: l[1:] for l in rows("fig4_example.txt")}
    D1, D2, D3 = 6, 4, 8
    g = Wl.fig4_graph(D1, D2, D3)
    r1 = P.plan(g.tensors, g.ops, k=1)
    r2 = P.plan(g.tensors, g.ops, k=2)
    elim = [g.ops[i]["kind"] for i, s in enumerate(r1["status"]) if s[0] == "eliminated"]
    assert elim == spec["eliminated"]
    assert [g.ops[i]["name"] for i in P.surviving(r1)] == spec["surviving"]
    stored = r1["store_chain"][0][2]
    lay1, lay2 = r1["layouts"][stored], r2["layouts"][stored]
    names = {0: "D1", 1: "D2", 2: "D3"}
    assert [names[d] for d in lay1["red_dims"]] == spec["requested_dims"]
    assert lay1["n_copies"] == int(spec["copies_k1"][0]) and lay2["n_copies"] == int(spec["copies_k2"][0])
    assert set(lay2["dim_order"][-2:]) == {0, 2}      # D1 and D3 on the two directly indexable dims
