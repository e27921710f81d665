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


# ---- one pin per reading the oracle planner states as data (oracle.planner.READINGS) ----

def _names(g, r):
    return {i: g.ops[i]["name"] for i in range(len(g.ops))}


def test_two_consumers_through_different_runs_go_to_the_loads():
    # one stored tensor can have one layout: MatMul -> {Transpose -> Reduce, Reshape -> Reduce'} keeps the natural
    # store and each consumer's load takes its own run (Table 5 "Eliminate 1st")
    g = Wl.Graph()
    x = g.tensor((4, 6))
    m = g.op("MATMUL", [x], (4, 6), name="mm", red=[1])
    g.op("REDUCE", [g.transpose(m, (1, 0))], (6, 1), name="r1", red=[1])
    g.op("REDUCE", [g.reshape(m, (2, 12))], (2, 1), name="r2", red=[1])
    r = P.plan(g.tensors, g.ops)
    assert r["store_chain"] == {}
    assert r["status"][1] == ("eliminated", 2, "load") and r["status"][3] == ("eliminated", 4, "load")
    assert r["action"][1] == r["action"][3] == "ELIM_1ST"
    # the transposed reader reduces over the stored dimension 0, the reshaped one over dimension 1: two copies at k=1
    assert r["layouts"][m]["red_dims"] == [0, 1] and r["layouts"][m]["n_copies"] == 2
    assert P.plan(g.tensors, g.ops, k=2)["layouts"][m]["n_copies"] == 1


def test_a_run_that_drops_elements_goes_to_the_load():
    # a store map is the inverse of the run; a Slice has none, so even with a single reader the load absorbs it
    g = Wl.Graph()
    x = g.tensor((4, 6))
    m = g.op("MATMUL", [x], (4, 6), name="mm", red=[1])
    g.op("MATMUL", [g.slice(m, 1, 0, 3)], (4, 3), name="mm2", red=[1])
    r = P.plan(g.tensors, g.ops)
    assert r["status"][1] == ("eliminated", 2, "load") and r["store_chain"] == {}
    # the same graph with a Transpose instead: one reader, invertible -> the producer's store ("Eliminate 2nd")
    g = Wl.Graph()
    x = g.tensor((4, 6))
    m = g.op("MATMUL", [x], (4, 6), name="mm", red=[1])
    g.op("MATMUL", [g.transpose(m, (1, 0))], (6, 4), name="mm2", red=[1])
    r = P.plan(g.tensors, g.ops)
    assert r["status"][1] == ("eliminated", 0, "store") and r["action"][1] == "ELIM_2ND" and r["load_chain"] == {}


def test_elementwise_operator_with_two_variable_producers():
    # Add(a, b) with independent MatMul producers: "Try fuse" applies to both pairs; the latest producer takes it
    g = Wl.Graph()
    x, y = g.tensor((4, 6)), g.tensor((4, 6))
    a = g.op("MATMUL", [x], (4, 6), name="a", red=[1])
    b = g.op("MATMUL", [y], (4, 6), name="b", red=[1])
    g.op("ADD", [a, b], (4, 6), name="add")
    r = P.plan(g.tensors, g.ops)
    assert r["status"] == [("kept",), ("kept",), ("fused", 1)] and r["node_group"][1] == "ILD_VAR"
    # residual: Add(x1, f(x1)) must not join x1's producer (the merged node would feed itself through f)
    g = Wl.Graph()
    x = g.tensor((4, 6))
    x1 = g.op("MATMUL", [x], (4, 6), name="p", red=[1])
    t = g.op("LAYERNORM", [x1], (4, 6), name="ln", red=[1])
    u = g.op("MATMUL", [t], (4, 6), name="f", red=[1])
    g.op("ADD", [u, x1], (4, 6), name="res")
    r = P.plan(g.tensors, g.ops)
    assert r["status"][3] == ("fused", 2)
    # two element-wise operators in a row with nothing layout-dependent near them stay ILI & Variable (Table 6)
    g = Wl.Graph()
    x = g.tensor((4, 6))
    g.op("UNARY", [g.op("UNARY", [x], (4, 6))], (4, 6))
    r = P.plan(g.tensors, g.ops)
    assert r["status"] == [("kept",), ("fused", 0)] and r["node_group"][0] == "ILI_VAR"


def test_output_run_is_stored_by_its_producer():
    # MatMul -> {Reduce, Transpose -> (graph output)}: nothing follows the Transpose, the MatMul stores it as well
    g = Wl.Graph()
    x = g.tensor((4, 6))
    m = g.op("MATMUL", [x], (4, 6), name="mm", red=[1])
    g.op("REDUCE", [m], (4, 1), name="r", red=[1])
    g.transpose(m, (1, 0))
    r = P.plan(g.tensors, g.ops)
    assert r["status"][2] == ("eliminated", 0, "store") and r["status"][1] == ("kept",)
    # a Fixed run between graph input and graph output meets no Variable operator: a copy
    g = Wl.Graph()
    g.reshape(g.transpose(g.tensor((4, 6)), (1, 0)), (24,))
    r = P.plan(g.tensors, g.ops)
    assert r["status"] == [("materialised",), ("materialised",)]


def _check_golden_plan(g, r, fname):
    want = rows(fname)
    name = {i: o["name"] for i, o in enumerate(g.ops)}
    kept = [name[i] for i in P.surviving(r)]
    assert kept == [l[1:] for l in want if l[0] == "kept"][0]
    fused = sorted((name[i], name[s[1]]) for i, s in enumerate(r["status"]) if s[0] == "fused")
    assert fused == sorted((l[1], l[2]) for l in want if l[0] == "fused")
    stores = sorted([name[p]] + [g.ops[f]["kind"] for f in v[3]] for p, v in r["store_chain"].items())
    assert stores == sorted(l[1:] for l in want if l[0] == "store")
    loads = sorted([name[c], str(s)] + [g.ops[f]["kind"] for f in v[2]] for (c, s), v in r["load_chain"].items())
    assert loads == sorted(l[1:] for l in want if l[0] == "load")
    for (c, s), v in r["load_chain"].items():                 # every eliminated operator names the node that took it
        for f in v[2]:
            assert ("eliminated", r["status"][c][1] if r["status"][c][0] == "fused" else c, "load") in r["absorbers"][f]


def test_hand_derived_plans_of_the_swin_block_and_the_llama_layer():
    g = Wl.swin_block_graph(2, 14, 14, 32, 2, 7, 3)
    _check_golden_plan(g, P.plan(g.tensors, g.ops), "plan_swin_block.txt")
    g = Wl.llama_layer_graph(1, 16, 64, 4, 96)
    _check_golden_plan(g, P.plan(g.tensors, g.ops), "plan_llama_layer.txt")


def test_random_graphs_reach_the_fixpoint_and_keep_every_view():
    # invariants of Sec. 3.2 on 300 random DAGs: every layout operator, and only those, is eliminated or run as a
    # copy; a fused operator names a kept one; applying a load chain to the stored tensor gives exactly the tensor
    # the explicit graph would have fed the consumer, and a store chain gives the tensor the explicit graph stores.
    for seed in range(300):
        g = Wl.random_graph(seed)
        r = P.plan(g.tensors, g.ops)
        n = len(g.ops)
        fixed = [i for i in range(n) if r["group"][i] in ("ILD_FIX", "ILI_FIX")]
        for i in range(n):
            st = r["status"][i]
            assert st[0] in ("kept", "fused", "eliminated", "materialised")
            assert (st[0] in ("eliminated", "materialised")) == (i in fixed), (seed, i, st)
            if st[0] == "fused":
                assert r["status"][st[1]] == ("kept",)
        in_chains = [f for v in r["load_chain"].values() for f in v[2]] + [f for v in r["store_chain"].values() for f in v[3]]
        assert all(f in fixed for f in in_chains)
        if any(o["kind"] == "GATHER" for o in g.ops):
            continue
        # explicit evaluation of every tensor as an index array over the graph inputs / Variable outputs
        val = {}
        for t in range(len(g.tensors)):
            val[t] = None
        for i, o in enumerate(g.ops):
            if i in fixed:
                src = val[o["in"][0]]
                base = src if src is not None else (o["in"][0], V.index_map(g.tensors[o["in"][0]], []))
                val[o["out"]] = (base[0], V.apply_chain(base[1], [P._view_of(o, g.tensors)]))
        for (c, s), (src, chain, run) in r["load_chain"].items():
            want = val[g.ops[c]["in"][s]]
            assert want is not None and want[0] == src, (seed, c, s)
            assert np.array_equal(V.index_map(g.tensors[src], chain), want[1]), (seed, c, s)
        for p_, (chain, inv, final_t, run) in r["store_chain"].items():
            first = g.ops[run[0]]["in"][0]
            assert val[final_t][0] == first and np.array_equal(V.index_map(g.tensors[first], chain), val[final_t][1])
            if inv is not None:
                back = V.index_map(g.tensors[final_t], inv).reshape(-1)
                assert np.array_equal(val[final_t][1].reshape(-1)[back], np.arange(back.size))
