"""Host logic of the library's planner (sm_layout_plan) against the paper's
tables (golden fixtures) and, graph by graph, against the oracle planner:
groups, actions, statuses, absorbing operators, merged-node groups, composed
load / store maps (bit-exact against the oracle's iota application) and layout
decisions."""
import os
import numpy as np
import pytest
from oracle import planner as P, views as V
from paper_2404_13528_amd import binding as sm, workloads as Wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rows(name):
    return [l.split() for l in open(os.path.join(GOLD, name)) if l.strip() and not l.startswith("#")]


def test_tables_3_5_6():
    for op, grp in rows("table3_groups.txt"):
        assert sm.op_group(op) == grp
    for a, b, act in rows("table5_action.txt"):
        assert sm.pair_action(a, b) == act
    for a, b, res, search in rows("table6_outcome.txt"):
        assert sm.pair_outcome(a, b) == (None if res == "NA" else res, search)


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


GRAPHS = {
    "swin_s3": lambda: Wl.swin_block_graph(1, 14, 14, 32, 2, 7, 3),
    "swin_s0": lambda: Wl.swin_block_graph(2, 14, 21, 32, 2, 7, 0),
    "llama": lambda: Wl.llama_layer_graph(1, 16, 64, 4, 96),
    "fig4": lambda: Wl.fig4_graph(),
}
for _a in ("MATMUL", "UNARY", "TRANSPOSE", "SLICE"):
    for _b in ("MATMUL", "UNARY", "TRANSPOSE", "SLICE"):
        GRAPHS["pair_%s_%s" % (_a, _b)] = (lambda a=_a, b=_b: two_op_graph(a, b))


def status_of(st):
    if st[0] == "eliminated":
        return "eliminated_" + st[2], st[1]
    if st[0] == "fused":
        return "fused", st[1]
    if st[0] == "materialised":
        return "materialised", -1
    return "kept", None


@pytest.mark.parametrize("name", sorted(GRAPHS))
@pytest.mark.parametrize("k", [1, 2])
def test_plan_matches_oracle(name, k):
    g = GRAPHS[name]()
    want = P.plan(g.tensors, g.ops, k=k)
    got = sm.Plan(g.tensors, g.ops, k=k)
    for i in range(len(g.ops)):
        o = got.op(i)
        assert o["group"] == want["group"][i], (i, o)
        st, by = status_of(want["status"][i])
        assert o["status"] == st, (i, o, want["status"][i])
        assert o["absorbed_by"] == (i if by is None else by), (i, o, want["status"][i])
        assert o["action"] == want["action"][i], (i, o, want["action"][i])
        if st == "kept":
            assert o["node_group"] == want["node_group"][i]
    for (c, slot), (src, chain, run) in want["load_chain"].items():
        m, stored = got.load_map(c, slot)
        assert stored == src and m is not None
        assert np.array_equal(m.eval_host(), V.index_map(g.tensors[src], chain))
    for prod, (chain, inv, final_t, run) in want["store_chain"].items():
        m, stored = got.store_map(prod)
        assert stored == final_t and m is not None
        assert np.array_equal(m.eval_host(), V.index_map(g.tensors[final_t], inv))
    for i in range(len(g.ops)):
        if i not in want["store_chain"]:
            assert got.store_map(i)[0] is None
    for t in range(len(g.tensors)):
        lay = got.tensor(t)
        if t in want["layouts"]:
            w = want["layouts"][t]
            assert lay is not None and lay["dim_order"] == w["dim_order"] and lay["red_dims"] == w["red_dims"] \
                and lay["n_copies"] == w["n_copies"], (t, lay, w)
        else:
            assert lay is None, (t, lay)


def test_fig4_example_from_the_paper():
    spec = {l[0]: l[1:] for l in rows("fig4_example.txt")}
    g = Wl.fig4_graph(6, 4, 8)
    p1, p2 = sm.Plan(g.tensors, g.ops, k=1), sm.Plan(g.tensors, g.ops, k=2)
    elim = [g.ops[i]["kind"] for i in range(len(g.ops)) if p1.op(i)["status"].startswith("eliminated")]
    assert elim == spec["eliminated"]
    assert [g.ops[i]["name"] for i in range(len(g.ops)) if p1.op(i)["status"] == "kept"] == spec["surviving"]
    stored = p1.store_map(0)[1]
    names = {0: "D1", 1: "D2", 2: "D3"}
    assert [names[d] for d in p1.tensor(stored)["red_dims"]] == spec["requested_dims"]
    assert p1.tensor(stored)["n_copies"] == int(spec["copies_k1"][0])
    assert p2.tensor(stored)["n_copies"] == int(spec["copies_k2"][0])


def test_fixpoint_and_swin_maps():
    g = Wl.swin_block_graph(2, 14, 14, 32, 2, 7, 3)
    p = sm.Plan(g.tensors, g.ops)
    kept = [i for i in range(len(g.ops)) if p.op(i)["status"] == "kept"]
    assert [g.ops[i]["name"] for i in kept] == ["ln1", "qkv", "attn", "proj", "ln2", "fc1", "fc2"]
    assert all(p.op(i)["node_group"] == "ILD_VAR" for i in kept)
    # q, k, v reach attention as strided views of the QKV output: affine, unit innermost stride
    attn = g.find("attn")
    for slot in range(3):
        m, _ = p.load_map(attn, slot)
        base, strides = m.affine()
        assert base == slot * 32 and strides == (49 * 96, 16, 96, 1)


def test_bad_graphs_are_rejected():
    g = Wl.swin_block_graph(1, 14, 14, 32, 2, 7, 0)
    with pytest.raises(sm.SmError):
        sm.Plan(g.tensors, list(reversed(g.ops)))            # not topological
    with pytest.raises(sm.SmError):
        sm.Plan(g.tensors, g.ops, k=0)
