"""Layout planner, written as the paper states it (TEST INFRASTRUCTURE ONLY).

Sec. 3.1: every operator is one of four groups (Table 3; definitions Table 4).
Sec. 3.2: look at one producer -> consumer pair at a time, take its action from
Table 5 (keep both / try fuse / eliminate 2nd / eliminate 1st / eliminate both),
give the survivor the type of Table 6, and repeat over rounds until no pair
changes; then "all preserved operators are ILD & Variable" (Sec. 3.2.2).
Sec. 3.2.2: every stored tensor gets the layout its consumers' reduction
dimensions ask for: the first k distinct ones innermost, one more copy for every
further k (k = number of directly indexable memory dimensions).

Graph: tensors = list of shapes; ops = list of {"kind", "in": [tensor ids],
"out": tensor id, "attr": {...}} in topological order; ILD & Variable operators
carry attr["red"] = reduction axis per operand (None where an operand has none).

READINGS: where the paper leaves a choice, it is written down here as data.
"""
import math
import numpy as np
from . import views as V

ILD_VAR, ILI_VAR, ILD_FIX, ILI_FIX = "ILD_VAR", "ILI_VAR", "ILD_FIX", "ILI_FIX"
GROUPS = (ILD_VAR, ILI_VAR, ILD_FIX, ILI_FIX)          # decreasing "optimization complexity" (Sec. 3.2)
GROUP_OF = {
    "CONV": ILD_VAR, "MATMUL": ILD_VAR, "LAYERNORM": ILD_VAR, "SOFTMAX": ILD_VAR,      # Table 3
    "RESHAPE": ILD_FIX, "TRANSPOSE": ILD_FIX, "DTOS": ILD_FIX, "STOD": ILD_FIX,
    "UNARY": ILI_VAR, "ADD": ILI_VAR, "GATHER": ILI_FIX, "SLICE": ILI_FIX,
    # not listed in the paper; placed by the Table 4 definitions
    "GROUPNORM": ILD_VAR, "RMSNORM": ILD_VAR, "ATTENTION": ILD_VAR, "REDUCE": ILD_VAR,
    "MUL": ILI_VAR, "BIAS": ILI_VAR, "ROPE": ILI_VAR, "ROLL": ILI_FIX, "CONCAT": ILI_FIX,
}
KEEP_BOTH, TRY_FUSE, ELIM_2ND, ELIM_1ST, ELIM_BOTH = "KEEP_BOTH", "TRY_FUSE", "ELIM_2ND", "ELIM_1ST", "ELIM_BOTH"
SEARCH_BOTH, SEARCH_FUSED, SEARCH_1ST, SEARCH_2ND, NO_SEARCH = (
    "SEARCH_BOTH", "SEARCH_FUSED", "SEARCH_1ST", "SEARCH_2ND", "NO_SEARCH")
_V, _F = (ILD_VAR, ILI_VAR), (ILD_FIX, ILI_FIX)
TABLE5 = {(a, b): (KEEP_BOTH if a == b == ILD_VAR else TRY_FUSE) if a in _V and b in _V else
          ELIM_2ND if a in _V else ELIM_1ST if b in _V else ELIM_BOTH for a in GROUPS for b in GROUPS}
TABLE6 = {}
for (_a, _b), _act in TABLE5.items():
    _kept = {KEEP_BOTH: ILD_VAR, TRY_FUSE: min(_a, _b, key=GROUPS.index), ELIM_2ND: _a, ELIM_1ST: _b, ELIM_BOTH: None}[_act]
    _how = {KEEP_BOTH: SEARCH_BOTH, TRY_FUSE: SEARCH_FUSED, ELIM_2ND: SEARCH_1ST, ELIM_1ST: SEARCH_2ND, ELIM_BOTH: NO_SEARCH}[_act]
    TABLE6[(_a, _b)] = (_kept, _how if _kept == ILD_VAR else NO_SEARCH)   # "layout search only happens for pairs involving ILD & Variable"

READINGS = {
    # Table 5 ranks its actions "from low to high" opportunity; a round takes the highest one that applies.
    "action_priority": (ELIM_BOTH, ELIM_2ND, ELIM_1ST, TRY_FUSE),
    # Among pairs with the same action: consumers in graph order, the latest producer of a consumer first.
    "pair_order": "consumer ascending, producer descending",
    # "Eliminate 2nd" rewrites the first operator's store, and one stored tensor has one layout: it needs the
    # Fixed operator to be the only reader of that tensor and to be invertible (a store map is the inverse of
    # the run).  Otherwise Table 5's other cell applies: the run goes into the load of what follows it.
    "store_side_needs": ("sole_consumer", "bijective"),
    # A run that nothing reads (graph output) has no second operator: its Variable producer stores it as well.
    "output_run": "store",
    # Fusion legality is DNNFusion's and is not re-derived; required here: the merged node stays acyclic.
    "fuse_needs": ("no_other_path",),
    # A Fixed operator that never meets a Variable operator is run as a copy.
    "orphan_run": "materialised",
}


def pair_action(first, second):
    return TABLE5[(first, second)]


def pair_outcome(first, second):
    return TABLE6[(first, second)]


def _view_of(op, tensors):
    k, a = op["kind"], op.get("attr", {})
    return {"RESHAPE": lambda: ("reshape", tuple(tensors[op["out"]])), "TRANSPOSE": lambda: ("permute", tuple(a["perm"])),
            "ROLL": lambda: ("roll", a["axis"], a["shift"]),
            "SLICE": lambda: ("slice", a["axis"], a["start"], a["stop"], a.get("step", 1))}.get(k, lambda: ("opaque", k))()


def _inverse(chain, src_shape):
    """The chain that undoes `chain`; None unless every step is a bijection."""
    inv, shape = [], tuple(src_shape)
    for v in chain:
        if v[0] == "reshape":
            inv.insert(0, ("reshape", shape)); shape = tuple(v[1])
        elif v[0] == "permute":
            inv.insert(0, ("permute", tuple(int(i) for i in np.argsort(v[1])))); shape = tuple(shape[p] for p in v[1])
        elif v[0] == "roll":
            inv.insert(0, ("roll", v[1], -v[2]))
        else:
            return None
    return inv


def plan(tensors, ops, k=1):
    n = len(ops)
    group = [GROUP_OF[o["kind"]] for o in ops]
    assert all(len(o["in"]) == 1 for o, g in zip(ops, group) if g in _F), "Fixed operators with several inputs are not planned"
    view = [_view_of(o, tensors) for o in ops]
    alive = set(range(n))                       # operators not eliminated
    node = list(range(n))                       # operator -> the operator its fused node is named after
    ntype = list(group)                         # type of the node named i (Table 6 as nodes merge)
    # per operand: [tensor read now, views pending on the load, the operators those views were]
    ins = [[[t, [], []] for t in o["in"]] for o in ops]
    # per operator: what it stores, as [tensor, views pending on the store, the operators those views were]
    outs = [[[o["out"], [], []]] for o in ops]
    action = [None] * n

    def producer(t):
        return next((i for i in sorted(alive) for e in outs[i] if e[0] == t), None)

    def readers(t):
        return [(c, s) for c in sorted(alive) for s, e in enumerate(ins[c]) if e[0] == t]

    def pairs():                                # (first, second, operand slot) in READINGS["pair_order"]
        ps = [(producer(e[0]), c, s) for c in sorted(alive) for s, e in enumerate(ins[c])]
        return sorted((p for p in ps if p[0] is not None and node[p[0]] != node[p[1]]), key=lambda p: (p[1], -p[0], p[2]))

    def other_path(a, b):                       # can node a reach node b through a third node?
        nxt = lambda x: {node[c] for i in alive if node[i] == x for e in outs[i] for c, _ in readers(e[0])} - {x}
        todo, seen = list(nxt(a) - {b}), set()
        while todo:
            x = todo.pop()
            if x == b:
                return True
            if x not in seen:
                seen.add(x); todo += list(nxt(x))
        return False

    def applies(act, p, c, s):
        if TABLE5[(ntype[node[p]], ntype[node[c]])] != act:
            return False
        if act == ELIM_2ND:
            t = ins[c][0][0]
            held = {"sole_consumer": len(readers(t)) == 1,
                    "bijective": _inverse(ins[c][0][1] + [view[c]], tensors[t]) is not None}
            output_run = READINGS["output_run"] == "store" and not readers(ops[c]["out"])
            return output_run or all(held[r] for r in READINGS["store_side_needs"])
        if act == TRY_FUSE:
            return not other_path(node[p], node[c])
        return True

    def apply(act, p, c, s):
        if act in (ELIM_BOTH, ELIM_1ST):        # the first operator's view moves onto the second's load
            e, f = ins[c][s], ins[p][0]
            ins[c][s] = [f[0], f[1] + [view[p]] + e[1], f[2] + [p] + e[2]]
            if not readers(ops[p]["out"]):
                alive.discard(p)
            for i in ((p, c) if act == ELIM_BOTH else (p,)):
                action[i] = action[i] or act
        elif act == ELIM_2ND:                   # the second operator's view moves onto the first's store
            t, chain, run = ins[c][0]
            e = next(e for e in outs[p] if e[0] == t)
            new = [ops[c]["out"], e[1] + chain + [view[c]], e[2] + run + [c]]
            if len(readers(t)) == 1:
                outs[p][outs[p].index(e)] = new
            else:
                outs[p].append(new)             # an output run beside other readers: one more stored tensor
            alive.discard(c)
            action[c] = action[c] or act
        else:                                   # fuse: the node of lower complexity joins the other (tie: the first stays)
            a, b = node[p], node[c]
            keep, lose = (a, b) if GROUPS.index(ntype[a]) <= GROUPS.index(ntype[b]) else (b, a)
            ntype[keep] = TABLE6[(ntype[a], ntype[b])][0]
            for i in range(n):
                if node[i] == lose:
                    node[i] = keep
                    action[i] = action[i] or TRY_FUSE

    changed = True
    while changed:                              # rounds, until no pair changes
        changed = False
        for act in READINGS["action_priority"]:
            hit = next((q for q in pairs() if applies(act, *q)), None)
            if hit:
                apply(act, *hit)
                changed = True
                break

    # ---- report
    status = [None] * n
    absorbers = [[] for _ in range(n)]
    load_chain, store_chain, stores = {}, {}, {}
    for i in sorted(alive):
        if group[i] in _F:                      # READINGS["orphan_run"]: never met a Variable operator
            for f in ins[i][0][2] + [i]:
                absorbers[f].append(("materialised",))
            continue
        status[i] = ("kept",) if node[i] == i else ("fused", node[i])
        action[i] = action[i] or KEEP_BOTH
        for s, (t, chain, run) in enumerate(ins[i]):
            if run:
                load_chain[(i, s)] = (t, chain, run)
                for f in run:
                    absorbers[f].append(("eliminated", node[i], "load"))
        for t, chain, run in outs[i]:
            if run:
                first = ops[i]["out"]
                entry = (chain, _inverse(chain, tensors[first]), t, run)
                stores.setdefault(node[i], []).append(entry)     # every mapped store of the node
                store_chain.setdefault(node[i], entry)           # the first of them
                for f in run:
                    absorbers[f].append(("eliminated", node[i], "store"))
    for f in range(n):
        if status[f] is None:
            status[f] = absorbers[f][-1]

    # ---- Sec. 3.2.2: reduction-dimension layout selection for every tensor an ILD & Variable operator reads
    wanted = {}
    for c in sorted(alive):
        red = ops[c].get("attr", {}).get("red") or []
        for s, axis in enumerate(red):
            if group[c] != ILD_VAR or axis is None:
                continue
            t, chain, _ = ins[c][s]
            if any(v[0] == "opaque" for v in chain):
                continue                        # read through a Gather: no static index expression, nothing to ask for
            m = V.index_map(tensors[t], chain)
            line = np.moveaxis(m, axis % m.ndim, 0).reshape(m.shape[axis % m.ndim], -1)[:, 0]
            coords = np.array(np.unravel_index(line, tensors[t]))           # stored coordinates along the reduction axis
            moves = (np.diff(coords, axis=1) != 0).sum(axis=1)              # how often each stored dimension changes
            d = int(len(moves) - 1 - np.argmax(moves[::-1])) if moves.any() else len(tensors[t]) - 1
            if d not in wanted.setdefault(t, []):
                wanted[t].append(d)
    layouts = {}
    for t, red_dims in wanted.items():
        inner = red_dims[:k]                    # the first k requested dimensions are made directly indexable
        layouts[t] = {"red_dims": red_dims, "n_copies": max(1, math.ceil(len(red_dims) / k)),
                      "dim_order": [d for d in range(len(tensors[t])) if d not in inner] + inner[::-1]}
    return {"group": group, "status": status, "action": action, "absorbers": absorbers,
            "node_group": [ntype[i] for i in range(n)], "load_chain": load_chain,
            "store_chain": store_chain, "stores": stores, "layouts": layouts}


def surviving(plan_result):
    return [i for i, s in enumerate(plan_result["status"]) if s[0] == "kept"]
