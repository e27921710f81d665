"""Layout planner: operator classification (Table 3), pairwise action and
outcome tables (Tables 5, 6), elimination / fusion to a fixpoint (Sec. 3.2,
"all preserved operators are ILD & Variable"), and reduction-dimension layout
selection (Sec. 3.2.2, local rule + global rule with k directly indexable
dimensions, redundant copies beyond k).

Graph: tensors = list of shapes; ops = list of dicts
    {"kind": str, "in": [tensor ids], "out": tensor id, "attr": {...}}
in topological order.  ILD & Variable ops carry attr["red"] = list with the
reduction axis of each operand (None where an operand has none).

Readings where the paper is silent:
  * Operators the paper does not list are classified by the Table 4
    definitions (see GROUP_OF).
  * A run of Fixed operators between two Variable operators can be absorbed
    by either side (Table 5 offers both "Eliminate 2nd" and "Eliminate 1st").
    Write side (the producer's store) is taken when every consumer of the
    producer's tensor sees it through the same run and the run is a bijection
    (no Slice / Gather); otherwise each consumer's load absorbs its own run.
    This follows "sub-optimally writing beats sub-optimally reading".
  * A Fixed run with no Variable operator on either side is materialised.
  * k = 1 on linear memory; copies = ceil(distinct requested dims / k).
"""
import math

ILD_VAR, ILI_VAR, ILD_FIX, ILI_FIX = "ILD_VAR", "ILI_VAR", "ILD_FIX", "ILI_FIX"
GROUPS = (ILD_VAR, ILI_VAR, ILD_FIX, ILI_FIX)

GROUP_OF = {
    # Table 3
    "CONV": ILD_VAR, "MATMUL": ILD_VAR, "LAYERNORM": ILD_VAR, "SOFTMAX": ILD_VAR,
    "RESHAPE": ILD_FIX, "TRANSPOSE": ILD_FIX, "DTOS": ILD_FIX, "STOD": ILD_FIX,
    "UNARY": ILI_VAR, "ADD": ILI_VAR,
    "GATHER": ILI_FIX, "SLICE": ILI_FIX,
    # classified by the Table 4 definitions (not listed in the paper)
    "GROUPNORM": ILD_VAR, "RMSNORM": ILD_VAR, "ATTENTION": ILD_VAR, "REDUCE": ILD_VAR,
    "MUL": ILI_VAR, "BIAS": ILI_VAR, "ROPE": ILI_VAR,
    "ROLL": ILI_FIX, "CONCAT": ILI_FIX,
}

KEEP_BOTH, TRY_FUSE, ELIM_2ND, ELIM_1ST, ELIM_BOTH = (
    "KEEP_BOTH", "TRY_FUSE", "ELIM_2ND", "ELIM_1ST", "ELIM_BOTH")
SEARCH_BOTH, SEARCH_FUSED, SEARCH_1ST, SEARCH_2ND, NO_SEARCH = (
    "SEARCH_BOTH", "SEARCH_FUSED", "SEARCH_1ST", "SEARCH_2ND", "NO_SEARCH")


def _is_var(g):
    return g in (ILD_VAR, ILI_VAR)


def pair_action(first, second):
    """Table 5."""
    if _is_var(first) and _is_var(second):
        return KEEP_BOTH if (first == ILD_VAR and second == ILD_VAR) else TRY_FUSE
    if _is_var(first):
        return ELIM_2ND
    if _is_var(second):
        return ELIM_1ST
    return ELIM_BOTH


def pair_outcome(first, second):
    """Table 6: (resulting group or None for N/A, layout search policy)."""
    a = pair_action(first, second)
    if a == KEEP_BOTH:
        return ILD_VAR, SEARCH_BOTH
    if a == TRY_FUSE:
        if ILD_VAR in (first, second):
            return ILD_VAR, SEARCH_FUSED
        return ILI_VAR, NO_SEARCH
    if a == ELIM_2ND:                     # the first operator is preserved
        return first, (SEARCH_1ST if first == ILD_VAR else NO_SEARCH)
    if a == ELIM_1ST:                     # the second operator is preserved
        return second, (SEARCH_2ND if second == ILD_VAR else NO_SEARCH)
    return None, NO_SEARCH


def _view_of(op, tensors):
    k = op["kind"]
    a = op.get("attr", {})
    if k == "RESHAPE":
        return ("reshape", tuple(tensors[op["out"]]))
    if k == "TRANSPOSE":
        return ("permute", tuple(a["perm"]))
    if k == "ROLL":
        return ("roll", a["axis"], a["shift"])
    if k == "SLICE":
        return ("slice", a["axis"], a["start"], a["stop"], a.get("step", 1))
    return ("opaque", k)


def _invert_chain(chain, src_shape):
    """Chain that undoes `chain` (which starts from src_shape); None if not a bijection."""
    shapes = [tuple(src_shape)]
    for v in chain:
        s = shapes[-1]
        if v[0] == "reshape":
            shapes.append(tuple(v[1]))
        elif v[0] == "permute":
            shapes.append(tuple(s[p] for p in v[1]))
        elif v[0] == "roll":
            shapes.append(s)
        else:
            return None
    inv = []
    for v, s_before in zip(reversed(chain), reversed(shapes[:-1])):
        if v[0] == "reshape":
            inv.append(("reshape", s_before))
        elif v[0] == "permute":
            p = v[1]
            ip = [0] * len(p)
            for k_, pk in enumerate(p):
                ip[pk] = k_
            inv.append(("permute", tuple(ip)))
        else:
            inv.append(("roll", v[1], -v[2]))
    return inv


def plan(tensors, ops, k=1):
    n = len(ops)
    group = [GROUP_OF[o["kind"]] for o in ops]
    producer = {o["out"]: i for i, o in enumerate(ops)}
    consumers = {}
    for i, o in enumerate(ops):
        for slot, t in enumerate(o["in"]):
            consumers.setdefault(t, []).append((i, slot))

    status = [("kept",)] * n
    action = [None] * n
    node_group = list(group)

    # ---- step 1: Fixed-Fixed pairs ("Eliminate both"): runs of Fixed ops
    # collapse into one pending view chain per consumer edge.
    def run_back(t):
        """Walk from tensor t back through Fixed ops; (stored tensor, chain, ops in run)."""
        chain, run = [], []
        while t in producer and not _is_var(group[producer[t]]):
            i = producer[t]
            chain.insert(0, _view_of(ops[i], tensors))
            run.insert(0, i)
            t = ops[i]["in"][0]
        return t, chain, run

    load_chain = {}     # (consumer op, slot) -> (stored tensor, chain, run)
    for i, o in enumerate(ops):
        if not _is_var(group[i]):
            continue
        for slot, t in enumerate(o["in"]):
            src, chain, run = run_back(t)
            if run:
                load_chain[(i, slot)] = (src, chain, run)
    out_runs = {}       # graph outputs reached through a Fixed run
    for i, o in enumerate(ops):
        if not _is_var(group[i]) and o["out"] not in consumers:
            src, chain, run = run_back(o["out"])
            out_runs[o["out"]] = (src, chain, run)
    for i in range(n):
        if _is_var(group[i]):
            continue
        t_in = ops[i]["in"][0]
        prev_fixed = t_in in producer and not _is_var(group[producer[t_in]])
        next_fixed = any(not _is_var(group[c]) for c, _ in consumers.get(ops[i]["out"], []))
        if prev_fixed or next_fixed:
            action[i] = ELIM_BOTH

    # ---- step 2: absorb each run into a Variable neighbour.
    store_chain = {}    # producer op -> (chain, inverse chain, final tensor id, run)
    by_src = {}
    for key, (src, chain, run) in load_chain.items():
        by_src.setdefault(src, []).append((key, chain, run))
    for t_out, (src, chain, run) in out_runs.items():
        by_src.setdefault(src, []).append((None, chain, run))
    for src, uses in by_src.items():
        direct = [c for c in consumers.get(src, []) if _is_var(group[c[0]])]
        chains = {tuple(ch) for _, ch, _ in uses}
        inv = _invert_chain(uses[0][1], tensors[src]) if src in producer else None
        write_side = (src in producer and not direct and len(chains) == 1 and inv is not None)
        if write_side:
            p = producer[src]
            final_t = ops[uses[0][2][-1]]["out"]
            store_chain[p] = (uses[0][1], inv, final_t, uses[0][2])
            for key, _, run in uses:
                for f in run:
                    status[f] = ("eliminated", p, "store")
                    action[f] = action[f] or ELIM_2ND
                if key is not None:
                    del load_chain[key]
        else:
            for key, _, run in uses:
                if key is None:
                    for f in run:
                        if src in producer:      # Variable producer, non-bijective run
                            status[f] = ("eliminated", producer[src], "store")
                            action[f] = action[f] or ELIM_2ND
                        else:
                            status[f] = ("materialised",)
                    continue
                for f in run:
                    status[f] = ("eliminated", key[0], "load")
                    action[f] = action[f] or ELIM_1ST

    # ---- step 3: fuse ILI & Variable ops into a neighbour until none is left
    # next to a Variable op ("Try fuse"); the merged node takes the Table 6 type.
    root = list(range(n))

    def find(i):
        while root[i] != i:
            i = root[i]
        return i

    def var_producers(i):
        res = []
        for slot, t in enumerate(ops[i]["in"]):
            if (i, slot) in load_chain:
                t = load_chain[(i, slot)][0]
            elif t in producer and not _is_var(group[producer[t]]):
                # reached through a run absorbed on the write side
                t = run_back(t)[0]
            if t in producer:
                res.append(find(producer[t]))
        return res

    changed = True
    while changed:
        changed = False
        for i in range(n):
            if group[i] != ILI_VAR or status[i][0] != "kept":
                continue
            prods = [q for q in var_producers(i) if q != i]
            if prods:
                tgt = max(prods)                     # the latest producer: epilogue fusion
            else:
                cons = [find(c) for c, _ in consumers.get(ops[i]["out"], []) if _is_var(group[c])]
                cons = [q for q in cons if q != i]
                if not cons:
                    continue
                tgt = min(cons)                      # prologue fusion
            res, _ = pair_outcome(node_group[tgt], ILI_VAR)
            status[i] = ("fused", tgt)
            action[i] = TRY_FUSE
            node_group[tgt] = res
            root[i] = tgt
            changed = True

    for i in range(n):
        if status[i][0] == "kept" and action[i] is None:
            action[i] = KEEP_BOTH                     # a preserved operator is reported as kept
        if status[i][0] == "eliminated":              # absorbed by the merged node's root
            status[i] = ("eliminated", find(status[i][1]), status[i][2])
    store_chain = {find(p_): v for p_, v in store_chain.items()}

    # ---- step 4: reduction-dimension layout selection for every stored tensor.
    from . import views as V
    import numpy as np
    layouts = {}
    for t, shape in enumerate(tensors):
        uses = []
        if t in producer and status[producer[t]][0] == "eliminated" and \
                t not in [sc[2] for sc in store_chain.values()]:
            continue                                  # a view that is never stored
        for (c, slot) in consumers.get(t, []):
            if group[c] != ILD_VAR or (c, slot) in load_chain:
                continue
            red = ops[c].get("attr", {}).get("red", [None] * len(ops[c]["in"]))[slot]
            if red is not None:
                uses.append((c, slot, [], red))
        for (c, slot), (src, chain, run) in load_chain.items():
            if src == t and group[c] == ILD_VAR:
                red = ops[c].get("attr", {}).get("red", [None] * len(ops[c]["in"]))[slot]
                if red is not None:
                    uses.append((c, slot, chain, red))
        if not uses:
            continue
        requested = []           # (stride in t's natural storage, extent), in consumer order
        for c, slot, chain, red in sorted(uses, key=lambda u: (u[0], u[1])):
            m = V.index_map(shape, chain)
            red = red % m.ndim
            ext = m.shape[red]
            if ext > 1:
                a = np.take(m, 0, axis=red).reshape(-1)[0]
                b = np.take(m, 1, axis=red).reshape(-1)[0]
                stride = int(b - a)
            else:
                stride = 1
            if (stride, ext) not in requested:
                requested.append((stride, ext))
        nat = [int(np.prod(shape[d + 1:])) for d in range(len(shape))]

        def dim_of(stride):
            for d in range(len(shape)):
                if nat[d] <= stride < nat[d] * shape[d]:
                    return d
            return len(shape) - 1
        red_dims = []
        for stride, _ in requested:
            d = dim_of(stride)
            if d not in red_dims:
                red_dims.append(d)
        n_copies = max(1, math.ceil(len(red_dims) / k))
        inner = red_dims[:k]
        order = [d for d in range(len(shape)) if d not in inner] + list(reversed(inner))
        layouts[t] = {"requested": requested, "red_dims": red_dims,
                      "dim_order": order, "n_copies": n_copies}

    return {"group": group, "status": status, "action": action,
            "node_group": node_group, "load_chain": load_chain,
            "store_chain": store_chain, "layouts": layouts}


def surviving(plan_result):
    return [i for i, s in enumerate(plan_result["status"]) if s[0] == "kept"]
