// Layout planner (paper Sec. 3.1 - 3.2): operator classification (Table 3),
// pair actions and outcomes (Tables 5, 6), elimination of Fixed operators into
// the store of the preceding or the load of the following Variable operator,
// fusion of ILI & Variable operators until only ILD & Variable operators are
// left, and reduction-dimension layout selection with k directly indexable
// dimensions (Sec. 3.2.2).  Host only.
//
// The paper rewrites one producer -> consumer pair at a time over rounds; this
// planner reaches the same fixpoint in passes over whole runs: (1) every maximal
// run of Fixed operators behind a stored tensor is collected per reader
// (Fixed-Fixed pairs: "Eliminate both"), (2) each run goes to a store or a load,
// (3) ILI & Variable operators are merged into neighbours with a union-find.
//
// Readings where the paper leaves a choice:
//  - a run goes to the write side (its producer's store, "Eliminate 2nd") when
//    it is the only reader of the producer's tensor and is a bijection (Reshape
//    / Transpose / Roll only): one stored tensor has one layout, and a store
//    map is the inverse of the run ("sub-optimally writing beats sub-optimally
//    reading", Sec. 3.2.2); otherwise each reader's load absorbs its own run
//    ("Eliminate 1st");
//  - a run that nothing reads (a graph output) is stored by its Variable
//    producer as one more output; without such a producer it is materialised;
//  - "Try fuse" pairs are taken with consumers in graph order and a consumer's
//    latest producer first; the node of lower optimisation complexity joins the
//    other (Table 6; on a tie the first operator stays); a merge that would make
//    the node feed itself through a third one is not legal.
#include <algorithm>
#include <map>
#include <memory>
#include <set>
#include <vector>
#include "common.h"
#include "index_map.h"

using namespace sm;

struct sm_plan {
  int k = 1;
  std::vector<std::vector<int64_t>> tensors;
  std::vector<sm_op_desc> ops;
  std::vector<int> group, action, status, absorbed_by, node_group;
  struct Edge { int stored_tensor; sm_map* map; };
  std::map<std::pair<int, int>, Edge> load;     // (consumer op, operand slot)
  std::map<int, Edge> store;                     // producer op
  struct Layout { std::vector<int> dim_order, red_dims; int n_copies; };
  std::map<int, Layout> layouts;
  ~sm_plan() {
    for (auto& e : load) delete e.second.map;
    for (auto& e : store) delete e.second.map;
  }
};

namespace {

bool known_kind(int kind) {
  static const int kinds[] = {SM_OP_CONV, SM_OP_MATMUL, SM_OP_LAYERNORM, SM_OP_SOFTMAX, SM_OP_GROUPNORM, SM_OP_RMSNORM,
                              SM_OP_ATTENTION, SM_OP_REDUCE, SM_OP_RESHAPE, SM_OP_TRANSPOSE, SM_OP_DTOS, SM_OP_STOD,
                              SM_OP_UNARY, SM_OP_ADD, SM_OP_MUL, SM_OP_BIAS, SM_OP_ROPE,
                              SM_OP_GATHER, SM_OP_SLICE, SM_OP_ROLL, SM_OP_CONCAT};
  for (int k : kinds) if (k == kind) return true;
  return false;
}
int group_of(int kind) { return kind < 16 ? SM_ILD_VAR : kind < 32 ? SM_ILD_FIX : kind < 48 ? SM_ILI_VAR : SM_ILI_FIX; }
bool is_var(int g) { return g == SM_ILD_VAR || g == SM_ILI_VAR; }

int action_of(int a, int b) {
  if (is_var(a) && is_var(b)) return (a == SM_ILD_VAR && b == SM_ILD_VAR) ? SM_KEEP_BOTH : SM_TRY_FUSE;
  if (is_var(a)) return SM_ELIM_2ND;
  if (is_var(b)) return SM_ELIM_1ST;
  return SM_ELIM_BOTH;
}
void outcome_of(int a, int b, int* res, int* search) {
  switch (action_of(a, b)) {
    case SM_KEEP_BOTH: *res = SM_ILD_VAR; *search = SM_SEARCH_BOTH; break;
    case SM_TRY_FUSE:
      if (a == SM_ILD_VAR || b == SM_ILD_VAR) { *res = SM_ILD_VAR; *search = SM_SEARCH_FUSED; }
      else { *res = SM_ILI_VAR; *search = SM_NO_SEARCH; }
      break;
    case SM_ELIM_2ND: *res = a; *search = a == SM_ILD_VAR ? SM_SEARCH_1ST : SM_NO_SEARCH; break;
    case SM_ELIM_1ST: *res = b; *search = b == SM_ILD_VAR ? SM_SEARCH_2ND : SM_NO_SEARCH; break;
    default: *res = -1; *search = SM_NO_SEARCH;
  }
}

// view operator of a Fixed op; kind -1 = cannot be composed (Gather, Concat, DtoS, StoD)
sm_view_op view_of(const sm_plan& p, const sm_op_desc& op) {
  sm_view_op v{};
  const std::vector<int64_t>& out = p.tensors[op.out];
  switch (op.kind) {
    case SM_OP_RESHAPE: v.kind = SM_VIEW_RESHAPE; v.n = (int)out.size(); for (size_t i = 0; i < out.size(); ++i) v.arg[i] = out[i]; break;
    case SM_OP_TRANSPOSE: v.kind = SM_VIEW_PERMUTE; v.n = (int)out.size(); for (int i = 0; i < v.n; ++i) v.arg[i] = op.attr[i]; break;
    case SM_OP_ROLL: v.kind = SM_VIEW_ROLL; v.n = 2; v.arg[0] = op.attr[0]; v.arg[1] = op.attr[1]; break;
    case SM_OP_SLICE: v.kind = SM_VIEW_SLICE; v.n = 4; for (int i = 0; i < 4; ++i) v.arg[i] = op.attr[i]; break;
    default: v.kind = -1;
  }
  return v;
}

// chain that undoes `chain` applied to a tensor of shape src; false if not a bijection
bool invert_chain(const std::vector<sm_view_op>& chain, const std::vector<int64_t>& src, std::vector<sm_view_op>* inv) {
  std::vector<std::vector<int64_t>> shapes{src};
  for (auto& v : chain) {
    const std::vector<int64_t>& s = shapes.back();
    if (v.kind == SM_VIEW_RESHAPE) shapes.emplace_back(v.arg, v.arg + v.n);
    else if (v.kind == SM_VIEW_PERMUTE) { std::vector<int64_t> t(v.n); for (int i = 0; i < v.n; ++i) t[i] = s[v.arg[i]]; shapes.push_back(t); }
    else if (v.kind == SM_VIEW_ROLL) shapes.push_back(s);
    else return false;
  }
  inv->clear();
  for (int i = (int)chain.size() - 1; i >= 0; --i) {
    const sm_view_op& v = chain[i];
    const std::vector<int64_t>& before = shapes[i];
    sm_view_op w{};
    if (v.kind == SM_VIEW_RESHAPE) { w.kind = SM_VIEW_RESHAPE; w.n = (int)before.size(); for (int j = 0; j < w.n; ++j) w.arg[j] = before[j]; }
    else if (v.kind == SM_VIEW_PERMUTE) { w.kind = SM_VIEW_PERMUTE; w.n = v.n; for (int j = 0; j < v.n; ++j) w.arg[v.arg[j]] = j; }
    else { w.kind = SM_VIEW_ROLL; w.n = 2; w.arg[0] = v.arg[0]; w.arg[1] = -v.arg[1]; }
    inv->push_back(w);
  }
  return true;
}

struct Run { int src; std::vector<sm_view_op> chain; std::vector<int> ops; bool composable; };

}  // namespace

extern "C" int sm_op_group(int kind, int* group) {
  if (!group || !known_kind(kind)) return fail(SM_ERR_INVALID_ARG, "sm_op_group: unknown operator kind %d", kind);
  *group = group_of(kind);
  return SM_OK;
}
extern "C" int sm_pair_action(int a, int b, int* action) {
  if (!action || a < 0 || a > 3 || b < 0 || b > 3) return fail(SM_ERR_INVALID_ARG, "sm_pair_action: bad argument");
  *action = action_of(a, b);
  return SM_OK;
}
extern "C" int sm_pair_outcome(int a, int b, int* res, int* search) {
  if (!res || !search || a < 0 || a > 3 || b < 0 || b > 3) return fail(SM_ERR_INVALID_ARG, "sm_pair_outcome: bad argument");
  outcome_of(a, b, res, search);
  return SM_OK;
}

extern "C" int sm_layout_plan(const sm_tensor_desc* tensors, int n_tensors, const sm_op_desc* ops, int n_ops, int k, sm_plan** out) {
  if (!tensors || !ops || !out || n_tensors < 1 || n_ops < 1) return fail(SM_ERR_INVALID_ARG, "sm_layout_plan: null or empty graph");
  if (k < 1) return fail(SM_ERR_INVALID_ARG, "sm_layout_plan: k must be >= 1");
  std::unique_ptr<sm_plan> p(new sm_plan());
  p->k = k;
  for (int t = 0; t < n_tensors; ++t) {
    if (tensors[t].rank < 1 || tensors[t].rank > SM_MAX_RANK) return fail(SM_ERR_INVALID_ARG, "sm_layout_plan: tensor %d has rank %d", t, tensors[t].rank);
    p->tensors.emplace_back(tensors[t].shape, tensors[t].shape + tensors[t].rank);
    for (auto s : p->tensors.back()) if (s < 1) return fail(SM_ERR_SHAPE, "sm_layout_plan: tensor %d has an extent < 1", t);
  }
  const int n = n_ops;
  p->ops.assign(ops, ops + n);
  std::map<int, int> producer;
  std::map<int, std::vector<std::pair<int, int>>> consumers;
  for (int i = 0; i < n; ++i) {
    const sm_op_desc& o = ops[i];
    if (!known_kind(o.kind)) return fail(SM_ERR_INVALID_ARG, "sm_layout_plan: operator %d has unknown kind %d", i, o.kind);
    if (o.n_in < 1 || o.n_in > 4 || o.out < 0 || o.out >= n_tensors) return fail(SM_ERR_INVALID_ARG, "sm_layout_plan: operator %d is malformed", i);
    if (!is_var(group_of(o.kind)) && o.n_in != 1) return fail(SM_ERR_UNSUPPORTED, "sm_layout_plan: operator %d: layout operators with several inputs are not planned", i);
    for (int s = 0; s < o.n_in; ++s) {
      if (o.in[s] < 0 || o.in[s] >= n_tensors) return fail(SM_ERR_INVALID_ARG, "sm_layout_plan: operator %d reads tensor %d", i, o.in[s]);
      if (producer.count(o.in[s]) && producer[o.in[s]] >= i) return fail(SM_ERR_INVALID_ARG, "sm_layout_plan: operators are not in topological order");
      consumers[o.in[s]].push_back({i, s});
    }
    if (producer.count(o.out)) return fail(SM_ERR_INVALID_ARG, "sm_layout_plan: tensor %d is produced twice", o.out);
    for (auto& c : consumers[o.out]) if (c.first <= i) return fail(SM_ERR_INVALID_ARG, "sm_layout_plan: operators are not in topological order");
    producer[o.out] = i;
  }
  p->group.resize(n); p->action.assign(n, -1); p->status.assign(n, SM_KEPT); p->absorbed_by.resize(n); p->node_group.resize(n);
  for (int i = 0; i < n; ++i) { p->group[i] = p->node_group[i] = group_of(ops[i].kind); p->absorbed_by[i] = i; }
  auto fixed_op = [&](int t) { return producer.count(t) && !is_var(p->group[producer[t]]); };

  // ---- Fixed-Fixed pairs ("Eliminate both"): a run of Fixed operators is one pending view chain
  auto run_back = [&](int t) {
    Run r; r.composable = true;
    while (fixed_op(t)) {
      const int i = producer[t];
      sm_view_op v = view_of(*p, ops[i]);
      if (v.kind < 0) r.composable = false;
      r.chain.insert(r.chain.begin(), v);
      r.ops.insert(r.ops.begin(), i);
      t = ops[i].in[0];
    }
    r.src = t;
    return r;
  };
  for (int i = 0; i < n; ++i) {
    if (is_var(p->group[i])) continue;
    bool next_fixed = false;
    for (auto& c : consumers[ops[i].out]) next_fixed |= !is_var(p->group[c.first]);
    if (fixed_op(ops[i].in[0]) || next_fixed) p->action[i] = SM_ELIM_BOTH;
  }
  struct Use { int consumer, slot; Run run; };
  std::map<int, std::vector<Use>> by_src;       // stored tensor -> the runs hanging off it
  for (int i = 0; i < n; ++i) {
    if (!is_var(p->group[i])) {
      if (consumers[ops[i].out].empty()) {       // graph output reached through a run
        Run r = run_back(ops[i].out);
        by_src[r.src].push_back({-1, -1, r});
      }
      continue;
    }
    for (int s = 0; s < ops[i].n_in; ++s) {
      Run r = run_back(ops[i].in[s]);
      if (!r.ops.empty()) by_src[r.src].push_back({i, s, r});
    }
  }

  // ---- absorb every run into a Variable neighbour
  std::map<int, std::vector<sm_view_op>> load_chain_of;   // key consumer*8+slot
  std::map<int, int> load_src;
  struct Store { int prod, final_t; std::vector<sm_view_op> chain; bool composable; };
  std::vector<Store> main_store, extra_store;              // a producer's own store / further outputs behind a run
  auto to_store = [&](const Use& u, int prod) {
    for (int f : u.run.ops) {
      p->status[f] = SM_ELIMINATED_STORE; p->absorbed_by[f] = prod;
      if (p->action[f] < 0) p->action[f] = SM_ELIM_2ND;
    }
  };
  for (auto& kv : by_src) {
    const int src = kv.first;
    const bool has_prod = producer.count(src) > 0;
    std::vector<Use> uses;                                  // the runs something reads
    for (auto& u : kv.second) {
      if (u.consumer >= 0) { uses.push_back(u); continue; }
      if (has_prod) {                                       // a run nothing reads: its producer stores it as well
        to_store(u, producer[src]);
        extra_store.push_back({producer[src], ops[u.run.ops.back()].out, u.run.chain, u.run.composable});
      } else {
        for (int f : u.run.ops) { p->status[f] = SM_MATERIALISED; p->absorbed_by[f] = -1; }
      }
    }
    if (uses.empty()) continue;
    bool direct = false;                                    // somebody reads the stored tensor as it is
    for (auto& c : consumers[src]) direct |= is_var(p->group[c.first]);
    bool one_run = true, composable = true;                 // one stored tensor has one layout
    for (auto& u : uses) { one_run &= u.run.ops == uses[0].run.ops; composable &= u.run.composable; }
    std::vector<sm_view_op> inv;
    if (has_prod && !direct && one_run && composable && invert_chain(uses[0].run.chain, p->tensors[src], &inv)) {
      to_store(uses[0], producer[src]);
      main_store.push_back({producer[src], ops[uses[0].run.ops.back()].out, uses[0].run.chain, true});
    } else {
      for (auto& u : uses) {
        for (int f : u.run.ops) {
          p->status[f] = SM_ELIMINATED_LOAD; p->absorbed_by[f] = u.consumer;
          if (p->action[f] < 0) p->action[f] = SM_ELIM_1ST;
        }
        load_src[u.consumer * 8 + u.slot] = src;
        if (u.run.composable) load_chain_of[u.consumer * 8 + u.slot] = u.run.chain;
      }
    }
  }

  // ---- "Try fuse": pair by pair (consumers in graph order, a consumer's latest producer first), the node of
  // lower optimisation complexity joins the other (Table 6), as long as the merged node does not feed itself
  std::vector<int> root(n);
  for (int i = 0; i < n; ++i) root[i] = i;
  auto find = [&](int i) { while (root[i] != i) i = root[i]; return i; };
  auto stored_source = [&](int t) { return fixed_op(t) ? run_back(t).src : t; };
  auto feeds_through_third = [&](int a, int b) {          // a path a ~> b that does not use an a -> b edge
    std::vector<int> todo; std::set<int> seen;
    auto push_next = [&](int x, bool skip_b) {
      for (int c = 0; c < n; ++c) {
        if (!is_var(p->group[c]) || find(c) == x) continue;
        for (int s2 = 0; s2 < ops[c].n_in; ++s2) {
          const int t = stored_source(ops[c].in[s2]);
          if (producer.count(t) && is_var(p->group[producer[t]]) && find(producer[t]) == x && !(skip_b && find(c) == b)) todo.push_back(find(c));
        }
      }
    };
    push_next(a, true);
    while (!todo.empty()) {
      const int x = todo.back(); todo.pop_back();
      if (x == b) return true;
      if (seen.insert(x).second) push_next(x, false);
    }
    return false;
  };
  for (bool changed = true; changed;) {
    changed = false;
    for (int c = 0; c < n && !changed; ++c) {
      if (!is_var(p->group[c])) continue;
      std::vector<int> prods;
      for (int s2 = 0; s2 < ops[c].n_in; ++s2) {
        const int t = stored_source(ops[c].in[s2]);
        if (producer.count(t) && is_var(p->group[producer[t]])) prods.push_back(producer[t]);
      }
      std::sort(prods.rbegin(), prods.rend());
      for (int q : prods) {
        const int a = find(q), b = find(c);
        if (a == b || action_of(p->node_group[a], p->node_group[b]) != SM_TRY_FUSE || feeds_through_third(a, b)) continue;
        const int keep = p->node_group[a] <= p->node_group[b] ? a : b, lose = keep == a ? b : a;
        int res, search;
        outcome_of(p->node_group[a], p->node_group[b], &res, &search);
        p->node_group[keep] = res;
        root[lose] = keep;
        changed = true;
        break;
      }
    }
  }
  for (int i = 0; i < n; ++i) {
    if (is_var(p->group[i])) {
      const int r = find(i);
      p->status[i] = r == i ? SM_KEPT : SM_FUSED;
      p->absorbed_by[i] = r;
      p->action[i] = r == i ? SM_KEEP_BOTH : SM_TRY_FUSE;
    } else if (p->status[i] == SM_ELIMINATED_STORE || p->status[i] == SM_ELIMINATED_LOAD) {
      p->absorbed_by[i] = find(p->absorbed_by[i]);
    }
  }

  // ---- compose the maps
  std::string err;
  for (auto& kv : load_src) {
    sm_map* m = nullptr;
    auto ch = load_chain_of.find(kv.first);
    if (ch != load_chain_of.end() &&
        map_create(p->tensors[kv.second], ch->second.data(), (int)ch->second.size(), &m, &err) != SM_OK)
      return fail(SM_ERR_SHAPE, "sm_layout_plan: load map of operator %d: %s", kv.first / 8, err.c_str());
    p->load[{kv.first / 8, kv.first % 8}] = {kv.second, m};
  }
  std::set<int> stored_final;
  main_store.insert(main_store.end(), extra_store.begin(), extra_store.end());
  std::stable_sort(main_store.begin(), main_store.end(), [](const Store& x, const Store& y) { return x.prod < y.prod; });
  for (auto& st : main_store) {
    stored_final.insert(st.final_t);
    if (p->store.count(find(st.prod))) continue;           // sm_plan_store_map reports a node's first mapped store
    std::vector<sm_view_op> inv;
    sm_map* m = nullptr;
    if (st.composable && invert_chain(st.chain, p->tensors[ops[st.prod].out], &inv) &&
        map_create(p->tensors[st.final_t], inv.data(), (int)inv.size(), &m, &err) != SM_OK)
      return fail(SM_ERR_SHAPE, "sm_layout_plan: store map of operator %d: %s", st.prod, err.c_str());
    p->store[find(st.prod)] = {st.final_t, m};
  }

  // ---- reduction-dimension layout selection (local rule per edge, global rule per tensor)
  for (int t = 0; t < n_tensors; ++t) {
    if (producer.count(t) && (p->status[producer[t]] == SM_ELIMINATED_STORE || p->status[producer[t]] == SM_ELIMINATED_LOAD) &&
        !stored_final.count(t)) continue;                 // a view that is never stored
    const std::vector<int64_t>& shape = p->tensors[t];
    const int rank = (int)shape.size();
    std::vector<int64_t> nat(rank, 1);
    for (int d = rank - 2; d >= 0; --d) nat[d] = nat[d + 1] * shape[d + 1];
    sm_plan::Layout lay;                                    // requested dimensions in consumer order
    auto request = [&](const sm_map* m, const std::vector<int64_t>& vshape, int64_t red) {
      const int vr = (int)vshape.size();
      if (red < 0) red += vr;
      if (red < 0 || red >= vr) return;
      // the stored dimension that moves most often while walking along the reduction axis (the innermost of
      // them on a tie: a reduction over merged dimensions asks for the fastest one); extent 1 asks for nothing
      int dim = rank - 1;
      std::vector<int64_t> moves(rank, 0), idx(vr, 0);
      int64_t prev = 0;
      for (int64_t i = 0; i < vshape[red]; ++i) {
        idx[red] = i;
        int64_t off = 0;
        if (m) off = m->at(idx.data());
        else for (int d = 0; d < vr; ++d) off = off * vshape[d] + idx[d];
        if (i > 0) for (int d = 0; d < rank; ++d) moves[d] += (off / nat[d]) % shape[d] != (prev / nat[d]) % shape[d];
        prev = off;
      }
      for (int d = 0; d < rank; ++d) if (moves[d] > 0 && moves[d] >= moves[dim]) dim = d;
      if (std::find(lay.red_dims.begin(), lay.red_dims.end(), dim) == lay.red_dims.end()) lay.red_dims.push_back(dim);
    };
    for (int c = 0; c < n; ++c) {
      if (p->group[c] != SM_ILD_VAR) continue;
      for (int s = 0; s < ops[c].n_in; ++s) {
        const int64_t red = s < ops[c].n_attr ? ops[c].attr[s] : -1;
        auto it = p->load.find({c, s});
        if (it != p->load.end()) {
          if (it->second.map && it->second.stored_tensor == t && red >= 0) request(it->second.map, it->second.map->shape, red);
        } else if (ops[c].in[s] == t && red >= 0) {
          request(nullptr, shape, red);
        }
      }
    }
    if (lay.red_dims.empty()) continue;
    lay.n_copies = std::max(1, ((int)lay.red_dims.size() + k - 1) / k);
    std::vector<int> inner(lay.red_dims.begin(), lay.red_dims.begin() + std::min<size_t>(k, lay.red_dims.size()));
    for (int d = 0; d < rank; ++d) if (std::find(inner.begin(), inner.end(), d) == inner.end()) lay.dim_order.push_back(d);
    for (int i = (int)inner.size() - 1; i >= 0; --i) lay.dim_order.push_back(inner[i]);
    p->layouts[t] = lay;
  }
  *out = p.release();
  return SM_OK;
}

extern "C" int sm_plan_op(const sm_plan* p, int op, int* group, int* action, int* status, int* absorbed_by, int* node_group) {
  if (!p || op < 0 || op >= (int)p->ops.size()) return fail(SM_ERR_INVALID_ARG, "sm_plan_op: bad plan or operator index");
  if (group) *group = p->group[op];
  if (action) *action = p->action[op];
  if (status) *status = p->status[op];
  if (absorbed_by) *absorbed_by = p->absorbed_by[op];
  if (node_group) *node_group = p->node_group[op];
  return SM_OK;
}

extern "C" int sm_plan_tensor(const sm_plan* p, int tensor, int* dim_order, int* red_dims, int* n_red, int* n_copies) {
  if (!p || tensor < 0 || tensor >= (int)p->tensors.size()) return fail(SM_ERR_INVALID_ARG, "sm_plan_tensor: bad plan or tensor index");
  auto it = p->layouts.find(tensor);
  if (it == p->layouts.end()) return fail(SM_ERR_INVALID_ARG, "sm_plan_tensor: tensor %d has no layout-sensitive consumer or is never stored", tensor);
  if (dim_order) for (size_t i = 0; i < it->second.dim_order.size(); ++i) dim_order[i] = it->second.dim_order[i];
  if (red_dims) for (size_t i = 0; i < it->second.red_dims.size(); ++i) red_dims[i] = it->second.red_dims[i];
  if (n_red) *n_red = (int)it->second.red_dims.size();
  if (n_copies) *n_copies = it->second.n_copies;
  return SM_OK;
}

extern "C" int sm_plan_load_map(const sm_plan* p, int consumer_op, int operand, const sm_map** borrowed, int* stored_tensor) {
  if (!p || !borrowed || consumer_op < 0 || consumer_op >= (int)p->ops.size() || operand < 0 || operand >= p->ops[consumer_op].n_in)
    return fail(SM_ERR_INVALID_ARG, "sm_plan_load_map: bad argument");
  auto it = p->load.find({consumer_op, operand});
  *borrowed = it == p->load.end() ? nullptr : it->second.map;
  if (stored_tensor) *stored_tensor = it == p->load.end() ? p->ops[consumer_op].in[operand] : it->second.stored_tensor;
  return SM_OK;
}

extern "C" int sm_plan_store_map(const sm_plan* p, int producer_op, const sm_map** borrowed, int* stored_tensor) {
  if (!p || !borrowed || producer_op < 0 || producer_op >= (int)p->ops.size()) return fail(SM_ERR_INVALID_ARG, "sm_plan_store_map: bad argument");
  auto it = p->store.find(producer_op);
  *borrowed = it == p->store.end() ? nullptr : it->second.map;
  if (stored_tensor) *stored_tensor = it == p->store.end() ? p->ops[producer_op].out : it->second.stored_tensor;
  return SM_OK;
}

extern "C" void sm_plan_destroy(sm_plan* p) { delete p; }
