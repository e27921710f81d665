// sm_fanout_graph: the multi-consumer example of the paper's global layout selection (Sec. 3.2.2, Fig. 4) executed
// end to end: MatMul -> Transpose -> Reshape -> {Reduce over D3, Reduce' over D1, Conv over D3}.
//
// The executor writes the graph down, asks sm_layout_plan (with the caller's k, the number of directly indexable
// memory dimensions) and does what the plan says: Transpose and Reshape are eliminated into the MatMul's store; the
// consumers ask for two reduction dimensions (D3 and D1), so with k = 1 (linear memory) the MatMul keeps TWO copies of
// its result, one per requested dimension, each consumer reading the copy whose innermost dimension is its reduction
// dimension; with k = 2 (the paper's 2.5D case) one layout has to serve both, and on linear memory the consumer whose
// dimension is not innermost reads with a stride.  SM_EXPLICIT materialises the Transpose as a copy kernel.
// The memory cost of the redundant copy (Sec. 4.6) is reported by sm_fanout_graph_plan.
#include <cstring>
#include <memory>
#include "common.h"
#include "copy_plan.h"
#include "graph_build.h"
#include "index_map.h"
#include "kernels.h"
#include "plan_chains.h"

using namespace sm;

namespace {

int check_cfg(const sm_fanout_cfg* c, const char* who) {
  if (!c) return fail(SM_ERR_INVALID_ARG, "%s: null configuration", who);
  if (!dtype_ok(c->dtype)) return fail(SM_ERR_INVALID_ARG, "%s: unknown dtype", who);
  if (c->D1 < 1 || c->D2 < 1 || c->D3 < 1 || c->Kin < 1 || c->Cout < 1) return fail(SM_ERR_SHAPE, "%s: non-positive dimension", who);
  const int vec = c->dtype == SM_F32 ? 4 : 8;
  if (c->Kin % vec || c->D3 % vec || c->D1 % vec) return fail(SM_ERR_SHAPE, "%s: Kin, D1 and D3 must be multiples of %d", who, vec);
  if (c->k != 1 && c->k != 2) return fail(SM_ERR_INVALID_ARG, "%s: k must be 1 or 2", who);
  if ((int64_t)c->D1 * c->D2 * c->D3 > INT32_MAX) return fail(SM_ERR_SHAPE, "%s: tensor too large", who);
  return SM_OK;
}

struct FanoutPlan { int n_copies; bool transposed_store; int red_dims[2]; int n_red; Copy transpose; TableRegion tables; };

// plans the graph; the executor refuses anything but the outcome of the paper's example
int make_plan(const sm_fanout_cfg* c, FanoutPlan* p, const char* who) {
  const int64_t D1 = c->D1, D2 = c->D2, D3 = c->D3, D0 = D2 * D3;
  GraphB g;
  const int a = g.tensor({D0, (int64_t)c->Kin});
  int t = g.op(SM_OP_MATMUL, {a}, {D0, D1}, "matmul", {1});
  t = g.transpose(t, {1, 0});
  t = g.reshape(t, {D1, D2, D3});
  g.op(SM_OP_REDUCE, {t}, {D1, D2}, "reduce", {2});
  g.op(SM_OP_REDUCE, {t}, {D2, D3}, "reduce_p", {0});
  g.op(SM_OP_CONV, {t}, {D1, D2, (int64_t)c->Cout}, "conv", {2});
  sm_plan* plan = nullptr;
  if (sm_layout_plan(g.tensors.data(), (int)g.tensors.size(), g.ops.data(), (int)g.ops.size(), c->k, &plan) != SM_OK) return SM_ERR_UNSUPPORTED;
  std::unique_ptr<sm_plan, void (*)(sm_plan*)> guard(plan, sm_plan_destroy);
  const sm_map* m = nullptr;
  int stored = -1;
  sm_plan_store_map(plan, g.find("matmul"), &m, &stored);
  p->transposed_store = m != nullptr;
  int order[SM_MAX_RANK], red[SM_MAX_RANK], n_red = 0, n_copies = 0;
  if (!m || sm_plan_tensor(plan, stored, order, red, &n_red, &n_copies) != SM_OK || n_red != 2)
    return fail(SM_ERR_UNSUPPORTED, "%s: the planner did not eliminate the layout operators into the MatMul's store", who);
  p->n_copies = n_copies; p->n_red = n_red; p->red_dims[0] = red[0]; p->red_dims[1] = red[1];
  std::string err;
  if (!make_copy({D0, D1}, {chains::permute({1, 0})}, (int)dtype_size(c->dtype), &p->tables, &p->transpose, &err))
    return fail(SM_ERR_UNSUPPORTED, "%s: %s", who, err.c_str());
  return SM_OK;
}

size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

}  // namespace

extern "C" int sm_fanout_graph_plan(const sm_fanout_cfg* c, int* n_copies, int* red_dims, int* n_red, size_t* copy_bytes) {
  int rc = check_cfg(c, "sm_fanout_graph_plan");
  if (rc) return rc;
  FanoutPlan p;
  if ((rc = make_plan(c, &p, "sm_fanout_graph_plan"))) return rc;
  if (n_copies) *n_copies = p.n_copies;
  if (n_red) *n_red = p.n_red;
  if (red_dims) { red_dims[0] = p.red_dims[0]; red_dims[1] = p.red_dims[1]; }
  if (copy_bytes) *copy_bytes = (size_t)c->D1 * c->D2 * c->D3 * dtype_size(c->dtype);
  return SM_OK;
}

extern "C" size_t sm_fanout_graph_workspace_bytes(const sm_fanout_cfg* c, int mode) {
  if (check_cfg(c, "sm_fanout_graph_workspace_bytes") != SM_OK) return 0;
  FanoutPlan p;
  if (make_plan(c, &p, "sm_fanout_graph_workspace_bytes") != SM_OK) return 0;
  const size_t t = align256((size_t)c->D1 * c->D2 * c->D3 * dtype_size(c->dtype));
  // elided: one stored tensor per copy the plan keeps; explicit: the MatMul's natural output and its transposed copy
  return (mode == SM_EXPLICIT ? 2 * t + p.tables.bytes : (size_t)p.n_copies * t);
}

extern "C" int sm_fanout_graph(const sm_fanout_cfg* c, const void* a, const void* w, const void* wconv, void* reduce_out,
                               void* reduce_p_out, void* conv_out, void* ws, size_t ws_bytes, int mode, void* stream) {
  int rc = check_cfg(c, "sm_fanout_graph");
  if (rc) return rc;
  if (!a || !w || !wconv || !reduce_out || !reduce_p_out || !conv_out || !ws) return fail(SM_ERR_INVALID_ARG, "sm_fanout_graph: null pointer");
  if (mode != SM_ELIDED && mode != SM_EXPLICIT) return fail(SM_ERR_INVALID_ARG, "sm_fanout_graph: unknown mode %d", mode);
  FanoutPlan p;
  if ((rc = make_plan(c, &p, "sm_fanout_graph"))) return rc;
  const size_t need = sm_fanout_graph_workspace_bytes(c, mode);
  if (ws_bytes < need) return fail(SM_ERR_WORKSPACE, "sm_fanout_graph: workspace of %zu bytes, %zu needed", ws_bytes, need);
  if (!aligned16(a) || !aligned16(w) || !aligned16(wconv) || !aligned16(ws) || !aligned16(conv_out)) return fail(SM_ERR_INVALID_ARG, "sm_fanout_graph: pointers must be 16-byte aligned");
  count_reset();
  const int dt = c->dtype;
  const int64_t D1 = c->D1, D2 = c->D2, D3 = c->D3, D0 = D2 * D3;
  const size_t t = align256((size_t)D1 * D0 * dtype_size(dt));
  char* base = (char*)ws;
  void* by_d3 = base;                 // [D1, D2, D3]: D3 innermost, what Reduce and Conv ask for
  void* by_d1 = base + t;             // [D2, D3, D1] = the MatMul's natural [D0, D1]: D1 innermost, what Reduce' asks for
  GemmArgs g; std::memset(&g, 0, sizeof(g));
  g.A = a; g.W = w; g.M = D0; g.N = (int)D1; g.K = c->Kin; g.dtype = dt; g.ldw = c->Kin;
  g.a_rows = identity_rows(c->Kin); g.c_rows = identity_rows(D1);
  auto launch_reduce = [&](bool last, const void* x, void* y, int64_t rows_or_inner, int n, const char* what) {
    char label[64];
    snprintf(label, sizeof(label), "reduce_%s_%s[%lld,%d]", last ? "last" : "first", dt == SM_F32 ? "f32" : "bf16", (long long)rows_or_inner, n);
    Timed tm(label, stream);
    const int lrc = last ? launch_reduce_last(x, y, rows_or_inner, n, dt, stream) : launch_reduce_first(x, y, n, rows_or_inner, dt, stream);
    if (lrc) return fail(SM_ERR_DEVICE, "sm_fanout_graph: %s launch failed (hip error %d)", what, lrc);
    count_compute();
    return (int)SM_OK;
  };
  if (mode == SM_ELIDED) {
    if (p.n_copies >= 2) {
      // one store per requested reduction dimension, both from the MatMul's epilogue
      g.C = by_d1; g.C2 = by_d3;
      if ((rc = gemm_checked(g, stream, "sm_fanout_graph(matmul)"))) return rc;
    } else {
      // a single layout (k = 2 on 2.5D memory): the first requested dimension innermost, written by the transposed store
      g.C = by_d3; g.c_transposed = 1; g.c_batch_rows = D0;
      if ((rc = gemm_checked(g, stream, "sm_fanout_graph(matmul)"))) return rc;
    }
  } else {
    g.C = by_d1;
    if ((rc = gemm_checked(g, stream, "sm_fanout_graph(matmul)"))) return rc;
    const void* tables = base + 2 * t;
    if ((rc = fill_tables(p.tables, base + 2 * t, stream, ~0ull))) return rc;
    if ((rc = copy_launch(p.transpose, tables, by_d1, by_d3, dt, stream))) return rc;
  }
  if ((rc = launch_reduce(true, by_d3, reduce_out, D1 * D2, (int)D3, "Reduce"))) return rc;
  if (mode == SM_ELIDED && p.n_copies >= 2) { if ((rc = launch_reduce(true, by_d1, reduce_p_out, D0, (int)D1, "Reduce'"))) return rc; }
  else if ((rc = launch_reduce(false, by_d3, reduce_p_out, D0, (int)D1, "Reduce'"))) return rc;
  GemmArgs cv; std::memset(&cv, 0, sizeof(cv));
  cv.A = by_d3; cv.W = wconv; cv.C = conv_out; cv.M = D1 * D2; cv.N = c->Cout; cv.K = (int)D3; cv.dtype = dt; cv.ldw = D3;
  cv.a_rows = identity_rows(D3); cv.c_rows = identity_rows(c->Cout);
  return gemm_checked(cv, stream, "sm_fanout_graph(conv)");
}
