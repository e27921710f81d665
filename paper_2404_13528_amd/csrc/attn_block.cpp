// sm_attn_block: a Llama-style decoder layer (prefill) and a diffusion-UNet
// spatial-transformer block, in elided and explicit-transpose modes.
//
// Each block is first written down as the exporter's operator graph and given
// to sm_layout_plan; the executor checks that the plan leaves exactly the
// compute kernels it is about to launch and takes the attention operands'
// strided views from the planned load / store maps (paper Sec. 3.2.1).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <vector>
#include "common.h"
#include "copy_plan.h"
#include "graph_build.h"
#include "index_map.h"
#include "kernels.h"
#include "plan_chains.h"
#include "plan_views.h"

using namespace sm;

namespace {

struct AttnPlan {
  View4 q1, k1, v1, o1;        // self attention operands as [B, h, S, d] views of their stored tensors
  View4 q2, k2, v2, o2;        // cross attention (SD)
  bool q2_scatter; int q2_gran; RowProg q2_rows, q2_cols;     // cross attention: q's Linear stores head-major when the planner says so
  Copy split_qkv, merge_o, to_tokens, split_q2, split_kv2, merge_o2, to_nchw;
  int n_kept, n_layout, n_eliminated;
  TableRegion el_tables, ex_tables;     // row-offset tables of the elided maps / of the explicit copies
  const TableRegion& tables(int mode) const { return mode == SM_EXPLICIT ? ex_tables : el_tables; }
};

struct Key { int v[12]; bool operator<(const Key& o) const { return std::memcmp(v, o.v, sizeof(v)) < 0; } };
std::mutex g_mu;
std::map<Key, std::shared_ptr<AttnPlan>> g_plans;

bool view_from(const sm_map* m, View4* v, std::string* err, const char* what) {
  int64_t st[SM_MAX_RANK];
  if (!m) { v->base = -1; return true; }
  if (m->shape.size() != 4 || !m->affine(&v->base, st) || st[3] != 1) { *err = std::string(what) + ": operand is not a strided [B, h, S, d] view"; return false; }
  for (int i = 0; i < 3; ++i) v->stride[i] = st[i];
  return true;
}

// operand `slot` of attention op `attn`: planned load map, or the natural layout of the tensor it reads
bool operand_view(const sm_plan* plan, const GraphB& g, int attn, int slot, View4* v, std::string* err) {
  const sm_map* m = nullptr;
  sm_plan_load_map(plan, attn, slot, &m, nullptr);
  if (m) return view_from(m, v, err, "attention load");
  // an element-wise operator fused into the producer (RoPE) is layout independent: it is applied in the
  // layout its producer stores, so the view it read through is the view attention reads through
  int t = g.ops[attn].in[slot];
  for (int i = (int)g.ops.size() - 1; i >= 0; --i) {
    if (g.ops[i].out != t) continue;
    int grp, st;
    sm_plan_op(plan, i, &grp, nullptr, &st, nullptr, nullptr);
    if (grp == SM_ILI_VAR && st == SM_FUSED && g.ops[i].n_in == 1) {
      sm_plan_load_map(plan, i, 0, &m, nullptr);
      if (m) return view_from(m, v, err, "attention load");
      t = g.ops[i].in[0];
    }
  }
  const std::vector<int64_t> s = g.shape(g.ops[attn].in[slot]);
  v->base = 0; v->stride[0] = s[1] * s[2] * s[3]; v->stride[1] = s[2] * s[3]; v->stride[2] = s[3];
  return true;
}
bool output_view(const sm_plan* plan, const GraphB& g, int attn, View4* v, std::string* err) {
  const sm_map* m = nullptr;
  sm_plan_store_map(plan, attn, &m, nullptr);
  if (m) return view_from(m, v, err, "attention store");
  const std::vector<int64_t> s = g.shape(g.ops[attn].out);
  v->base = 0; v->stride[0] = s[1] * s[2] * s[3]; v->stride[1] = s[2] * s[3]; v->stride[2] = s[3];
  return true;
}

bool count_plan(const sm_plan* plan, const GraphB& g, AttnPlan* p) {
  p->n_kept = p->n_layout = p->n_eliminated = 0;
  for (int i = 0; i < (int)g.ops.size(); ++i) {
    int grp, st;
    sm_plan_op(plan, i, &grp, nullptr, &st, nullptr, nullptr);
    p->n_kept += st == SM_KEPT;
    if (grp == SM_ILD_FIX || grp == SM_ILI_FIX) { ++p->n_layout; p->n_eliminated += (st == SM_ELIMINATED_STORE || st == SM_ELIMINATED_LOAD); }
  }
  return p->n_eliminated == p->n_layout;
}

// multi-head attention sub-graph: xq [B, Sq, E], xkv [B, Sk, Ekv]; fused_qkv: one MatMul then slices
int mha_graph(GraphB& g, int xq, int xkv, int64_t B, int64_t Sq, int64_t Sk, int64_t E, int64_t h, bool self, bool rope, const char* name, bool out_bias, bool qkv_bias = false) {
  const int64_t d = E / h;
  std::vector<int> parts;
  auto split = [&](int t, int64_t S) { t = g.reshape(t, {B, S, h, d}); return g.transpose(t, {0, 2, 1, 3}); };
  if (self) {
    const int qkv = g.linear(xq, 3 * E, "qkv", qkv_bias);
    for (int k = 0; k < 3; ++k) {
      int u = split(g.slice(qkv, 2, k * E, (k + 1) * E), Sq);
      if (rope && k < 2) u = g.op(SM_OP_ROPE, {u}, {B, h, Sq, d}, "rope");
      parts.push_back(u);
    }
  } else {
    parts.push_back(split(g.linear(xq, E, "q", false), Sq));
    const int kv = g.linear(xkv, 2 * E, "kv", false);
    for (int k = 0; k < 2; ++k) parts.push_back(split(g.slice(kv, 2, k * E, (k + 1) * E), Sk));
  }
  int t = g.op(SM_OP_ATTENTION, parts, {B, h, Sq, d}, name, {3, 3, -1});
  t = g.transpose(t, {0, 2, 1, 3});
  t = g.reshape(t, {B, Sq, E});
  return g.linear(t, E, "out", out_bias);
}

std::shared_ptr<AttnPlan> attn_plan(const sm_attn_cfg& c, std::string* err) {
  Key key{{c.kind, c.dtype, c.B, c.S, c.E, c.heads, c.F, c.Hs, c.Ws, c.groups, c.Sc, c.Dc}};
  std::lock_guard<std::mutex> lock(g_mu);
  auto it = g_plans.find(key);
  if (it != g_plans.end()) return it->second;
  auto p = std::make_shared<AttnPlan>();
  const int64_t B = c.B, S = c.S, E = c.E, h = c.heads, d = E / h, F = c.F;
  const int es = (int)dtype_size(c.dtype);
  GraphB g;
  int attn1 = -1, attn2 = -1, expect_kept = 0;
  if (c.kind == SM_ATTN_LLAMA) {
    const int x = g.tensor({B, S, E});
    int t = g.op(SM_OP_RMSNORM, {x}, {B, S, E}, "rms1", {2});
    t = mha_graph(g, t, t, B, S, S, E, h, true, true, "attn1", false);
    const int h1 = g.op(SM_OP_ADD, {x, t}, {B, S, E}, "res1");
    t = g.op(SM_OP_RMSNORM, {h1}, {B, S, E}, "rms2", {2});
    const int gu = g.linear(t, 2 * F, "gate_up", false);
    const int ga = g.op(SM_OP_UNARY, {g.slice(gu, 2, 0, F)}, {B, S, F}, "silu");
    const int up = g.slice(gu, 2, F, 2 * F);
    t = g.op(SM_OP_MUL, {ga, up}, {B, S, F}, "swiglu");
    t = g.linear(t, E, "down", false);
    g.op(SM_OP_ADD, {h1, t}, {B, S, E}, "res2");
    expect_kept = 7;
  } else if (c.kind == SM_ATTN_VIT) {
    const int x = g.tensor({B, S, E});
    int t = g.op(SM_OP_LAYERNORM, {x}, {B, S, E}, "ln1", {2});
    t = mha_graph(g, t, t, B, S, S, E, h, true, false, "attn1", true, true);
    const int x1 = g.op(SM_OP_ADD, {x, t}, {B, S, E}, "res1");
    t = g.op(SM_OP_LAYERNORM, {x1}, {B, S, E}, "ln2", {2});
    t = g.linear(t, F, "fc1", true);
    t = g.op(SM_OP_UNARY, {t}, {B, S, F}, "gelu");
    t = g.linear(t, E, "fc2", true);
    g.op(SM_OP_ADD, {x1, t}, {B, S, E}, "res2");
    expect_kept = 7;
  } else {
    const int64_t Hs = c.Hs, Ws = c.Ws;
    const int x = g.tensor({B, E, Hs, Ws});
    const int ctx = g.tensor({B, c.Sc, c.Dc});
    int t = g.op(SM_OP_GROUPNORM, {x}, {B, E, Hs, Ws}, "gn", {1});
    t = g.reshape(t, {B, E, S});
    t = g.transpose(t, {0, 2, 1});
    const int t0 = g.linear(t, E, "proj_in", true);
    t = g.op(SM_OP_LAYERNORM, {t0}, {B, S, E}, "ln1", {2});
    t = mha_graph(g, t, t, B, S, S, E, h, true, false, "attn1", true);
    const int t1 = g.op(SM_OP_ADD, {t0, t}, {B, S, E}, "res1");
    t = g.op(SM_OP_LAYERNORM, {t1}, {B, S, E}, "ln2", {2});
    t = mha_graph(g, t, ctx, B, S, c.Sc, E, h, false, false, "attn2", true);
    const int t2 = g.op(SM_OP_ADD, {t1, t}, {B, S, E}, "res2");
    t = g.op(SM_OP_LAYERNORM, {t2}, {B, S, E}, "ln3", {2});
    const int z = g.linear(t, 2 * F, "ff1", true);
    const int val = g.slice(z, 2, 0, F);
    const int gate = g.op(SM_OP_UNARY, {g.slice(z, 2, F, 2 * F)}, {B, S, F}, "gelu");
    t = g.op(SM_OP_MUL, {val, gate}, {B, S, F}, "geglu");
    t = g.linear(t, E, "ff2", true);
    const int t3 = g.op(SM_OP_ADD, {t2, t}, {B, S, E}, "res3");
    t = g.linear(t3, E, "proj_out", true);
    t = g.transpose(t, {0, 2, 1});
    t = g.reshape(t, {B, E, Hs, Ws});
    g.op(SM_OP_ADD, {t, x}, {B, E, Hs, Ws}, "res_out");
    expect_kept = 15;
  }
  sm_plan* plan = nullptr;
  if (sm_layout_plan(g.tensors.data(), (int)g.tensors.size(), g.ops.data(), (int)g.ops.size(), 1, &plan) != SM_OK) { *err = sm_last_error(); return nullptr; }
  std::unique_ptr<sm_plan, void (*)(sm_plan*)> guard(plan, sm_plan_destroy);
  if (!count_plan(plan, g, p.get()) || p->n_kept != expect_kept) { *err = "planner did not reduce the block to its compute kernels"; return nullptr; }
  attn1 = g.find("attn1"); attn2 = g.find("attn2");
  if (!operand_view(plan, g, attn1, 0, &p->q1, err) || !operand_view(plan, g, attn1, 1, &p->k1, err) ||
      !operand_view(plan, g, attn1, 2, &p->v1, err) || !output_view(plan, g, attn1, &p->o1, err)) return nullptr;
  if (attn2 >= 0 && (!operand_view(plan, g, attn2, 0, &p->q2, err) || !operand_view(plan, g, attn2, 1, &p->k2, err) ||
                     !operand_view(plan, g, attn2, 2, &p->v2, err) || !output_view(plan, g, attn2, &p->o2, err))) return nullptr;
  p->q2_scatter = false;
  if (c.kind == SM_ATTN_SD) {
    const sm_map* qm = nullptr;
    // index of the cross attention's q Linear: the MatMul named "q"
    sm_plan_store_map(plan, g.find("q"), &qm, nullptr);
    if (qm) {
      p->q2_gran = c.dtype == SM_F32 ? 4 : 8;       // whole 16-byte vectors when the head size allows, else per element
      if (!qm->compile_rows_cols(p->q2_gran, &p->q2_rows, &p->q2_cols, err)) {
        p->q2_gran = 1;
        if (!qm->compile_rows_cols(1, &p->q2_rows, &p->q2_cols, err)) return nullptr;
      }
      p->el_tables.add(&p->q2_rows, (int64_t)B * S, (int64_t)B * S * E);
      p->el_tables.add(&p->q2_cols, E / p->q2_gran, (int64_t)B * S * E);
      p->q2_scatter = true;
    }
    // GroupNorm must have been told to store token-major (its consumer reduces over C), proj_out to store NCHW
    const sm_map* m = nullptr;
    sm_plan_store_map(plan, g.find("gn"), &m, nullptr);
    if (!m) { *err = "no store map planned for GroupNorm"; return nullptr; }
    sm_plan_store_map(plan, g.find("proj_out"), &m, nullptr);
    if (!m) { *err = "no store map planned for proj_out"; return nullptr; }
  }
  // explicit mode: copies
  std::vector<sm_view_op> qkv_split{chains::reshape({B, S, 3, h, d}), chains::permute({2, 0, 3, 1, 4})};
  if (!make_copy({B, S, 3 * E}, qkv_split, es, &p->ex_tables, &p->split_qkv, err)) return nullptr;
  if (!make_copy({B, h, S, d}, chains::head_merge(B, S, h, d), es, &p->ex_tables, &p->merge_o, err)) return nullptr;
  if (c.kind == SM_ATTN_SD) {
    if (!make_copy({B, E, S}, {chains::permute({0, 2, 1})}, es, &p->ex_tables, &p->to_tokens, err)) return nullptr;
    if (!make_copy({B, S, E}, {chains::permute({0, 2, 1})}, es, &p->ex_tables, &p->to_nchw, err)) return nullptr;
    if (!make_copy({B, S, E}, chains::head_split(B, S, h, d), es, &p->ex_tables, &p->split_q2, err)) return nullptr;
    std::vector<sm_view_op> kv_split{chains::reshape({B, c.Sc, 2, h, d}), chains::permute({2, 0, 3, 1, 4})};
    if (!make_copy({B, c.Sc, 2 * E}, kv_split, es, &p->ex_tables, &p->split_kv2, err)) return nullptr;
    p->merge_o2 = p->merge_o;
  }
  if (g_plans.size() >= 64) g_plans.clear();      // host objects only; entries in use stay alive through their shared_ptr
  g_plans[key] = p;
  return p;
}

int check_cfg(const sm_attn_cfg* c, const char* who) {
  if (!c) return fail(SM_ERR_INVALID_ARG, "%s: null configuration", who);
  if (c->kind != SM_ATTN_LLAMA && c->kind != SM_ATTN_SD && c->kind != SM_ATTN_VIT) return fail(SM_ERR_INVALID_ARG, "%s: unknown kind %d", who, c->kind);
  if (c->dtype != SM_BF16) return fail(SM_ERR_UNSUPPORTED, "%s: bf16 only", who);
  if (c->B < 1 || c->S < 1 || c->E < 1 || c->heads < 1 || c->F < 1 || c->E % c->heads) return fail(SM_ERR_SHAPE, "%s: bad shape", who);
  const int d = c->E / c->heads;
  if (d % 8 || d > 128) return fail(SM_ERR_SHAPE, "%s: head size must be a multiple of 8 and <= 128", who);
  if (c->F % 32) return fail(SM_ERR_SHAPE, "%s: MLP width must be a multiple of 32", who);
  if (c->kind == SM_ATTN_LLAMA && d % 64) return fail(SM_ERR_SHAPE, "%s: RoPE needs a head size that is a multiple of 64", who);
  if (c->kind == SM_ATTN_SD) {
    if (c->Hs < 1 || c->Ws < 1 || c->Hs * c->Ws != c->S) return fail(SM_ERR_SHAPE, "%s: S must equal Hs * Ws", who);
    if (c->groups < 1 || c->E % c->groups || c->Sc < 1 || c->Dc < 8 || c->Dc % 8) return fail(SM_ERR_SHAPE, "%s: bad GroupNorm / context shape", who);
  }
  return SM_OK;
}

size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

struct Sizes { size_t te, tf, ctx, total; };
Sizes sizes(const sm_attn_cfg* c, int mode) {
  Sizes z;
  const size_t T = (size_t)c->B * c->S, es = dtype_size(c->dtype);
  z.te = align256(T * c->E * es);
  z.tf = align256(T * c->F * es);
  z.ctx = c->kind == SM_ATTN_SD ? align256((size_t)c->B * c->Sc * 2 * c->E * es) : 0;
  // buffers: n (1), qkv (3), o (1), r1, r2, r3 (3), act (F); explicit adds qkv' (3), o' (1), extra (1), ctx copies
  const size_t units = mode == SM_EXPLICIT ? 13 : 8;
  z.total = units * z.te + z.tf + 2 * z.ctx;
  if (c->kind == SM_ATTN_SD) z.total += align256((size_t)2 * c->B * c->groups * sizeof(float));      // GroupNorm statistics
  return z;
}


int norm(const void* x, const void* g, const void* b, void* y, int64_t rows, int C, float eps, int rms, int dt, void* stream) {
  NormArgs a; std::memset(&a, 0, sizeof(a));
  a.x = x; a.gamma = g; a.beta = b; a.y = y; a.rows = rows; a.C = C; a.eps = eps; a.rms = rms; a.dtype = dt; a.nseg = 1;
  a.load = identity_rows(C); a.store = identity_rows(C);
  return norm_checked(a, stream, "norm");
}

int gemm(const void* A, const void* W, const void* bias, const void* res, void* C, int64_t M, int N, int K, int dt, int act, void* stream,
         int rope_cols = 0, int rope_dim = 0, int rope_seq = 0, float rope_base = 0.f, int64_t transposed_batch = 0) {
  GemmArgs g; std::memset(&g, 0, sizeof(g));
  g.A = A; g.W = W; g.bias = bias; g.residual = res; g.C = C; g.M = M; g.N = N; g.K = K; g.dtype = dt; g.act = act; g.ldw = K;
  g.rope_cols = rope_cols; g.rope_dim = rope_dim; g.rope_seq = rope_seq; g.rope_base = rope_base;
  g.c_transposed = transposed_batch ? 1 : 0; g.c_batch_rows = transposed_batch;
  const int n_out = (act == SM_ACT_SWIGLU || act == SM_ACT_GEGLU) ? N / 2 : N;
  g.a_rows = identity_rows(K); g.c_rows = identity_rows(n_out);
  return gemm_checked(g, stream, "linear");
}

int attention(int kind, int dt, int B, int h, int nq, int nk, int d, const View4& q, const View4& k, const View4& v, const View4& o,
              const void* qb, const void* kb, const void* vb, void* ob, void* stream) {
  sm_attention_desc a; std::memset(&a, 0, sizeof(a));
  a.kind = kind; a.dtype = dt; a.nb = B; a.heads = h; a.nq = nq; a.nk = nk; a.d = d; a.scale = 1.0f / sqrtf((float)d);
  for (int i = 0; i < 3; ++i) { a.q_stride[i] = q.stride[i]; a.k_stride[i] = k.stride[i]; a.v_stride[i] = v.stride[i]; a.o_stride[i] = o.stride[i]; }
  const size_t es = dtype_size(dt);
  return attention_checked(a, (const char*)qb + q.base * es, (const char*)kb + k.base * es, (const char*)vb + v.base * es,
                           (char*)ob + o.base * es, nullptr, stream, "attention");
}

View4 contiguous_view(int64_t h, int64_t S, int64_t d, int64_t base = 0) { View4 v; v.base = base; v.stride[0] = h * S * d; v.stride[1] = S * d; v.stride[2] = d; return v; }

}  // namespace

namespace sm {
bool plan_operand_view(const sm_plan* plan, const GraphB& g, int op, int slot, View4* v, std::string* err) { return operand_view(plan, g, op, slot, v, err); }
bool plan_output_view(const sm_plan* plan, const GraphB& g, int op, View4* v, std::string* err) { return output_view(plan, g, op, v, err); }
}

extern "C" size_t sm_attn_block_workspace_bytes(const sm_attn_cfg* c, int mode) {
  if (check_cfg(c, "sm_attn_block_workspace_bytes") != SM_OK) return 0;
  if (mode != SM_ELIDED && mode != SM_EXPLICIT) { set_error("sm_attn_block_workspace_bytes: unknown mode %d", mode); return 0; }
  std::string err;
  auto plan = attn_plan(*c, &err);
  if (!plan) { set_error("sm_attn_block_workspace_bytes: %s", err.c_str()); return 0; }
  return sizes(c, mode).total + plan->tables(mode).bytes;
}

extern "C" int sm_attn_block(const sm_attn_cfg* c, const void* const* w, const void* x, const void* context,
                             void* y, void* ws, size_t ws_bytes, int mode, void* stream) {
  int rc = check_cfg(c, "sm_attn_block");
  if (rc) return rc;
  if (!w || !x || !y || !ws) return fail(SM_ERR_INVALID_ARG, "sm_attn_block: null pointer");
  if (c->kind == SM_ATTN_SD && !context) return fail(SM_ERR_INVALID_ARG, "sm_attn_block: the spatial transformer needs a context");
  if (mode != SM_ELIDED && mode != SM_EXPLICIT) return fail(SM_ERR_INVALID_ARG, "sm_attn_block: unknown mode %d", mode);
  const int nw = c->kind == SM_ATTN_LLAMA ? 6 : (c->kind == SM_ATTN_VIT ? 12 : 23);
  for (int i = 0; i < nw; ++i) if (!w[i] || !aligned16(w[i])) return fail(SM_ERR_INVALID_ARG, "sm_attn_block: weight %d is null or misaligned", i);
  const Sizes z = sizes(c, mode);
  if (!aligned16(x) || !aligned16(y) || !aligned16(ws) || (context && !aligned16(context))) return fail(SM_ERR_INVALID_ARG, "sm_attn_block: pointers must be 16-byte aligned");
  std::string err;
  auto plan = attn_plan(*c, &err);
  if (!plan) return fail(SM_ERR_UNSUPPORTED, "sm_attn_block: %s", err.c_str());
  const size_t need = z.total + plan->tables(mode).bytes;
  if (ws_bytes < need) return fail(SM_ERR_WORKSPACE, "sm_attn_block: workspace of %zu bytes, %zu needed", ws_bytes, need);
  count_reset();
  // the row-offset tables of this call's maps, behind the activation buffers, before the first kernel
  const void* tables = (char*)ws + z.total;
  if ((rc = fill_tables(plan->tables(mode), (char*)ws + z.total, stream, ~0ull))) return rc;
  const int dt = c->dtype, B = c->B, S = c->S, E = c->E, h = c->heads, d = E / h, F = c->F;
  const int64_t T = (int64_t)B * S;
  char* base = (char*)ws;
  void* n = base; void* qkv = base + z.te; void* o = base + 4 * z.te;
  void* r1 = base + 5 * z.te; void* r2 = base + 6 * z.te; void* r3 = base + 7 * z.te;
  char* after = base + 8 * z.te;
  void *qkvp = nullptr, *op = nullptr, *extra = nullptr;
  if (mode == SM_EXPLICIT) { qkvp = after; op = after + 3 * z.te; extra = after + 4 * z.te; after += 5 * z.te; }
  void* act = after; after += z.tf;
  void* kv = after; char* kvp = after + z.ctx;
  const bool el = mode == SM_ELIDED;

  if (c->kind == SM_ATTN_LLAMA) {
    if ((rc = norm(x, w[0], nullptr, n, T, E, c->eps_norm, 1, dt, stream))) return rc;
    if ((rc = gemm(n, w[1], nullptr, nullptr, qkv, T, 3 * E, E, dt, SM_ACT_NONE, stream, 2 * E, d, S, c->rope_base))) return rc;
    if (el) {
      if ((rc = attention(SM_ATT_CAUSAL, dt, B, h, S, S, d, plan->q1, plan->k1, plan->v1, plan->o1, qkv, qkv, qkv, o, stream))) return rc;
    } else {
      if ((rc = copy_launch(plan->split_qkv, tables, qkv, qkvp, dt, stream))) return rc;
      const View4 cq = contiguous_view(h, S, d, 0), ck = contiguous_view(h, S, d, T * E), cv = contiguous_view(h, S, d, 2 * T * E);
      if ((rc = attention(SM_ATT_CAUSAL, dt, B, h, S, S, d, cq, ck, cv, cq, qkvp, qkvp, qkvp, op, stream))) return rc;
      if ((rc = copy_launch(plan->merge_o, tables, op, o, dt, stream))) return rc;
    }
    if ((rc = gemm(o, w[2], nullptr, x, r1, T, E, E, dt, SM_ACT_NONE, stream))) return rc;
    if ((rc = norm(r1, w[3], nullptr, n, T, E, c->eps_norm, 1, dt, stream))) return rc;
    if ((rc = gemm(n, w[4], nullptr, nullptr, act, T, 2 * F, E, dt, SM_ACT_SWIGLU, stream))) return rc;
    if ((rc = gemm(act, w[5], nullptr, r1, y, T, E, F, dt, SM_ACT_NONE, stream))) return rc;
    return SM_OK;
  }

  if (c->kind == SM_ATTN_VIT) {
    // w: ln1_g, ln1_b, wqkv, bqkv, wo, bo, ln2_g, ln2_b, w1, b1, w2, b2
    if ((rc = norm(x, w[0], w[1], n, T, E, c->eps_norm, 0, dt, stream))) return rc;
    if ((rc = gemm(n, w[2], w[3], nullptr, qkv, T, 3 * E, E, dt, SM_ACT_NONE, stream))) return rc;
    if (el) {
      if ((rc = attention(SM_ATT_FULL, dt, B, h, S, S, d, plan->q1, plan->k1, plan->v1, plan->o1, qkv, qkv, qkv, o, stream))) return rc;
    } else {
      if ((rc = copy_launch(plan->split_qkv, tables, qkv, qkvp, dt, stream))) return rc;
      const View4 cq = contiguous_view(h, S, d, 0), ck = contiguous_view(h, S, d, T * E), cv = contiguous_view(h, S, d, 2 * T * E);
      if ((rc = attention(SM_ATT_FULL, dt, B, h, S, S, d, cq, ck, cv, cq, qkvp, qkvp, qkvp, op, stream))) return rc;
      if ((rc = copy_launch(plan->merge_o, tables, op, o, dt, stream))) return rc;
    }
    if ((rc = gemm(o, w[4], w[5], x, r1, T, E, E, dt, SM_ACT_NONE, stream))) return rc;
    if ((rc = norm(r1, w[6], w[7], n, T, E, c->eps_norm, 0, dt, stream))) return rc;
    if ((rc = gemm(n, w[8], w[9], nullptr, act, T, F, E, dt, SM_ACT_GELU, stream))) return rc;
    if ((rc = gemm(act, w[10], w[11], r1, y, T, E, F, dt, SM_ACT_NONE, stream))) return rc;
    return SM_OK;
  }

  // ---- spatial transformer
  const int Sc = c->Sc;
  GroupNormArgs ga{x, w[0], w[1], el ? o : extra, B, E, S, c->groups, c->eps_gn, el ? 1 : 0, dt, (float*)(kvp + z.ctx)};
  {
    char label[64];
    snprintf(label, sizeof(label), "groupnorm_bf16[%d,%d,%d,%d]", B, E, S, c->groups);
    Timed tm(label, stream);
    int lrc = launch_groupnorm(ga, stream);
    if (lrc) return fail(SM_ERR_DEVICE, "sm_attn_block: GroupNorm launch failed (hip error %d)", lrc);
  }
  count_compute(groupnorm_launches(ga));
  if (!el) { if ((rc = copy_launch(plan->to_tokens, tables, extra, o, dt, stream))) return rc; }
  if ((rc = gemm(o, w[2], w[3], nullptr, r1, T, E, E, dt, SM_ACT_NONE, stream))) return rc;                     // proj_in -> t0
  if ((rc = norm(r1, w[4], w[5], n, T, E, c->eps_norm, 0, dt, stream))) return rc;
  if ((rc = gemm(n, w[6], nullptr, nullptr, qkv, T, 3 * E, E, dt, SM_ACT_NONE, stream))) return rc;
  if (el) {
    if ((rc = attention(SM_ATT_FULL, dt, B, h, S, S, d, plan->q1, plan->k1, plan->v1, plan->o1, qkv, qkv, qkv, o, stream))) return rc;
  } else {
    if ((rc = copy_launch(plan->split_qkv, tables, qkv, qkvp, dt, stream))) return rc;
    const View4 cq = contiguous_view(h, S, d, 0), ck = contiguous_view(h, S, d, T * E), cv = contiguous_view(h, S, d, 2 * T * E);
    if ((rc = attention(SM_ATT_FULL, dt, B, h, S, S, d, cq, ck, cv, cq, qkvp, qkvp, qkvp, op, stream))) return rc;
    if ((rc = copy_launch(plan->merge_o, tables, op, o, dt, stream))) return rc;
  }
  if ((rc = gemm(o, w[7], w[8], r1, r2, T, E, E, dt, SM_ACT_NONE, stream))) return rc;                          // t1
  if ((rc = norm(r2, w[9], w[10], n, T, E, c->eps_norm, 0, dt, stream))) return rc;
  {                                                                                                            // q of the cross attention
    GemmArgs gq; std::memset(&gq, 0, sizeof(gq));
    gq.A = n; gq.W = w[11]; gq.C = qkv; gq.M = T; gq.N = E; gq.K = E; gq.dtype = dt; gq.ldw = E;
    gq.a_rows = identity_rows(E); gq.c_rows = identity_rows(E);
    if (el && plan->q2_scatter) { gq.c_rows = bound(plan->q2_rows, tables); gq.c_cols = bound(plan->q2_cols, tables); gq.c_cols_on = 1; gq.c_gran = plan->q2_gran; }
    if ((rc = gemm_checked(gq, stream, "linear"))) return rc;
  }
  if ((rc = gemm(context, w[12], nullptr, nullptr, kv, (int64_t)B * Sc, 2 * E, c->Dc, dt, SM_ACT_NONE, stream))) return rc;
  if (el) {
    if ((rc = attention(SM_ATT_FULL, dt, B, h, S, Sc, d, plan->q2, plan->k2, plan->v2, plan->o2, qkv, kv, kv, o, stream))) return rc;
  } else {
    if ((rc = copy_launch(plan->split_q2, tables, qkv, qkvp, dt, stream))) return rc;
    if ((rc = copy_launch(plan->split_kv2, tables, kv, kvp, dt, stream))) return rc;
    const View4 cq = contiguous_view(h, S, d, 0), ck = contiguous_view(h, Sc, d, 0), cv = contiguous_view(h, Sc, d, (int64_t)B * Sc * E);
    if ((rc = attention(SM_ATT_FULL, dt, B, h, S, Sc, d, cq, ck, cv, cq, qkvp, kvp, kvp, op, stream))) return rc;
    if ((rc = copy_launch(plan->merge_o2, tables, op, o, dt, stream))) return rc;
  }
  if ((rc = gemm(o, w[13], w[14], r2, r3, T, E, E, dt, SM_ACT_NONE, stream))) return rc;                        // t2
  if ((rc = norm(r3, w[15], w[16], n, T, E, c->eps_norm, 0, dt, stream))) return rc;
  if ((rc = gemm(n, w[17], w[18], nullptr, act, T, 2 * F, E, dt, SM_ACT_GEGLU, stream))) return rc;
  if ((rc = gemm(act, w[19], w[20], r3, r1, T, E, F, dt, SM_ACT_NONE, stream))) return rc;                      // t3
  if (el) {
    if ((rc = gemm(r1, w[21], w[22], x, y, T, E, E, dt, SM_ACT_NONE, stream, 0, 0, 0, 0.f, S))) return rc;       // NCHW store + x
  } else {
    if ((rc = gemm(r1, w[21], w[22], nullptr, o, T, E, E, dt, SM_ACT_NONE, stream))) return rc;
    if ((rc = copy_launch(plan->to_nchw, tables, o, y, dt, stream, x))) return rc;
  }
  return SM_OK;
}
