// Block and chain executors: sm_swin_block and sm_run_chain.
//
// Each executor asks the composer for the maps of the layout transformations
// in its operator chain and hands them to the kernels (elided mode), or runs
// one copy kernel per transformation that moves data (explicit mode: Reshape
// is metadata only on linear memory, paper Sec. 2.3).  Plans are host memory
// only and are cached per configuration (a bounded cache behind a mutex); the
// per-row offset tables of their maps live in the caller's workspace and are
// filled on the caller's stream at the start of every call.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <tuple>
#include <vector>
#include "common.h"
#include "index_map.h"
#include "kernels.h"
#include "plan_chains.h"
#include "copy_plan.h"
#include "graph_build.h"

using namespace sm;

namespace {

struct SwinPlan {
  // elided: what sm_layout_plan decided for the block's operator graph
  RowProg ln1_store;     // natural token row -> row offset in the window-major tensor
  RowProg proj_store;    // window-major row -> row offset in the natural tensor
  RowProg x_gather;      // window-major row -> row offset in the natural tensor, roll included: the A-load of QKV when
                         // LayerNorm-1 is folded into it (the map LayerNorm's store would have applied, read side)
  int64_t qkv_base[3], qkv_stride[3][3], o_stride[3];   // q, k, v and o as strided views [B_, h, N, d]
  // explicit
  bool has_roll;
  Copy roll, partition, head_split, head_merge, reverse, unroll;
  int n_layout_ops, n_eliminated;
  TableRegion el_tables, ex_tables;   // row-offset tables of the elided maps / of the explicit copies
  const TableRegion& tables(int mode) const { return mode == SM_EXPLICIT ? ex_tables : el_tables; }
};

struct Key {
  int v[8];
  bool operator<(const Key& o) const { return std::memcmp(v, o.v, sizeof(v)) < 0; }
};

std::mutex g_mu;
std::map<Key, std::shared_ptr<SwinPlan>> g_swin;
// plans are small host objects; a cache that has seen many configurations starts over (entries in use stay alive
// through their shared_ptr)
constexpr size_t kMaxCachedPlans = 64;
template <typename M> void bound_cache(M& m) { if (m.size() >= kMaxCachedPlans) m.clear(); }

int64_t numel_of(const std::vector<int64_t>& s) { int64_t n = 1; for (auto e : s) n *= e; return n; }

bool make_rows(const std::vector<int64_t>& src, const std::vector<sm_view_op>& chain, TableRegion* tables, RowProg* out, std::string* err) {
  sm_map* m = nullptr;
  if (map_create(src, chain.data(), (int)chain.size(), &m, err) != SM_OK) return false;
  const bool ok = m->compile_rows(out, err);
  if (ok) tables->add(out, m->numel() / m->shape.back(), numel_of(src));
  delete m;
  return ok;
}

std::shared_ptr<SwinPlan> swin_plan(const sm_swin_cfg& c, std::string* err) {
  Key key{{c.B, c.H, c.W, c.C, c.heads, c.window, c.shift, c.dtype}};
  std::lock_guard<std::mutex> lock(g_mu);
  auto it = g_swin.find(key);
  if (it != g_swin.end()) return it->second;
  auto p = std::make_shared<SwinPlan>();
  const int64_t B = c.B, H = c.H, W = c.W, C = c.C, w = c.window, s = c.shift, h = c.heads;
  const int64_t N = w * w, d = C / h, B_ = B * (H / w) * (W / w);
  const int es = (int)dtype_size(c.dtype);
  // elided: describe the block as the exporter's operator graph and let the planner decide
  {
    GraphB g;
    const int x = g.tensor({B, H * W, C});
    int t = g.op(SM_OP_LAYERNORM, {x}, {B, H * W, C}, "ln1", {2});
    t = g.reshape(t, {B, H, W, C});
    if (s) { t = g.roll(t, 1, -s); t = g.roll(t, 2, -s); }
    t = g.reshape(t, {B, H / w, w, W / w, w, C});
    t = g.transpose(t, {0, 1, 3, 2, 4, 5});
    t = g.reshape(t, {B_, N, C});
    t = g.linear(t, 3 * C, "qkv", true);
    t = g.reshape(t, {B_, N, 3, h, d});
    t = g.transpose(t, {2, 0, 3, 1, 4});
    std::vector<int> qkv;
    for (int k = 0; k < 3; ++k) qkv.push_back(g.reshape(g.slice(t, 0, k, k + 1), {B_, h, N, d}));
    t = g.op(SM_OP_ATTENTION, qkv, {B_, h, N, d}, "attn", {3, 3, -1});
    t = g.transpose(t, {0, 2, 1, 3});
    t = g.reshape(t, {B_, N, C});
    t = g.linear(t, C, "proj", true);
    t = g.reshape(t, {B, H / w, W / w, w, w, C});
    t = g.transpose(t, {0, 1, 3, 2, 4, 5});
    t = g.reshape(t, {B, H, W, C});
    if (s) { t = g.roll(t, 1, s); t = g.roll(t, 2, s); }
    t = g.reshape(t, {B, H * W, C});
    const int x1 = g.op(SM_OP_ADD, {x, t}, {B, H * W, C}, "res1");
    t = g.op(SM_OP_LAYERNORM, {x1}, {B, H * W, C}, "ln2", {2});
    t = g.linear(t, c.mlp_ratio * C, "fc1", true);
    t = g.op(SM_OP_UNARY, {t}, {B, H * W, c.mlp_ratio * C}, "gelu");
    t = g.linear(t, C, "fc2", true);
    g.op(SM_OP_ADD, {x1, t}, {B, H * W, C}, "res2");
    sm_plan* plan = nullptr;
    if (sm_layout_plan(g.tensors.data(), (int)g.tensors.size(), g.ops.data(), (int)g.ops.size(), 1, &plan) != SM_OK) { *err = sm_last_error(); return nullptr; }
    std::unique_ptr<sm_plan, void (*)(sm_plan*)> guard(plan, sm_plan_destroy);
    int kept = 0, layout_ops = 0, eliminated = 0;
    for (int i = 0; i < (int)g.ops.size(); ++i) {
      int grp, st;
      sm_plan_op(plan, i, &grp, nullptr, &st, nullptr, nullptr);
      kept += st == SM_KEPT;
      if (grp == SM_ILD_FIX || grp == SM_ILI_FIX) { ++layout_ops; eliminated += (st == SM_ELIMINATED_STORE || st == SM_ELIMINATED_LOAD); }
    }
    p->n_layout_ops = layout_ops; p->n_eliminated = eliminated;
    if (kept != 7 || eliminated != layout_ops) { *err = "planner did not reduce the Swin block to its seven compute kernels"; return nullptr; }
    const sm_map* m = nullptr;
    sm_plan_store_map(plan, g.find("ln1"), &m, nullptr);
    if (!m || !m->compile_rows(&p->ln1_store, err)) { if (!m) *err = "no store map planned for LayerNorm"; return nullptr; }
    p->el_tables.add(&p->ln1_store, B * H * W, B * H * W * C);
    sm_plan_store_map(plan, g.find("proj"), &m, nullptr);
    if (!m || !m->compile_rows(&p->proj_store, err)) { if (!m) *err = "no store map planned for proj"; return nullptr; }
    p->el_tables.add(&p->proj_store, B_ * N, B * H * W * C);
    const int attn = g.find("attn");
    int64_t st8[SM_MAX_RANK];
    for (int k = 0; k < 3; ++k) {
      sm_plan_load_map(plan, attn, k, &m, nullptr);
      if (!m || !m->affine(&p->qkv_base[k], st8) || st8[3] != 1) { *err = "attention operand is not a strided view"; return nullptr; }
      for (int j = 0; j < 3; ++j) p->qkv_stride[k][j] = st8[j];
    }
    int64_t obase;
    sm_plan_store_map(plan, attn, &m, nullptr);
    if (!m || !m->affine(&obase, st8) || st8[3] != 1 || obase != 0) { *err = "attention output is not a strided view"; return nullptr; }
    for (int j = 0; j < 3; ++j) p->o_stride[j] = st8[j];
  }
  if (!make_rows({B, H, W, C}, chains::window_partition(B, H, W, C, w, s), &p->el_tables, &p->x_gather, err)) return nullptr;
  // explicit: one copy per transformation that moves data
  p->has_roll = s != 0;
  if (s) {
    if (!make_copy({B, H, W, C}, chains::roll2(-s), es, &p->ex_tables, &p->roll, err)) return nullptr;
    if (!make_copy({B, H, W, C}, chains::roll2(s), es, &p->ex_tables, &p->unroll, err)) return nullptr;
  }
  if (!make_copy({B, H, W, C}, chains::window_partition(B, H, W, C, w, 0), es, &p->ex_tables, &p->partition, err)) return nullptr;
  if (!make_copy({B_, N, C}, chains::window_reverse(B, H, W, C, w, 0), es, &p->ex_tables, &p->reverse, err)) return nullptr;
  if (!make_copy({B_, N, 3 * C}, chains::qkv_split(B_, N, h, d), es, &p->ex_tables, &p->head_split, err)) return nullptr;
  if (!make_copy({B_, h, N, d}, chains::head_merge(B_, N, h, d), es, &p->ex_tables, &p->head_merge, err)) return nullptr;
  bound_cache(g_swin);
  g_swin[key] = p;
  return p;
}

int check_swin(const sm_swin_cfg* c, const char* who) {
  if (!c) return fail(SM_ERR_INVALID_ARG, "%s: null configuration", who);
  if (!dtype_ok(c->dtype)) return fail(SM_ERR_INVALID_ARG, "%s: unknown dtype", who);
  if (c->B < 1 || c->H < 1 || c->W < 1 || c->C < 1 || c->heads < 1 || c->window < 1 || c->mlp_ratio < 1)
    return fail(SM_ERR_SHAPE, "%s: non-positive dimension", who);
  if (c->H % c->window || c->W % c->window)
    return fail(SM_ERR_SHAPE, "%s: grid %d x %d is not a multiple of the window %d", who, c->H, c->W, c->window);
  if (c->C % c->heads) return fail(SM_ERR_SHAPE, "%s: C = %d is not a multiple of heads = %d", who, c->C, c->heads);
  if (c->shift < 0 || c->shift >= c->window) return fail(SM_ERR_SHAPE, "%s: shift out of range", who);
  const int vec = c->dtype == SM_F32 ? 4 : 8;
  if ((c->C / c->heads) % vec) return fail(SM_ERR_SHAPE, "%s: head size must be a multiple of %d", who, vec);
  return SM_OK;
}

size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }


int run_norm(const void* x, const void* g, const void* b, void* y, int64_t rows, int C, float eps, int rms, int dtype,
             const RowProg* load, int nseg, const RowProg* store, void* stream) {
  NormArgs a; std::memset(&a, 0, sizeof(a));
  a.x = x; a.gamma = g; a.beta = b; a.y = y; a.rows = rows; a.C = C; a.eps = eps; a.rms = rms; a.dtype = dtype; a.nseg = nseg;
  a.load = load ? *load : identity_rows(C);
  a.store = store ? *store : identity_rows(C);
  return norm_checked(a, stream, "norm");
}

// ln_g != null: LayerNorm (gamma ln_g, beta ln_b, eps) of A's rows folded into the load
int run_gemm(const void* A, const void* W, const void* bias, const void* res, void* C, int64_t M, int N, int K, int dtype,
             int act, const RowProg* a_rows, const RowProg* c_rows, void* stream,
             const void* ln_g = nullptr, const void* ln_b = nullptr, float ln_eps = 0.f) {
  GemmArgs g; std::memset(&g, 0, sizeof(g));
  g.A = A; g.W = W; g.bias = bias; g.residual = res; g.C = C; g.M = M; g.N = N; g.K = K; g.dtype = dtype; g.act = act; g.ldw = K;
  if (ln_g) { g.norm = 1; g.norm_gamma = ln_g; g.norm_beta = ln_b; g.norm_eps = ln_eps; }
  const int n_out = (act == SM_ACT_SWIGLU || act == SM_ACT_GEGLU) ? N / 2 : N;
  g.a_rows = a_rows ? *a_rows : identity_rows(K);
  g.c_rows = c_rows ? *c_rows : identity_rows(n_out);
  return gemm_checked(g, stream, "linear");
}

// A LayerNorm is folded into the Linear that consumes it where that is faster than two kernels: the folded Linear
// stages A through registers (slower per tile than the LDS-DMA path) and repeats the norm per column tile, so it
// wins only while the Linear has few column tiles (measured: up to N = 512).
bool fold_norm(int n_cols) { return n_cols <= 512; }

// LayerNorm-2 + FC1 + GELU + FC2 + residual as the fused MLP kernel, when the caller packed the weights for it
bool mlp_is_fused(const sm_swin_cfg& c, const sm_swin_weights* wt) {
  return wt->mlp_packed && mlp_fused_supported(c.C, c.mlp_ratio * c.C, c.dtype);
}
// ... and the output projection with its window-reverse store and the first residual in front of it (elided mode)
bool proj_is_fused(const sm_swin_cfg& c, const sm_swin_weights* wt) {
  return wt->proj_packed && wt->mlp_packed && mlp_proj_supported(c.C, c.mlp_ratio * c.C, c.dtype);
}
// Where the row at window-major position r of a block with shift c.shift goes in the window-major tensor of a block
// with shift next_shift: the composed map reverse(next) then partition(this), read as a store (Sec. 3.2.1: two runs of
// layout operators between two surviving operators collapse into one index expression)
struct NextStore { RowProg rows; TableRegion tables; };
std::map<Key, std::shared_ptr<NextStore>> g_next_store;
std::shared_ptr<NextStore> next_norm_store(const sm_swin_cfg& c, int next_shift, std::string* err) {
  Key key{{c.B, c.H, c.W, c.C, c.window, c.shift, next_shift, c.dtype}};
  std::lock_guard<std::mutex> lock(g_mu);
  auto it = g_next_store.find(key);
  if (it != g_next_store.end()) return it->second;
  const int64_t B = c.B, H = c.H, W = c.W, C = c.C, w = c.window;
  std::vector<sm_view_op> ch = chains::window_reverse(B, H, W, C, w, next_shift);
  for (auto& op : chains::window_partition(B, H, W, C, w, c.shift)) ch.push_back(op);
  auto p = std::make_shared<NextStore>();
  if (!make_rows({B * (H / w) * (W / w), w * w, C}, ch, &p->tables, &p->rows, err)) return nullptr;
  bound_cache(g_next_store);
  g_next_store[key] = p;
  return p;
}

// LayerNorm-1 of the block that follows in a chain, emitted by this block's last kernel as a second output (window-major,
// i.e. through the following block's own partition map) into the workspace slot that block reads its QKV input from
// which of a plan's elided tables (el_tables items, in the order swin_plan adds them: LayerNorm-1 store, projection
// store, x gather) the block's kernels read: the projection's always, one of the other two unless the block's QKV
// input was produced by the block before it (pre)
enum { TBL_LN1_STORE = 1, TBL_PROJ_STORE = 2, TBL_X_GATHER = 4 };
uint64_t el_tables_needed(const sm_swin_cfg& c, const sm_swin_weights* wt, int pre) {
  uint64_t need = TBL_PROJ_STORE;
  if (pre == 0) need |= ((wt->qkv_packed && lin32_supported(3 * c.C, c.C, c.dtype)) || fold_norm(3 * c.C)) ? TBL_X_GATHER : TBL_LN1_STORE;
  return need;
}

struct NextNorm { const void* gamma; const void* beta; RowProg store; const void* wq_p; const void* bq; };   // wq_p: ... and its QKV Linear
int run_proj_mlp_fused(const sm_swin_cfg& c, const sm_swin_weights* wt, const void* attn_out, const void* x, void* y, int64_t T,
                       const RowProg& store, const NextNorm* next, void* next_out, void* stream) {      // next_out: norm or QKV slot
  MlpArgs a; std::memset(&a, 0, sizeof(a));
  a.X = attn_out; a.Wp = wt->mlp_packed; a.b1 = wt->b1; a.b2 = wt->b2; a.Y = y;
  a.M = T; a.C = c.C; a.Hd = c.mlp_ratio * c.C;
  a.norm = 1; a.norm_eps = c.eps; a.norm_gamma = wt->ln2_g; a.norm_beta = wt->ln2_b;
  a.Wproj_p = wt->proj_packed; a.bproj = wt->bproj; a.resid0 = x;
  a.x_rows = identity_rows(c.C); a.y_rows = store;
  if (next) {
    a.Y2 = next_out; a.ln2_gamma = next->gamma; a.ln2_beta = next->beta; a.ln2_eps = c.eps; a.y2_rows = next->store;
    a.Wq_p = next->wq_p; a.bq = next->bq;
  }
  return mlp_checked(a, stream, "sm_swin_block(proj+mlp)");
}
int run_mlp_fused(const sm_swin_cfg& c, const sm_swin_weights* wt, const void* x1, void* y, int64_t T, void* stream) {
  MlpArgs a; std::memset(&a, 0, sizeof(a));
  a.X = x1; a.Wp = wt->mlp_packed; a.b1 = wt->b1; a.b2 = wt->b2; a.residual = x1; a.Y = y;
  a.M = T; a.C = c.C; a.Hd = c.mlp_ratio * c.C;
  a.norm = 1; a.norm_eps = c.eps; a.norm_gamma = wt->ln2_g; a.norm_beta = wt->ln2_b;
  a.x_rows = identity_rows(c.C); a.y_rows = identity_rows(c.C);
  return mlp_checked(a, stream, "sm_swin_block(mlp)");
}

}  // namespace

namespace {
// activation buffers of one block (without its row-offset tables)
size_t swin_act_bytes(const sm_swin_cfg* c, int mode) {
  const size_t tc = align256((size_t)c->B * c->H * c->W * c->C * dtype_size(c->dtype));
  const size_t units = mode == SM_EXPLICIT ? 4 + 3 + 3 + 1 + c->mlp_ratio : 1 + 3 + 1 + 1 + c->mlp_ratio;
  return tc * units;
}
int swin_block_impl(const sm_swin_cfg* c, const sm_swin_weights* wt, const void* x, void* y, void* ws, size_t ws_bytes, int mode,
                    void* stream, const NextNorm* next, int pre, const void* tables);
}

extern "C" size_t sm_swin_block_workspace_bytes(const sm_swin_cfg* c, int mode) {
  if (check_swin(c, "sm_swin_block_workspace_bytes") != SM_OK) return 0;
  if (mode != SM_ELIDED && mode != SM_EXPLICIT) { set_error("sm_swin_block_workspace_bytes: unknown mode %d", mode); return 0; }
  std::string err;
  auto plan = swin_plan(*c, &err);
  if (!plan) { set_error("sm_swin_block_workspace_bytes: %s", err.c_str()); return 0; }
  return swin_act_bytes(c, mode) + plan->tables(mode).bytes;
}

extern "C" int sm_swin_block(const sm_swin_cfg* c, const sm_swin_weights* wt, const void* x, void* y,
                             void* ws, size_t ws_bytes, int mode, void* stream) {
  return swin_block_impl(c, wt, x, y, ws, ws_bytes, mode, stream, nullptr, 0, nullptr);
}

namespace {
// next (elided mode, projection + MLP fused only): also emit the following block's LayerNorm-1 into this workspace's
// first slot, or (next->wq_p) its QKV Linear's output into the QKV slot; pre = 1: the first slot already holds this
// block's LayerNorm-1 output, pre = 2: the QKV slot already holds this block's QKV (the previous block emitted it).
// tables: where the plan's row-offset tables for `mode` were already filled on this stream (the chain executor fills
// them once per stage and shift); null: they go behind the activation buffers of ws and are filled here
int swin_block_impl(const sm_swin_cfg* c, const sm_swin_weights* wt, const void* x, void* y, void* ws, size_t ws_bytes, int mode,
                    void* stream, const NextNorm* next, int pre, const void* tables) {
  int rc = check_swin(c, "sm_swin_block");
  if (rc) return rc;
  if (!wt || !x || !y || !ws) return fail(SM_ERR_INVALID_ARG, "sm_swin_block: null pointer");
  if (mode != SM_ELIDED && mode != SM_EXPLICIT) return fail(SM_ERR_INVALID_ARG, "sm_swin_block: unknown mode %d", mode);
  if (!aligned16(x) || !aligned16(y) || !aligned16(ws)) return fail(SM_ERR_INVALID_ARG, "sm_swin_block: pointers must be 16-byte aligned");
  std::string err;
  auto plan = swin_plan(*c, &err);
  if (!plan) return fail(SM_ERR_UNSUPPORTED, "sm_swin_block: %s", err.c_str());
  const size_t need = swin_act_bytes(c, mode) + (tables ? 0 : plan->tables(mode).bytes);
  if (ws_bytes < need) return fail(SM_ERR_WORKSPACE, "sm_swin_block: workspace of %zu bytes, %zu needed", ws_bytes, need);
  count_reset();
  if (!tables) {
    void* region = (char*)ws + swin_act_bytes(c, mode);
    if ((rc = fill_tables(plan->tables(mode), region, stream, mode == SM_ELIDED ? el_tables_needed(*c, wt, pre) : ~0ull))) return rc;
    tables = region;
  }
  const RowProg ln1_store = bound(plan->ln1_store, tables), proj_store = bound(plan->proj_store, tables),
                x_gather = bound(plan->x_gather, tables);
  const int64_t T = (int64_t)c->B * c->H * c->W;
  const int C = c->C, h = c->heads, w = c->window, N = w * w, d = C / h, dt = c->dtype;
  const int64_t B_ = T / N;
  const size_t tc = align256((size_t)T * C * dtype_size(dt));
  char* base = (char*)ws;
  const float eps = c->eps;

  sm_attention_desc ad; std::memset(&ad, 0, sizeof(ad));
  ad.kind = SM_ATT_WINDOW; ad.dtype = dt; ad.nb = (int)B_; ad.heads = h; ad.nq = N; ad.nk = N; ad.d = d;
  ad.scale = 1.0f / sqrtf((float)d);
  ad.window = w; ad.shift = c->shift; ad.H = c->H; ad.W = c->W;

  if (mode == SM_ELIDED) {
    void* bufA = base; void* qkv = base + tc; void* bufO = base + 4 * tc; void* x1 = base + 5 * tc; void* hid = base + 6 * tc;
    if (pre == 2) {
      // nothing: the QKV slot is filled
    } else if (pre == 1) {
      if ((rc = run_gemm(bufA, wt->wqkv, wt->bqkv, nullptr, qkv, T, 3 * C, C, dt, SM_ACT_NONE, nullptr, nullptr, stream))) return rc;
    } else if (wt->qkv_packed && lin32_supported(3 * C, C, dt)) {
      // LayerNorm-1 + QKV as one packed-weight Linear: x's rows gathered in window-major order (roll included), the
      // tile normalised in LDS, the weight streamed
      Lin32Args a; std::memset(&a, 0, sizeof(a));
      a.X = x; a.Wp = wt->qkv_packed; a.bias = wt->bqkv; a.Y = qkv; a.M = T; a.N = 3 * C; a.K = C; a.act = SM_ACT_NONE;
      a.norm = 1; a.norm_eps = eps; a.norm_gamma = wt->ln1_g; a.norm_beta = wt->ln1_b;
      a.x_rows = x_gather; a.y_rows = identity_rows(3 * C);
      if ((rc = lin32_checked(a, stream, "sm_swin_block(ln1+qkv)"))) return rc;
    } else if (fold_norm(3 * C)) {
      if ((rc = run_gemm(x, wt->wqkv, wt->bqkv, nullptr, qkv, T, 3 * C, C, dt, SM_ACT_NONE, &x_gather, nullptr, stream, wt->ln1_g, wt->ln1_b, eps))) return rc;
    } else {
      if ((rc = run_norm(x, wt->ln1_g, wt->ln1_b, bufA, T, C, eps, 0, dt, nullptr, 1, &ln1_store, stream))) return rc;
      if ((rc = run_gemm(bufA, wt->wqkv, wt->bqkv, nullptr, qkv, T, 3 * C, C, dt, SM_ACT_NONE, nullptr, nullptr, stream))) return rc;
    }
    const size_t es = dtype_size(dt);
    for (int i = 0; i < 3; ++i) {
      ad.q_stride[i] = plan->qkv_stride[0][i]; ad.k_stride[i] = plan->qkv_stride[1][i]; ad.v_stride[i] = plan->qkv_stride[2][i];
      ad.o_stride[i] = plan->o_stride[i];
    }
    if ((rc = attention_checked(ad, (char*)qkv + plan->qkv_base[0] * es, (char*)qkv + plan->qkv_base[1] * es, (char*)qkv + plan->qkv_base[2] * es,
                                bufO, wt->rpb_table, stream, "window attention"))) return rc;
    if (proj_is_fused(*c, wt)) return run_proj_mlp_fused(*c, wt, bufO, x, y, T, proj_store, next, next && next->wq_p ? qkv : bufA, stream);
    if (next) return fail(SM_ERR_INVALID_ARG, "sm_swin_block: the next block's norm can only be emitted by the fused projection + MLP kernel");
    if ((rc = run_gemm(bufO, wt->wproj, wt->bproj, x, x1, T, C, C, dt, SM_ACT_NONE, nullptr, &proj_store, stream))) return rc;
    if (mlp_is_fused(*c, wt)) return run_mlp_fused(*c, wt, x1, y, T, stream);
    if (fold_norm(c->mlp_ratio * C)) {
      if ((rc = run_gemm(x1, wt->w1, wt->b1, nullptr, hid, T, c->mlp_ratio * C, C, dt, SM_ACT_GELU, nullptr, nullptr, stream, wt->ln2_g, wt->ln2_b, eps))) return rc;
    } else {
      if ((rc = run_norm(x1, wt->ln2_g, wt->ln2_b, bufA, T, C, eps, 0, dt, nullptr, 1, nullptr, stream))) return rc;
      if ((rc = run_gemm(bufA, wt->w1, wt->b1, nullptr, hid, T, c->mlp_ratio * C, C, dt, SM_ACT_GELU, nullptr, nullptr, stream))) return rc;
    }
    if ((rc = run_gemm(hid, wt->w2, wt->b2, x1, y, T, C, c->mlp_ratio * C, dt, SM_ACT_NONE, nullptr, nullptr, stream))) return rc;
    return SM_OK;
  }

  if (next || pre) return fail(SM_ERR_INVALID_ARG, "sm_swin_block: cross-block norm emission is an elided-mode path");
  void* s0 = base; void* s1 = base + tc; void* s2 = base + 2 * tc; void* s3 = base + 3 * tc;
  void* qkv = base + 4 * tc; void* qkvp = base + 7 * tc; void* x1 = base + 10 * tc; void* hid = base + 11 * tc;
  // (a row-wise norm commutes with the row permutations that follow it: where LayerNorm-1 is folded into QKV the
  // copies move x itself)
  const bool f1 = fold_norm(3 * C);
  const void* cur = x;
  if (!f1) { if ((rc = run_norm(x, wt->ln1_g, wt->ln1_b, s0, T, C, eps, 0, dt, nullptr, 1, nullptr, stream))) return rc; cur = s0; }
  if (plan->has_roll) { if ((rc = copy_launch(plan->roll, tables, cur, s1, dt, stream))) return rc; cur = s1; }
  if ((rc = copy_launch(plan->partition, tables, cur, s2, dt, stream))) return rc;
  if ((rc = run_gemm(s2, wt->wqkv, wt->bqkv, nullptr, qkv, T, 3 * C, C, dt, SM_ACT_NONE, nullptr, nullptr, stream,
                     f1 ? wt->ln1_g : nullptr, wt->ln1_b, eps))) return rc;
  if ((rc = copy_launch(plan->head_split, tables, qkv, qkvp, dt, stream))) return rc;          // [3, B_, h, N, d]
  ad.q_stride[0] = ad.k_stride[0] = ad.v_stride[0] = ad.o_stride[0] = (int64_t)h * N * d;
  ad.q_stride[1] = ad.k_stride[1] = ad.v_stride[1] = ad.o_stride[1] = (int64_t)N * d;
  ad.q_stride[2] = ad.k_stride[2] = ad.v_stride[2] = ad.o_stride[2] = d;
  const size_t part = (size_t)T * C * dtype_size(dt);
  if ((rc = attention_checked(ad, qkvp, (char*)qkvp + part, (char*)qkvp + 2 * part, s0, wt->rpb_table, stream, "window attention"))) return rc;
  if ((rc = copy_launch(plan->head_merge, tables, s0, s1, dt, stream))) return rc;             // [B_, N, C]
  if ((rc = run_gemm(s1, wt->wproj, wt->bproj, nullptr, s2, T, C, C, dt, SM_ACT_NONE, nullptr, nullptr, stream))) return rc;
  if (plan->has_roll) {
    if ((rc = copy_launch(plan->reverse, tables, s2, s3, dt, stream))) return rc;
    if ((rc = copy_launch(plan->unroll, tables, s3, x1, dt, stream, x))) return rc;            // + residual
  } else {
    if ((rc = copy_launch(plan->reverse, tables, s2, x1, dt, stream, x))) return rc;
  }
  if (mlp_is_fused(*c, wt)) return run_mlp_fused(*c, wt, x1, y, T, stream);
  if (fold_norm(c->mlp_ratio * C)) {
    if ((rc = run_gemm(x1, wt->w1, wt->b1, nullptr, hid, T, c->mlp_ratio * C, C, dt, SM_ACT_GELU, nullptr, nullptr, stream, wt->ln2_g, wt->ln2_b, eps))) return rc;
  } else {
    if ((rc = run_norm(x1, wt->ln2_g, wt->ln2_b, s0, T, C, eps, 0, dt, nullptr, 1, nullptr, stream))) return rc;
    if ((rc = run_gemm(s0, wt->w1, wt->b1, nullptr, hid, T, c->mlp_ratio * C, C, dt, SM_ACT_GELU, nullptr, nullptr, stream))) return rc;
  }
  if ((rc = run_gemm(hid, wt->w2, wt->b2, x1, y, T, C, c->mlp_ratio * C, dt, SM_ACT_NONE, nullptr, nullptr, stream))) return rc;
  return SM_OK;
}
}  // namespace

// ---------------------------------------------------------------------------
// sm_run_chain
// ---------------------------------------------------------------------------
namespace {

struct MergePlan { RowProg ln_load; Copy gather; TableRegion tables; };
struct EmbedPlan { RowProg a_rows, a_cols; Copy unfold; TableRegion tables; };
std::map<Key, std::shared_ptr<MergePlan>> g_merge;
std::map<Key, std::shared_ptr<EmbedPlan>> g_embed;

std::shared_ptr<MergePlan> merge_plan(int B, int H, int W, int C, int dtype, std::string* err) {
  Key key{{B, H, W, C, dtype, 0, 0, 1}};
  std::lock_guard<std::mutex> lock(g_mu);
  auto it = g_merge.find(key);
  if (it != g_merge.end()) return it->second;
  auto p = std::make_shared<MergePlan>();
  // LayerNorm's load absorbs the 2x2 gather: a logical row of 4C is four segments of C
  std::vector<sm_view_op> ch = chains::patch_merge(B, H, W, C);
  ch.push_back(chains::reshape({(int64_t)B * (H / 2) * (W / 2) * 4, C}));
  if (!make_rows({B, H, W, C}, ch, &p->tables, &p->ln_load, err)) return nullptr;
  if (!make_copy({B, H, W, C}, chains::patch_merge(B, H, W, C), (int)dtype_size(dtype), &p->tables, &p->gather, err)) return nullptr;
  bound_cache(g_merge);
  g_merge[key] = p;
  return p;
}

std::shared_ptr<EmbedPlan> embed_plan(int B, int Cin, int img, int patch, int dtype, std::string* err) {
  Key key{{B, Cin, img, patch, dtype, 0, 0, 2}};
  std::lock_guard<std::mutex> lock(g_mu);
  auto it = g_embed.find(key);
  if (it != g_embed.end()) return it->second;
  auto p = std::make_shared<EmbedPlan>();
  sm_map* m = nullptr;
  std::vector<sm_view_op> ch = chains::patch_embed(B, Cin, img, img, patch);
  if (map_create({B, Cin, img, img}, ch.data(), (int)ch.size(), &m, err) != SM_OK) return nullptr;
  bool ok = m->compile_rows_cols(4, &p->a_rows, &p->a_cols, err);
  const int64_t kk = m->shape.back(), src_numel = (int64_t)B * Cin * img * img;
  if (ok) { p->tables.add(&p->a_rows, m->numel() / kk, src_numel); p->tables.add(&p->a_cols, kk / 4, src_numel); }
  delete m;
  ok = ok && make_copy({B, Cin, img, img}, ch, (int)dtype_size(dtype), &p->tables, &p->unfold, err);
  if (!ok) return nullptr;
  bound_cache(g_embed);
  g_embed[key] = p;
  return p;
}

int check_chain(const sm_chain_desc* c, const char* who) {
  if (!c) return fail(SM_ERR_INVALID_ARG, "%s: null descriptor", who);
  if (!dtype_ok(c->dtype)) return fail(SM_ERR_INVALID_ARG, "%s: unknown dtype", who);
  if (c->B < 1 || c->n_stages < 1 || c->n_stages > 4 || c->window < 1 || c->mlp_ratio < 1) return fail(SM_ERR_SHAPE, "%s: bad descriptor", who);
  for (int s = 0; s < c->n_stages; ++s) {
    const sm_stage_desc& st = c->stages[s];
    sm_swin_cfg bc{c->B, st.H, st.W, st.C, st.heads, c->window, 0, c->mlp_ratio, c->dtype, c->eps};
    int rc = check_swin(&bc, who);
    if (rc) return rc;
    if (st.depth < 1) return fail(SM_ERR_SHAPE, "%s: stage %d has no blocks", who, s);
    if (s > 0) {
      const sm_stage_desc& pr = c->stages[s - 1];
      if (pr.H % 2 || pr.W % 2 || st.H != pr.H / 2 || st.W != pr.W / 2 || st.C != 2 * pr.C)
        return fail(SM_ERR_SHAPE, "%s: stage %d does not follow a 2x2 patch merge of stage %d", who, s, s - 1);
    }
  }
  if (c->has_embed) {
    if (c->patch != 4) return fail(SM_ERR_UNSUPPORTED, "%s: patch size must be 4", who);
    if (c->img % c->patch || c->img / c->patch != c->stages[0].H || c->stages[0].H != c->stages[0].W)
      return fail(SM_ERR_SHAPE, "%s: image / patch does not match stage 0", who);
    if (c->in_ch < 1) return fail(SM_ERR_SHAPE, "%s: in_ch", who);
  }
  if (c->has_head && c->n_cls < 1) return fail(SM_ERR_SHAPE, "%s: n_cls", who);
  return SM_OK;
}

int chain_weight_count(const sm_chain_desc* c) {
  int n = c->has_embed ? 4 : 0;
  for (int s = 0; s < c->n_stages; ++s) n += 16 * c->stages[s].depth + (s + 1 < c->n_stages ? 3 : 0);
  return n + (c->has_head ? 4 : 0);
}

// Everything a chain call needs to know before its first launch: the plans of every stage (host objects) and where
// each plan's row-offset tables lie in the workspace: [block buffers | activation ping | pong | table regions ...]
struct ChainLayout {
  size_t act = 0, block = 0, total = 0;
  std::shared_ptr<EmbedPlan> embed; size_t embed_off = 0;
  struct Stage {
    std::shared_ptr<SwinPlan> plan[2]; size_t plan_off[2];       // [0] blocks without shift, [1] shifted blocks (if any)
    std::shared_ptr<NextStore> next[2]; size_t next_off[2];      // elided: store of the block after a [0] / [1] block
    std::shared_ptr<MergePlan> merge; size_t merge_off;
  };
  std::vector<Stage> stages;
};
int shift_of(const sm_chain_desc* c, const sm_stage_desc& st, int k) { return (k % 2 == 1 && std::min(st.H, st.W) > c->window) ? c->window / 2 : 0; }

bool chain_layout(const sm_chain_desc* c, int mode, ChainLayout* L, std::string* err) {
  const int dt = c->dtype;
  for (int s = 0; s < c->n_stages; ++s) {
    const sm_stage_desc& st = c->stages[s];
    sm_swin_cfg bc{c->B, st.H, st.W, st.C, st.heads, c->window, 0, c->mlp_ratio, dt, c->eps};
    L->block = std::max(L->block, swin_act_bytes(&bc, mode));
    L->act = std::max(L->act, align256((size_t)c->B * st.H * st.W * st.C * dtype_size(dt)));
  }
  size_t at = L->block + 2 * L->act;
  if (c->has_embed) {
    if (!(L->embed = embed_plan(c->B, c->in_ch, c->img, c->patch, dt, err))) return false;
    L->embed_off = at; at += L->embed->tables.bytes;
  }
  L->stages.resize((size_t)c->n_stages);
  for (int s = 0; s < c->n_stages; ++s) {
    const sm_stage_desc& st = c->stages[s];
    ChainLayout::Stage& S = L->stages[(size_t)s];
    const bool shifts = st.depth > 1 && shift_of(c, st, 1) != 0;
    for (int sh = 0; sh < (shifts ? 2 : 1); ++sh) {
      sm_swin_cfg bc{c->B, st.H, st.W, st.C, st.heads, c->window, sh ? c->window / 2 : 0, c->mlp_ratio, dt, c->eps};
      if (!(S.plan[sh] = swin_plan(bc, err))) return false;
      S.plan_off[sh] = at; at += S.plan[sh]->tables(mode).bytes;
      if (mode == SM_ELIDED && st.depth > 1) {
        const int nshift = shifts && !sh ? c->window / 2 : 0;
        if (!(S.next[sh] = next_norm_store(bc, nshift, err))) return false;
        S.next_off[sh] = at; at += S.next[sh]->tables.bytes;
      }
    }
    if (s + 1 < c->n_stages) {
      if (!(S.merge = merge_plan(c->B, st.H, st.W, st.C, dt, err))) return false;
      S.merge_off = at; at += S.merge->tables.bytes;
    }
  }
  L->total = at;
  return true;
}

}  // namespace

extern "C" size_t sm_run_chain_workspace_bytes(const sm_chain_desc* c, int mode) {
  if (check_chain(c, "sm_run_chain_workspace_bytes") != SM_OK) return 0;
  if (mode != SM_ELIDED && mode != SM_EXPLICIT) { set_error("sm_run_chain_workspace_bytes: unknown mode %d", mode); return 0; }
  ChainLayout L; std::string err;
  if (!chain_layout(c, mode, &L, &err)) { set_error("sm_run_chain_workspace_bytes: %s", err.c_str()); return 0; }
  return L.total;
}

extern "C" int sm_run_chain(const sm_chain_desc* c, const void* const* weights, int n_weights, const void* x,
                            void* y, void* y_feat, void* ws, size_t ws_bytes, int mode, void* stream) {
  int rc = check_chain(c, "sm_run_chain");
  if (rc) return rc;
  if (!weights || !x || !y || !ws) return fail(SM_ERR_INVALID_ARG, "sm_run_chain: null pointer");
  if (mode != SM_ELIDED && mode != SM_EXPLICIT) return fail(SM_ERR_INVALID_ARG, "sm_run_chain: unknown mode %d", mode);
  if (n_weights != chain_weight_count(c)) return fail(SM_ERR_INVALID_ARG, "sm_run_chain: %d weight pointers given, %d expected", n_weights, chain_weight_count(c));
  {
    // every pointer is required except a block's last three (the packed MLP, projection and QKV weights)
    std::vector<char> optional((size_t)n_weights, 0);
    int at = c->has_embed ? 4 : 0;
    for (int s = 0; s < c->n_stages; ++s) {
      for (int k = 0; k < c->stages[s].depth; ++k) { optional[(size_t)at + 13] = optional[(size_t)at + 14] = optional[(size_t)at + 15] = 1; at += 16; }
      if (s + 1 < c->n_stages) at += 3;
    }
    for (int i = 0; i < n_weights; ++i)
      if ((!weights[i] && !optional[(size_t)i]) || !aligned16(weights[i]))
        return fail(SM_ERR_INVALID_ARG, "sm_run_chain: weight %d is null or misaligned", i);
  }
  // build every plan before the first launch so that an unsupported shape enqueues nothing
  ChainLayout z; std::string err;
  if (!chain_layout(c, mode, &z, &err)) return fail(SM_ERR_UNSUPPORTED, "sm_run_chain: %s", err.c_str());
  if (ws_bytes < z.total) return fail(SM_ERR_WORKSPACE, "sm_run_chain: workspace of %zu bytes, %zu needed", ws_bytes, z.total);
  if (!aligned16(x) || !aligned16(y) || !aligned16(ws) || (y_feat && !aligned16(y_feat))) return fail(SM_ERR_INVALID_ARG, "sm_run_chain: pointers must be 16-byte aligned");
  const int dt = c->dtype;
  // first pass, no launches: what each block hands to the next one, hence which tables are read at all
  struct BlockStep { bool next; bool next_qkv; int pre; };
  std::vector<std::vector<BlockStep>> steps((size_t)c->n_stages);
  std::vector<uint64_t> need[2];
  need[0].assign((size_t)c->n_stages, 0); need[1].assign((size_t)c->n_stages, 0);
  std::vector<char> need_next[2];
  need_next[0].assign((size_t)c->n_stages, 0); need_next[1].assign((size_t)c->n_stages, 0);
  {
    const void* const* wq = weights + (c->has_embed ? 4 : 0);
    for (int s = 0; s < c->n_stages; ++s) {
      const sm_stage_desc& st = c->stages[s];
      int pre = 0;
      for (int k = 0; k < st.depth; ++k) {
        const int shift = shift_of(c, st, k), sh = shift ? 1 : 0;
        sm_swin_cfg bc{c->B, st.H, st.W, st.C, st.heads, c->window, shift, c->mlp_ratio, dt, c->eps};
        sm_swin_weights bw, nwt;
        std::memcpy(&bw, wq, sizeof(bw));
        wq += 16;
        BlockStep b{false, false, pre};
        // within a stage, elided, with the projection + MLP kernel: that kernel also writes the next block's
        // LayerNorm-1 (through the next block's own partition map) or its QKV, and the next block starts there
        // (where LayerNorm-1 is folded into the QKV Linear's load, C <= 170, only the norm + QKV form applies)
        if (mode == SM_ELIDED && k + 1 < st.depth && proj_is_fused(bc, &bw)) {
          std::memcpy(&nwt, wq, sizeof(nwt));
          const bool with_qkv = nwt.qkv_packed && c->mlp_ratio >= 3;    // (the kernel keeps the QKV bias where the first MLP bias was)
          if (!fold_norm(3 * st.C) || with_qkv) { b.next = true; b.next_qkv = with_qkv; }
        }
        need[sh][(size_t)s] |= mode == SM_ELIDED ? el_tables_needed(bc, &bw, pre) : ~0ull;
        if (b.next) need_next[sh][(size_t)s] = 1;
        pre = b.next ? (b.next_qkv ? 2 : 1) : 0;
        steps[(size_t)s].push_back(b);
      }
      if (s + 1 < c->n_stages) wq += 3;
    }
  }
  char* base = (char*)ws;
  count_reset();
  // the row-offset tables of every map the chain reads, before its first kernel
  TableFiller filler(stream);
  if (z.embed && (rc = filler.add(z.embed->tables, base + z.embed_off, mode == SM_ELIDED ? 3ull : ~3ull))) return rc;   // A rows + columns | the unfold copy
  for (int s = 0; s < c->n_stages; ++s) {
    const ChainLayout::Stage& S = z.stages[(size_t)s];
    for (int sh = 0; sh < 2; ++sh) {
      if (S.plan[sh] && need[sh][(size_t)s] && (rc = filler.add(S.plan[sh]->tables(mode), base + S.plan_off[sh], need[sh][(size_t)s]))) return rc;
      if (S.next[sh] && need_next[sh][(size_t)s] && (rc = filler.add(S.next[sh]->tables, base + S.next_off[sh], ~0ull))) return rc;
    }
    if (S.merge && (rc = filler.add(S.merge->tables, base + S.merge_off, mode == SM_ELIDED ? 1ull : ~1ull))) return rc;      // LayerNorm's gather | the copy
  }
  if ((rc = filler.flush())) return rc;
  void* blk_ws = base;
  void* act[2] = {base + z.block, base + z.block + z.act};
  int n_compute = 0, n_copy = 0;
  auto tally = [&]() { int a, b; counts(&a, &b); n_compute += a; n_copy += b; count_reset(); };
  const void* const* wp = weights;
  const void* cur = x;
  int flip = 0;
  if (c->has_embed) {
    const sm_stage_desc& st = c->stages[0];
    const int64_t T = (int64_t)c->B * st.H * st.W;
    const int K = c->in_ch * c->patch * c->patch;
    void* tmp = blk_ws;
    if (mode == SM_ELIDED) {
      GemmArgs g; std::memset(&g, 0, sizeof(g));
      g.A = x; g.W = wp[0]; g.bias = wp[1]; g.C = tmp; g.M = T; g.N = st.C; g.K = K; g.dtype = dt; g.ldw = K;
      const void* tb = base + z.embed_off;
      g.a_rows = bound(z.embed->a_rows, tb); g.a_cols = bound(z.embed->a_cols, tb); g.a_gran = 4; g.c_rows = identity_rows(st.C);
      if ((rc = gemm_checked(g, stream, "patch embedding"))) return rc;
    } else {
      void* unf = (char*)blk_ws + align256((size_t)T * st.C * dtype_size(dt));
      if ((rc = copy_launch(z.embed->unfold, base + z.embed_off, x, unf, dt, stream))) return rc;
      if ((rc = run_gemm(unf, wp[0], wp[1], nullptr, tmp, T, st.C, K, dt, SM_ACT_NONE, nullptr, nullptr, stream))) return rc;
    }
    if ((rc = run_norm(tmp, wp[2], wp[3], act[flip], T, st.C, c->eps, 0, dt, nullptr, 1, nullptr, stream))) return rc;
    cur = act[flip]; flip ^= 1;
    wp += 4;
    tally();
  }
  for (int s = 0; s < c->n_stages; ++s) {
    const sm_stage_desc& st = c->stages[s];
    const bool last_stage = s + 1 == c->n_stages;
    const ChainLayout::Stage& S = z.stages[(size_t)s];
    for (int k = 0; k < st.depth; ++k) {
      const int shift = shift_of(c, st, k), sh = shift ? 1 : 0;
      const BlockStep& step = steps[(size_t)s][(size_t)k];
      sm_swin_cfg bc{c->B, st.H, st.W, st.C, st.heads, c->window, shift, c->mlp_ratio, dt, c->eps};
      sm_swin_weights bw;
      std::memcpy(&bw, wp, sizeof(bw));
      wp += 16;
      const bool final_out = last_stage && k + 1 == st.depth && !c->has_head;
      void* out = final_out ? y : act[flip];
      NextNorm nn; const NextNorm* next = nullptr;
      if (step.next) {
        sm_swin_weights nw;
        std::memcpy(&nw, wp, sizeof(nw));
        nn.gamma = nw.ln1_g; nn.beta = nw.ln1_b; nn.store = bound(S.next[sh]->rows, base + S.next_off[sh]);
        nn.wq_p = step.next_qkv ? nw.qkv_packed : nullptr; nn.bq = nw.bqkv;
        next = &nn;
      }
      if ((rc = swin_block_impl(&bc, &bw, cur, out, blk_ws, z.block, mode, stream, next, step.pre, base + S.plan_off[sh]))) return rc;
      tally();
      cur = out; flip ^= 1;
    }
    if (!last_stage) {
      const int64_t T4 = (int64_t)c->B * (st.H / 2) * (st.W / 2);
      void* normed = blk_ws;
      const RowProg merge_load = bound(S.merge->ln_load, base + S.merge_off);
      if (mode == SM_ELIDED) {
        if ((rc = run_norm(cur, wp[0], wp[1], normed, T4, 4 * st.C, c->eps, 0, dt, &merge_load, 4, nullptr, stream))) return rc;
      } else {
        void* gathered = (char*)blk_ws + align256((size_t)T4 * 4 * st.C * dtype_size(dt));
        if ((rc = copy_launch(S.merge->gather, base + S.merge_off, cur, gathered, dt, stream))) return rc;
        if ((rc = run_norm(gathered, wp[0], wp[1], normed, T4, 4 * st.C, c->eps, 0, dt, nullptr, 1, nullptr, stream))) return rc;
      }
      if ((rc = run_gemm(normed, wp[2], nullptr, nullptr, act[flip], T4, 2 * st.C, 4 * st.C, dt, SM_ACT_NONE, nullptr, nullptr, stream))) return rc;
      cur = act[flip]; flip ^= 1;
      wp += 3;
      tally();
    }
  }
  if (c->has_head) {
    const sm_stage_desc& st = c->stages[c->n_stages - 1];
    const int L = st.H * st.W;
    void* feat = y_feat ? y_feat : act[flip];
    if ((rc = run_norm(cur, wp[0], wp[1], feat, (int64_t)c->B * L, st.C, c->eps, 0, dt, nullptr, 1, nullptr, stream))) return rc;
    void* pooled = blk_ws;
    int lrc;
    char label[64];
    snprintf(label, sizeof(label), "mean_tokens_%s[%d,%d,%d]", dt == SM_F32 ? "f32" : "bf16", c->B, L, st.C);
    { Timed tm(label, stream); lrc = launch_mean_tokens(feat, pooled, c->B, L, st.C, dt, stream); }
    if (lrc) return fail(SM_ERR_DEVICE, "sm_run_chain: mean launch failed (hip error %d)", lrc);
    count_compute();
    if ((rc = run_gemm(pooled, wp[2], wp[3], nullptr, y, c->B, c->n_cls, st.C, dt, SM_ACT_NONE, nullptr, nullptr, stream))) return rc;
    tally();
  }
  count_reset(); count_compute(n_compute); count_copy(n_copy);
  return SM_OK;
}
