// sm_decode_step: a GPT-NeoX / Pythia-style layer at a decode step (one new token per sequence against a key /
// value cache; the decoder-only workload of the paper's Table 7 at its memory-bound end), elided and explicit.
//
// The step is written down as the exporter's operator graph and planned (Sec. 3.2): the query / key / value Slices
// and Permutes and the head merge are eliminated (the query is read in place from the stored [B, h, 3, d] result of
// the fused Linear, the attention output is stored merged).  The Concat that puts the new key / value row behind the
// cached ones has two inputs and is outside the planner; it is eliminated by the same rule applied by hand (the
// producer writes the layout the consumer reads, Sec. 3.2.2): the cache buffer has room for the new row, and the
// Linear that produces it stores it at position L.  In explicit mode every one of these operators is a copy kernel,
// the Concat included (it rewrites the whole cache).
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

namespace sm { int decode_attn_block(int d); int decode_counter_stride(); size_t decode_out_smem(int B, int E, int F, int nks); }      // keys of one block of the attention kernel (k_decode.hip)

namespace {

struct DecodePlan {
  View4 q, o;                      // query operand and attention output as [B, h, 1, d] views of qkv [B, 3E] and o [B, E]
  Copy split[3], merge;            // explicit chain: Slice + Permute of q, k, v; Permute + Reshape of the attention output
  TableRegion ex_tables;
  int n_layout, n_eliminated, n_kept;
};

struct Key { int v[6]; bool operator<(const Key& o) const { return std::memcmp(v, o.v, sizeof(v)) < 0; } };
std::mutex g_mu;
std::map<Key, std::shared_ptr<DecodePlan>> g_plans;

std::shared_ptr<DecodePlan> decode_plan(const sm_decode_cfg& c, std::string* err) {
  Key key{{c.B, c.E, c.heads, c.F, c.L, c.dtype}};
  std::lock_guard<std::mutex> lock(g_mu);
  auto it = g_plans.find(key);
  if (it != g_plans.end()) return it->second;
  auto p = std::make_shared<DecodePlan>();
  const int64_t B = c.B, E = c.E, h = c.heads, d = E / h, F = c.F, L = c.L;
  GraphB g;
  const int x = g.tensor({B, 1, E});
  const int Kfull = g.tensor({B, h, L + 1, d}), Vfull = g.tensor({B, h, L + 1, d});     // the caches with the new row appended
  int t = g.op(SM_OP_LAYERNORM, {x}, {B, 1, E}, "ln1", {2});
  const int qkv = g.reshape(g.linear(t, 3 * E, "qkv", true), {B, 1, h, 3 * d});
  int part[3];
  for (int k = 0; k < 3; ++k) {
    part[k] = g.transpose(g.slice(qkv, 3, k * d, (k + 1) * d), {0, 2, 1, 3});
    if (k < 2) part[k] = g.op(SM_OP_ROPE, {part[k]}, {B, h, 1, d}, "rope");
  }
  t = g.op(SM_OP_ATTENTION, {part[0], Kfull, Vfull}, {B, h, 1, d}, "attn", {3, 3, -1});
  t = g.reshape(g.transpose(t, {0, 2, 1, 3}), {B, 1, E});
  t = g.linear(t, E, "dense", true);
  const int r1 = g.op(SM_OP_ADD, {x, t}, {B, 1, E}, "res1");
  t = g.op(SM_OP_LAYERNORM, {x}, {B, 1, E}, "ln2", {2});
  t = g.linear(t, F, "fc1", true);
  t = g.op(SM_OP_UNARY, {t}, {B, 1, F}, "gelu");
  t = g.linear(t, E, "fc2", true);
  g.op(SM_OP_ADD, {r1, t}, {B, 1, E}, "res2");
  sm_plan* plan = nullptr;
  if (sm_layout_plan(g.tensors.data(), (int)g.tensors.size(), g.ops.data(), (int)g.ops.size(), 1, &plan) != SM_OK) { *err = sm_last_error(); return nullptr; }
  std::unique_ptr<sm_plan, void (*)(sm_plan*)> guard(plan, sm_plan_destroy);
  p->n_kept = p->n_layout = p->n_eliminated = 0;
  for (int i = 0; i < (int)g.ops.size(); ++i) {
    int grp, st;
    sm_plan_op(plan, i, &grp, nullptr, &st, nullptr, nullptr);
    p->n_kept += st == SM_KEPT;
    if (grp == SM_ILD_FIX || grp == SM_ILI_FIX) { ++p->n_layout; p->n_eliminated += (st == SM_ELIMINATED_STORE || st == SM_ELIMINATED_LOAD); }
  }
  // LayerNorm x 2, the four Linears and attention survive; every Reshape / Slice / Transpose is an address
  if (p->n_eliminated != p->n_layout || p->n_kept != 7) { *err = "planner did not reduce the decode step to its compute operators"; return nullptr; }
  const int attn = g.find("attn");
  if (!plan_operand_view(plan, g, attn, 0, &p->q, err) || !plan_output_view(plan, g, attn, &p->o, err)) return nullptr;
  const int es = (int)dtype_size(c.dtype);
  for (int k = 0; k < 3; ++k) {
    std::vector<sm_view_op> ch{chains::reshape({B, 1, h, 3 * d}), chains::slice(3, k * d, (k + 1) * d), chains::permute({0, 2, 1, 3})};
    if (!make_copy({B, 1, 3 * E}, ch, es, &p->ex_tables, &p->split[k], err)) return nullptr;
  }
  if (!make_copy({B, h, 1, d}, chains::head_merge(B, 1, h, d), es, &p->ex_tables, &p->merge, err)) return nullptr;
  if (g_plans.size() >= 64) g_plans.clear();
  g_plans[key] = p;
  return p;
}

int check_cfg(const sm_decode_cfg* c, const char* who) {
  if (!c) return fail(SM_ERR_INVALID_ARG, "%s: null configuration", who);
  if (c->dtype != SM_BF16) return fail(SM_ERR_UNSUPPORTED, "%s: bf16 only", who);
  if (c->B < 1 || c->B > 32) return fail(SM_ERR_SHAPE, "%s: 1 to 32 sequences per step", who);
  if (c->E < 64 || c->E % 64 || c->E > 8192 || c->heads < 1 || c->E % c->heads) return fail(SM_ERR_SHAPE, "%s: hidden size must be a multiple of 64 (at most 8192) and of the head count", who);
  const int d = c->E / c->heads;
  if (d != 64 && d != 128 && d != 256) return fail(SM_ERR_SHAPE, "%s: head size must be 64, 128 or 256", who);
  if (c->F < 64 || c->F % 64) return fail(SM_ERR_SHAPE, "%s: MLP width must be a multiple of 64", who);
  if (c->rot != 0 && c->rot != 32 && c->rot != 64) return fail(SM_ERR_SHAPE, "%s: rotary features must be 0, 32 or 64", who);
  if (c->L < 0 || c->cache_pitch < c->L) return fail(SM_ERR_SHAPE, "%s: the cache pitch must cover the cached tokens", who);
  if (decode_in_smem(c->B, c->E) > 160 * 1024) return fail(SM_ERR_SHAPE, "%s: B x E too large for the LDS token tile", who);
  if (decode_out_smem(c->B, c->E, c->F, 64) > 48 * 1024) return fail(SM_ERR_SHAPE, "%s: B x (E + F) too large for the last kernel's LDS tile", who);
  return SM_OK;
}

size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }
int attn_splits(const sm_decode_cfg& c) {
  // about two workgroups per CU, each with at least two blocks of keys
  const int bh = c.B * c.heads, block = decode_attn_block(c.E / c.heads), blocks = (c.L + 1 + block - 1) / block;
  int s = (512 + bh - 1) / bh;
  s = std::min(s, std::max(1, blocks / 2));
  return std::max(1, std::min(s, 256));
}
int out_splits(const sm_decode_cfg& c) {
  const int slices = c.E / 32, steps = (c.E + c.F) / 16;
  int s = (256 + slices - 1) / slices;
  s = std::min(s, std::max(1, steps / 32));          // at least 16 steps per wave
  s = std::max(2, std::min(s, 64));                  // at least one split for each of the two matrices
  while (s < 64 && decode_out_smem(c.B, c.E, c.F, s) > 48 * 1024) ++s;      // a split's activation rows must fit its LDS tile
  return s;
}

struct Sizes { size_t qkv, hid, o, part_a, part_o, counters, small, total; };
Sizes sizes(const sm_decode_cfg& c, int mode) {
  Sizes z;
  const size_t B = c.B, E = c.E, h = c.heads, d = E / h;
  z.qkv = align256(B * 3 * E * 2);
  z.hid = align256(B * c.F * 2);
  z.o = align256(B * E * 2);
  z.part_a = align256(B * h * attn_splits(c) * (d + 2) * sizeof(float));
  z.part_o = align256((size_t)out_splits(c) * B * E * sizeof(float));
  z.counters = align256((B * h + E / 32) * decode_counter_stride() * sizeof(int));
  z.small = mode == SM_EXPLICIT ? 5 * z.o : 0;       // q, new k, new v, unmerged output, spare
  z.total = z.qkv + z.hid + z.o + z.part_a + z.part_o + z.counters + z.small;
  return z;
}

}  // namespace

extern "C" size_t sm_decode_step_workspace_bytes(const sm_decode_cfg* c, int mode) {
  if (check_cfg(c, "sm_decode_step_workspace_bytes") != SM_OK) return 0;
  if (mode != SM_ELIDED && mode != SM_EXPLICIT) { set_error("sm_decode_step_workspace_bytes: unknown mode %d", mode); return 0; }
  std::string err;
  auto plan = decode_plan(*c, &err);
  if (!plan) { set_error("sm_decode_step_workspace_bytes: %s", err.c_str()); return 0; }
  return sizes(*c, mode).total + (mode == SM_EXPLICIT ? plan->ex_tables.bytes : 0);
}

extern "C" int sm_decode_step(const sm_decode_cfg* c, const sm_decode_weights* w, const void* x, void* k_cache, void* v_cache,
                              void* y, void* k_out, void* v_out, void* ws, size_t ws_bytes, int mode, void* stream) {
  int rc = check_cfg(c, "sm_decode_step");
  if (rc) return rc;
  if (mode != SM_ELIDED && mode != SM_EXPLICIT) return fail(SM_ERR_INVALID_ARG, "sm_decode_step: unknown mode %d", mode);
  if (!w || !x || !y || !ws || !k_cache || !v_cache) return fail(SM_ERR_INVALID_ARG, "sm_decode_step: null pointer");
  const void* wp[12] = {w->ln1_g, w->ln1_b, w->wqkv_p, w->bqkv, w->wdense_p, w->bdense, w->ln2_g, w->ln2_b, w->w1_p, w->b1, w->w2_p, w->b2};
  for (int i = 0; i < 12; ++i) if (!wp[i] || !aligned16(wp[i])) return fail(SM_ERR_INVALID_ARG, "sm_decode_step: weight %d is null or misaligned", i);
  if (!aligned16(x) || !aligned16(y) || !aligned16(ws) || !aligned16(k_cache) || !aligned16(v_cache)) return fail(SM_ERR_INVALID_ARG, "sm_decode_step: pointers must be 16-byte aligned");
  const bool el = mode == SM_ELIDED;
  if (el && c->cache_pitch <= c->L) return fail(SM_ERR_SHAPE, "sm_decode_step: elided mode appends in place: the cache needs room for token %d (pitch %d)", c->L, c->cache_pitch);
  if (!el && (!k_out || !v_out || !aligned16(k_out) || !aligned16(v_out))) return fail(SM_ERR_INVALID_ARG, "sm_decode_step: explicit mode writes the grown caches to k_out / v_out");
  std::string err;
  auto plan = decode_plan(*c, &err);
  if (!plan) return fail(SM_ERR_UNSUPPORTED, "sm_decode_step: %s", err.c_str());
  const Sizes z = sizes(*c, mode);
  const size_t need = z.total + (el ? 0 : plan->ex_tables.bytes);
  if (ws_bytes < need) return fail(SM_ERR_WORKSPACE, "sm_decode_step: workspace of %zu bytes, %zu needed", ws_bytes, need);
  count_reset();
  const int B = c->B, E = c->E, h = c->heads, d = E / h, F = c->F, L = c->L;
  char* base = (char*)ws;
  unsigned short* qkv = (unsigned short*)base; base += z.qkv;
  unsigned short* hid = (unsigned short*)base; base += z.hid;
  unsigned short* o = (unsigned short*)base; base += z.o;
  float* part_a = (float*)base; base += z.part_a;
  float* part_o = (float*)base; base += z.part_o;
  int* counters = (int*)base; base += z.counters;
  char* small = base; base += z.small;
  const void* tables = base;
  if (!el && (rc = fill_tables(plan->ex_tables, base, stream, ~0ull))) return rc;
  const int64_t cache_bh = (int64_t)c->cache_pitch * d;
  char label[96];

  DecodeInArgs a; std::memset(&a, 0, sizeof(a));
  a.x = (const unsigned short*)x;
  a.ln1_g = (const unsigned short*)w->ln1_g; a.ln1_b = (const unsigned short*)w->ln1_b;
  a.ln2_g = (const unsigned short*)w->ln2_g; a.ln2_b = (const unsigned short*)w->ln2_b; a.eps = c->eps;
  a.wqkv_p_ = w->wqkv_p; a.w1_p_ = w->w1_p; a.bqkv = (const unsigned short*)w->bqkv; a.b1 = (const unsigned short*)w->b1;
  a.B = B; a.E = E; a.h = h; a.d = d; a.F = F; a.rot = c->rot; a.L = L; a.rope_base = c->rope_base;
  a.hid = hid; a.counters = counters; a.n_counters = B * h + E / 32;
  // the fused Linear's result [B, h, 3, d] in its natural layout ...
  for (int t = 0; t < 3; ++t) { a.dst[t] = qkv + t * d; a.dst_b[t] = 3 * E; a.dst_h[t] = 3 * d; }
  if (el) {        // ... except that the new key / value rows go where the Concat would have put them
    a.dst[1] = (unsigned short*)k_cache + (int64_t)L * d; a.dst[2] = (unsigned short*)v_cache + (int64_t)L * d;
    a.dst_b[1] = a.dst_b[2] = (int64_t)h * cache_bh; a.dst_h[1] = a.dst_h[2] = cache_bh;
  }
  {
    snprintf(label, sizeof(label), "decode_ln+qkv+rope|ln+fc1+gelu_bf16[%d,%d,%d]", B, 3 * E + F, E);
    Timed tm(label, stream);
    if (int e = launch_decode_in(a, stream)) return fail(SM_ERR_DEVICE, "sm_decode_step: first kernel launch failed (hip error %d)", e);
    count_compute();
  }

  DecodeAttnArgs t; std::memset(&t, 0, sizeof(t));
  t.part = part_a; t.counters = counters; t.B = B; t.h = h; t.d = d; t.n_keys = L + 1;
  t.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)d));
  void* o_final = o;
  if (el) {
    // query in place in the stored qkv tensor (planned load map), caches in place, output stored merged (planned store map)
    t.q = qkv + plan->q.base; t.q_b = plan->q.stride[0]; t.q_h = plan->q.stride[1];
    t.K = (const unsigned short*)k_cache; t.V = (const unsigned short*)v_cache; t.kv_b = (int64_t)h * cache_bh; t.kv_h = cache_bh;
    t.o = o + plan->o.base; t.o_b = plan->o.stride[0]; t.o_h = plan->o.stride[1];
  } else {
    unsigned short* qc = (unsigned short*)small; unsigned short* kn = (unsigned short*)(small + z.o); unsigned short* vn = (unsigned short*)(small + 2 * z.o);
    unsigned short* ou = (unsigned short*)(small + 3 * z.o);
    unsigned short* parts[3] = {qc, kn, vn};
    for (int k = 0; k < 3; ++k) if ((rc = copy_launch(plan->split[k], tables, qkv, parts[k], c->dtype, stream))) return rc;
    const void* fresh[2] = {kn, vn}; const void* cache[2] = {k_cache, v_cache}; void* grown[2] = {k_out, v_out};
    for (int k = 0; k < 2; ++k) {
      snprintf(label, sizeof(label), "concat_bf16[%d,%d,%d]", B * h, L + 1, d);
      Timed tm(label, stream);
      if (int e = launch_decode_concat(cache[k], cache_bh, fresh[k], grown[k], B * h, L, d, stream)) return fail(SM_ERR_DEVICE, "sm_decode_step: concat launch failed (hip error %d)", e);
      count_copy();
    }
    t.q = qc; t.q_b = E; t.q_h = d;
    t.K = (const unsigned short*)k_out; t.V = (const unsigned short*)v_out; t.kv_h = (int64_t)(L + 1) * d; t.kv_b = (int64_t)h * t.kv_h;
    t.o = ou; t.o_b = E; t.o_h = d;
  }
  {
    snprintf(label, sizeof(label), "decode_attention_bf16[%d,%d,%d,%d]", B, h, L + 1, d);
    Timed tm(label, stream);
    if (int e = launch_decode_attn(t, attn_splits(*c), stream)) return fail(SM_ERR_DEVICE, "sm_decode_step: attention launch failed (hip error %d)", e);
    count_compute();
  }
  if (!el) { if ((rc = copy_launch(plan->merge, tables, small + 3 * z.o, o_final, c->dtype, stream))) return rc; }

  DecodeOutArgs u; std::memset(&u, 0, sizeof(u));
  u.o = o; u.hid = hid; u.x = (const unsigned short*)x; u.y = (unsigned short*)y;
  u.wdense_p_ = w->wdense_p; u.w2_p_ = w->w2_p; u.bdense = (const unsigned short*)w->bdense; u.b2 = (const unsigned short*)w->b2;
  u.part = part_o; u.counters = counters + (size_t)B * h * decode_counter_stride(); u.B = B; u.E = E; u.F = F;
  {
    snprintf(label, sizeof(label), "decode_dense+fc2+res_bf16[%d,%d,%d]", B, E, E + F);
    Timed tm(label, stream);
    if (int e = launch_decode_out(u, out_splits(*c), stream)) return fail(SM_ERR_DEVICE, "sm_decode_step: last kernel launch failed (hip error %d)", e);
    count_compute();
  }
  return SM_OK;
}
