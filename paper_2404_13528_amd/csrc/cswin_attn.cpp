// sm_cswin_attention: cross-shaped window self-attention of the CSwin Transformer (Table 1 counts its Reshape /
// Transpose operators, Table 7 evaluates it), elided and explicit.
//
// The operator is written down as the exporter's graph and planned (Sec. 3.2): per half of the channels, the Slices
// that take q, k, v out of the fused projection, the stripe partition (Transpose, Reshape, Transpose, Reshape), the
// head split, and after the attention the head merge and the stripe merge.  The plan eliminates every one of them;
// what remains are two attention operators whose load and store maps are strided in the factored index
// (image, stripe, head, run, token in run, feature): the executor asks the composer for exactly that factoring and
// hands the strides to the attention kernel.  The Concat that joins the two halves has two inputs and is outside the
// planner; it is eliminated by the same rule applied by hand (the producer stores the layout the consumer reads,
// Sec. 3.2.2): each attention stores into its half of the output's channels.  In explicit mode every run of layout
// operators is a copy kernel, the Concat included.
//
// With the locally-enhanced positional encoding the graph has, per half, a depth-wise convolution of the values laid
// out as stripe images and an Add of its result to the attention output.  The plan keeps the convolution, fuses the Add
// into the attention and eliminates the Reshapes / Transposes on both sides of the convolution.  The convolution
// kernel reads the values in place (its planned load map is checked against the kernel's token-major addressing when
// the plan is built) and writes where the sum will finally live, in the output's layout; the attention then adds to
// what it finds there.  In the elided chain the two halves share one launch of each kernel (the attentions only when
// both halves have one shape, i.e. on square grids): these kernels are short, and a launch costs as much as their work.
//
// sm_cswin_block (below) puts the block's other operators around it: they have no layout operator between them.
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

using namespace sm;

namespace {

// element strides of an attention operand in the factored index (image, stripe, head, run, token in run, feature)
struct Strides6 { int64_t base, img, stripe, head, runs, tok; };
struct Branch {
  int64_t Hs, Ws, S, stripes, run, nwin;
  Strides6 q, k, v, o;            // elided: views of qkv [B, L, 3C] and of this half's result [B, L, C/2]
  Copy split, merge;              // explicit
  Copy v_images, pe_split;        // explicit, with the positional encoding: values as [nwin, S, C/2], its result head-split
};
struct CswinPlan {
  Branch br[2];
  TableRegion ex_tables;
  int n_layout, n_eliminated, n_kept;
};

struct Key { int v[8]; bool operator<(const Key& o) const { return std::memcmp(v, o.v, sizeof(v)) < 0; } };
std::mutex g_mu;
std::map<Key, std::shared_ptr<CswinPlan>> g_plans;

// the planned map of a [nwin, heads, S, d] operand, looked at as [B, stripes, heads, S / run, run, d]: strided or refused
bool factored(const sm_map* m, const Branch& b, int64_t B, int64_t hb, int64_t d, Strides6* out, std::string* err, const char* what) {
  if (!m) { *err = std::string(what) + ": no map planned"; return false; }
  std::vector<sm_view_op> ch = m->chain;
  ch.push_back(chains::reshape({B, b.stripes, hb, b.S / b.run, b.run, d}));
  sm_map* m6 = nullptr;
  if (map_create(m->src_shape, ch.data(), (int)ch.size(), &m6, err) != SM_OK) return false;
  std::unique_ptr<sm_map> guard(m6);
  int64_t st[SM_MAX_RANK];
  if (!m6->affine(&out->base, st) || st[5] != 1) { *err = std::string(what) + ": not strided in (image, stripe, head, run, token, feature)"; return false; }
  out->img = st[0]; out->stripe = st[1]; out->head = st[2]; out->runs = st[3]; out->tok = st[4];
  return true;
}

std::shared_ptr<CswinPlan> cswin_plan(const sm_cswin_cfg& c, bool lepe, std::string* err) {
  Key key{{c.B, c.H, c.W, c.C, c.heads, c.sw, c.dtype, lepe ? 1 : 0}};
  std::lock_guard<std::mutex> lock(g_mu);
  auto it = g_plans.find(key);
  if (it != g_plans.end()) return it->second;
  auto p = std::make_shared<CswinPlan>();
  const int64_t B = c.B, H = c.H, W = c.W, C = c.C, L = H * W, hb = c.heads / 2, Cb = C / 2, d = C / c.heads;
  for (int i = 0; i < 2; ++i) {
    Branch& b = p->br[i];
    b.Hs = i == 0 ? H : c.sw; b.Ws = i == 0 ? c.sw : W;
    b.S = b.Hs * b.Ws;
    b.stripes = (H / b.Hs) * (W / b.Ws);
    b.nwin = B * b.stripes;
    b.run = i == 0 ? c.sw : b.S;          // vertical stripe: sw adjacent tokens per grid row; horizontal: whole rows, all adjacent
  }
  GraphB g;
  const int qkv = g.tensor({B, L, 3 * C});
  const int t4 = g.reshape(qkv, {B, L, 3, C});
  int whole[3];
  for (int k = 0; k < 3; ++k) whole[k] = g.reshape(g.slice(t4, 2, k, k + 1), {B, L, C});
  for (int i = 0; i < 2; ++i) {
    const Branch& b = p->br[i];
    int part[3];
    for (int k = 0; k < 3; ++k) {
      int t = g.slice(whole[k], 2, i * Cb, (i + 1) * Cb);
      t = g.transpose(t, {0, 2, 1});
      t = g.reshape(t, {B, Cb, H / b.Hs, b.Hs, W / b.Ws, b.Ws});
      t = g.transpose(t, {0, 2, 4, 3, 5, 1});
      t = g.reshape(t, {b.nwin, b.S, Cb});
      t = g.reshape(t, {b.nwin, b.S, hb, d});
      part[k] = g.transpose(t, {0, 2, 1, 3});
    }
    int pe = -1;
    if (lepe) {        // before the attention in graph order: the Add then joins the attention, its later producer
      int u = g.slice(whole[2], 2, i * Cb, (i + 1) * Cb);
      u = g.transpose(u, {0, 2, 1});
      u = g.reshape(u, {B, Cb, H / b.Hs, b.Hs, W / b.Ws, b.Ws});
      u = g.transpose(u, {0, 2, 4, 1, 3, 5});
      u = g.reshape(u, {b.nwin, Cb, b.Hs, b.Ws});
      u = g.op(SM_OP_CONV, {u}, {b.nwin, Cb, b.Hs, b.Ws}, i == 0 ? "lepe0" : "lepe1");
      u = g.reshape(u, {b.nwin, hb, d, b.S});
      pe = g.transpose(u, {0, 1, 3, 2});
    }
    int t = g.op(SM_OP_ATTENTION, {part[0], part[1], part[2]}, {b.nwin, hb, b.S, d}, i == 0 ? "attn0" : "attn1", {3, 3, -1});
    if (lepe) t = g.op(SM_OP_ADD, {t, pe}, {b.nwin, hb, b.S, d}, "add_pe");
    t = g.transpose(t, {0, 2, 1, 3});
    t = g.reshape(t, {b.nwin, b.S, Cb});
    t = g.reshape(t, {B, H / b.Hs, W / b.Ws, b.Hs, b.Ws, Cb});
    t = g.transpose(t, {0, 1, 3, 2, 4, 5});
    g.reshape(t, {B, L, Cb});
  }
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
  if (p->n_eliminated != p->n_layout || p->n_kept != (lepe ? 4 : 2)) {
    char msg[160];
    snprintf(msg, sizeof(msg), "planner did not reduce the operator to its attentions and convolutions (%d kept, %d of %d layout operators eliminated)",
             p->n_kept, p->n_eliminated, p->n_layout);
    *err = msg; return nullptr;
  }
  const int es = (int)dtype_size(c.dtype);
  for (int i = 0; i < 2; ++i) {
    Branch& b = p->br[i];
    const int attn = g.find(i == 0 ? "attn0" : "attn1");
    const sm_map* m = nullptr;
    Strides6* dst[3] = {&b.q, &b.k, &b.v};
    for (int k = 0; k < 3; ++k) {
      sm_plan_load_map(plan, attn, k, &m, nullptr);
      if (!factored(m, b, B, hb, d, dst[k], err, "attention load")) return nullptr;
    }
    sm_plan_store_map(plan, attn, &m, nullptr);
    if (!factored(m, b, B, hb, d, &b.o, err, "attention store")) return nullptr;
    // explicit chain: q, k, v of this half in one copy [3, nwin, heads, S, d]; head merge + stripe merge in another
    std::vector<sm_view_op> split{chains::reshape({B, L, 3, C}), chains::slice(3, i * Cb, (i + 1) * Cb), chains::permute({2, 0, 3, 1}),
                                  chains::reshape({3, B, Cb, H / b.Hs, b.Hs, W / b.Ws, b.Ws}), chains::permute({0, 1, 3, 5, 4, 6, 2}),
                                  chains::reshape({3, b.nwin, b.S, hb, d}), chains::permute({0, 1, 3, 2, 4})};
    if (!make_copy({B, L, 3 * C}, split, es, &p->ex_tables, &b.split, err)) return nullptr;
    std::vector<sm_view_op> merge{chains::permute({0, 2, 1, 3}), chains::reshape({b.nwin, b.S, Cb}), chains::reshape({B, H / b.Hs, W / b.Ws, b.Hs, b.Ws, Cb}),
                                  chains::permute({0, 1, 3, 2, 4, 5}), chains::reshape({B, L, Cb})};
    if (!make_copy({b.nwin, hb, b.S, d}, merge, es, &p->ex_tables, &b.merge, err)) return nullptr;
    if (lepe) {
      // the convolution kernel addresses element (image, y, x, channel) of the values at
      // image * 3CL + (y W + x) * 3C + channel, from 2C + i C/2: the planned load map must say the same
      const int conv = g.find(i == 0 ? "lepe0" : "lepe1");
      sm_plan_load_map(plan, conv, 0, &m, nullptr);
      if (!m || m->shape.size() != 4) { *err = "convolution load: no map planned"; return nullptr; }
      const int64_t wst = W / b.Ws;                   // stripes per grid row
      uint64_t rng = 0x9e3779b97f4a7c15ull;
      for (int trial = 0; trial < 256; ++trial) {
        int64_t idx[4];
        for (int a = 0; a < 4; ++a) {
          rng = rng * 6364136223846793005ull + 1442695040888963407ull;
          const int64_t n = m->shape[a];
          idx[a] = trial == 0 ? 0 : (trial == 1 ? n - 1 : (int64_t)((rng >> 33) % (uint64_t)n));
        }
        const int64_t win = idx[0], img = win / b.stripes, sidx = win % b.stripes;
        const int64_t y = (sidx / wst) * b.Hs + idx[2], x = (sidx % wst) * b.Ws + idx[3];
        if (m->at(idx) != 2 * C + i * Cb + idx[1] + img * 3 * C * L + (y * W + x) * 3 * C) { *err = "convolution load: the planned map is not the token-major view the kernel reads"; return nullptr; }
      }
      std::vector<sm_view_op> vi{chains::reshape({B, L, 3, C}), chains::slice(2, 2, 3), chains::reshape({B, L, C}), chains::slice(2, i * Cb, (i + 1) * Cb),
                                 chains::permute({0, 2, 1}), chains::reshape({B, Cb, H / b.Hs, b.Hs, W / b.Ws, b.Ws}), chains::permute({0, 2, 4, 3, 5, 1}),
                                 chains::reshape({b.nwin, b.S, Cb})};
      if (!make_copy({B, L, 3 * C}, vi, es, &p->ex_tables, &b.v_images, err)) return nullptr;
      if (!make_copy({b.nwin, b.S, Cb}, chains::head_split(b.nwin, b.S, hb, d), es, &p->ex_tables, &b.pe_split, err)) return nullptr;
    }
  }
  if (g_plans.size() >= 64) g_plans.clear();
  g_plans[key] = p;
  return p;
}

int check_cfg(const sm_cswin_cfg* c, const char* who) {
  if (!c) return fail(SM_ERR_INVALID_ARG, "%s: null configuration", who);
  if (c->dtype != SM_BF16) return fail(SM_ERR_UNSUPPORTED, "%s: bf16 only", who);
  if (c->B < 1 || c->H < 1 || c->W < 1 || c->C < 1 || c->heads < 2 || c->sw < 1) return fail(SM_ERR_SHAPE, "%s: bad shape", who);
  if (c->heads % 2 || c->C % c->heads) return fail(SM_ERR_SHAPE, "%s: the channels must split into an even number of heads", who);
  const int d = c->C / c->heads;
  if (d % 8 || d > 32) return fail(SM_ERR_SHAPE, "%s: head size must be a multiple of 8, at most 32", who);
  if (c->H % c->sw || c->W % c->sw) return fail(SM_ERR_SHAPE, "%s: grid %d x %d is not a multiple of the stripe width %d", who, c->H, c->W, c->sw);
  if ((int64_t)c->sw * std::max(c->H, c->W) > 65536) return fail(SM_ERR_SHAPE, "%s: a stripe may hold at most 65536 tokens", who);
  if ((int64_t)c->B * c->H * c->W * 3 * c->C >= (1LL << 31)) return fail(SM_ERR_SHAPE, "%s: more than 2^31 elements", who);
  return SM_OK;
}

size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }
// explicit mode: per half, [3, nwin, heads/2, S, d] operands, the attention result, the merged result (5 units; with
// the positional encoding also the values as stripe images and the encoding: 7)
size_t half_bytes(const sm_cswin_cfg& c) { return align256((size_t)c.B * c.H * c.W * (c.C / 2) * dtype_size(c.dtype)); }

}  // namespace

extern "C" size_t sm_cswin_attention_workspace_bytes(const sm_cswin_cfg* c, int mode) {
  if (check_cfg(c, "sm_cswin_attention_workspace_bytes") != SM_OK) return 0;
  if (mode != SM_ELIDED && mode != SM_EXPLICIT) { set_error("sm_cswin_attention_workspace_bytes: unknown mode %d", mode); return 0; }
  std::string err;
  auto plan = cswin_plan(*c, true, &err);        // the larger of the two forms
  if (!plan || !cswin_plan(*c, false, &err)) { set_error("sm_cswin_attention_workspace_bytes: %s", err.c_str()); return 0; }
  if (mode == SM_ELIDED) return 256;       // nothing is staged (0 is this query's error value)
  return 14 * half_bytes(*c) + plan->ex_tables.bytes;
}

namespace {
int cswin_attention_impl(const sm_cswin_cfg* c, const void* qkv, const void* lepe_w, const void* lepe_b, void* out,
                         void* ws, size_t ws_bytes, int mode, void* stream, bool reset_counts);
}
extern "C" int sm_cswin_attention(const sm_cswin_cfg* c, const void* qkv, const void* lepe_w, const void* lepe_b, void* out,
                                  void* ws, size_t ws_bytes, int mode, void* stream) {
  return cswin_attention_impl(c, qkv, lepe_w, lepe_b, out, ws, ws_bytes, mode, stream, true);
}
namespace {
int cswin_attention_impl(const sm_cswin_cfg* c, const void* qkv, const void* lepe_w, const void* lepe_b, void* out,
                         void* ws, size_t ws_bytes, int mode, void* stream, bool reset_counts) {
  int rc = check_cfg(c, "sm_cswin_attention");
  if (rc) return rc;
  if (!qkv || !out) return fail(SM_ERR_INVALID_ARG, "sm_cswin_attention: null pointer");
  if (mode != SM_ELIDED && mode != SM_EXPLICIT) return fail(SM_ERR_INVALID_ARG, "sm_cswin_attention: unknown mode %d", mode);
  if (!aligned16(qkv) || !aligned16(out) || (ws && !aligned16(ws))) return fail(SM_ERR_INVALID_ARG, "sm_cswin_attention: pointers must be 16-byte aligned");
  if ((lepe_w == nullptr) != (lepe_b == nullptr)) return fail(SM_ERR_INVALID_ARG, "sm_cswin_attention: the positional encoding needs both its weights and its bias");
  if (lepe_w && (!aligned16(lepe_w) || !aligned16(lepe_b))) return fail(SM_ERR_INVALID_ARG, "sm_cswin_attention: pointers must be 16-byte aligned");
  const bool lepe = lepe_w != nullptr;
  std::string err;
  auto plan = cswin_plan(*c, lepe, &err);
  if (!plan) return fail(SM_ERR_UNSUPPORTED, "sm_cswin_attention: %s", err.c_str());
  const bool el = mode == SM_ELIDED;
  const size_t hbytes = half_bytes(*c);
  if (!el) {
    const size_t need = (lepe ? 14 : 10) * hbytes + plan->ex_tables.bytes;
    if (!ws || ws_bytes < need) return fail(SM_ERR_WORKSPACE, "sm_cswin_attention: workspace of %zu bytes, %zu needed", ws ? ws_bytes : (size_t)0, need);
  }
  if (reset_counts) count_reset();
  const int64_t B = c->B, L = (int64_t)c->H * c->W, C = c->C, Cb = C / 2, hb = c->heads / 2, d = C / c->heads;
  const unsigned short* src = (const unsigned short*)qkv;
  unsigned short* dst = (unsigned short*)out;
  char* base = (char*)ws;
  const size_t units = lepe ? 7 : 5;
  const void* tables = el ? nullptr : base + 2 * units * hbytes;
  if (!el && (rc = fill_tables(plan->ex_tables, base + 2 * units * hbytes, stream, ~0ull))) return rc;
  // i < 0: both halves of the channels in one launch (whole images, each half with its own stripe shape)
  auto conv = [&](const Branch& b, int i, const void* v, void* o, int n_img, int gh, int gw, int64_t v_img, int64_t v_tok, int64_t o_img, int64_t o_tok) -> int {
    DwconvArgs k; std::memset(&k, 0, sizeof(k));
    const int first = i < 0 ? 0 : i;
    k.v = v; k.out = o; k.w = (const unsigned short*)lepe_w + (size_t)first * Cb * 9; k.bias = (const unsigned short*)lepe_b + (size_t)first * Cb;
    k.n_img = n_img; k.H = gh; k.W = gw; k.Cn = (int)(i < 0 ? C : Cb); k.Hs = (int)b.Hs; k.Ws = (int)b.Ws;
    if (i < 0) { k.split_c = (int)Cb; k.Hs2 = (int)plan->br[1].Hs; k.Ws2 = (int)plan->br[1].Ws; }
    k.v_img = v_img; k.v_tok = v_tok; k.o_img = o_img; k.o_tok = o_tok;
    char label[96];
    snprintf(label, sizeof(label), "dwconv3x3_bf16[%d,%d,%d,%d]", n_img, gh, gw, k.Cn);
    Timed tm(label, stream);
    if (int e = launch_dwconv3x3(k, stream)) return fail(SM_ERR_DEVICE, "sm_cswin_attention: convolution launch failed (hip error %d)", e);
    count_compute();
    return SM_OK;
  };
  void* merged[2] = {nullptr, nullptr};
  sm_attention_desc el_desc[2];
  // elided: the encoding of both halves first, in one launch, straight into the output (stripe-aware taps)
  if (el && lepe && (rc = conv(plan->br[0], -1, src + 2 * C, dst, (int)B, c->H, c->W, 3 * C * L, 3 * C, C * L, C))) return rc;
  for (int i = 0; i < 2; ++i) {
    const Branch& b = plan->br[i];
    sm_attention_desc a; std::memset(&a, 0, sizeof(a));
    a.dtype = c->dtype; a.nb = (int)b.nwin; a.heads = (int)hb; a.nq = a.nk = (int)b.S; a.d = (int)d;
    a.scale = (float)(1.0 / std::sqrt((double)d));
    a.accumulate = lepe ? 1 : 0;
    if (el) {
      a.kind = SM_ATT_STRIPE; a.stripes = (int)b.stripes; a.run = (int)b.run;
      const Strides6* in[3] = {&b.q, &b.k, &b.v};
      int64_t* st[3] = {a.q_stride, a.k_stride, a.v_stride};
      int64_t* sp[3] = {a.q_stripe, a.k_stripe, a.v_stripe};
      for (int k = 0; k < 3; ++k) { st[k][0] = in[k]->img; st[k][1] = in[k]->head; st[k][2] = in[k]->tok; sp[k][0] = in[k]->stripe; sp[k][1] = in[k]->runs; }
      // the planned store map addresses this half's result [B, L, C/2]; the Concat puts that tensor into columns
      // [i C/2, (i + 1) C/2) of rows of C elements: token strides grow by C / (C/2), the column offset is added
      const Strides6& o = b.o;
      if (o.img % Cb || o.stripe % Cb || o.runs % Cb || o.tok % Cb || o.base != 0 || o.head >= Cb)
        return fail(SM_ERR_UNSUPPORTED, "sm_cswin_attention: the planned store is not by whole tokens");
      a.o_stride[0] = o.img / Cb * C; a.o_stride[1] = o.head; a.o_stride[2] = o.tok / Cb * C;
      a.o_stripe[0] = o.stripe / Cb * C; a.o_stripe[1] = o.runs / Cb * C;
      el_desc[i] = a;
    } else {
      char* mine = base + (size_t)i * units * hbytes;
      unsigned short* parts = (unsigned short*)mine;      // [3, nwin, heads/2, S, d]
      unsigned short* res = (unsigned short*)(mine + 3 * hbytes);
      merged[i] = mine + 4 * hbytes;
      if ((rc = copy_launch(b.split, tables, qkv, parts, c->dtype, stream))) return rc;
      if (lepe) {        // values as stripe images [nwin, Hs, Ws, C/2], the convolution on them, its result head-split under the attention's
        void* vimg = mine + 5 * hbytes; void* pe = mine + 6 * hbytes;
        if ((rc = copy_launch(b.v_images, tables, qkv, vimg, c->dtype, stream))) return rc;
        if ((rc = conv(b, i, vimg, pe, (int)b.nwin, (int)b.Hs, (int)b.Ws, b.S * Cb, Cb, b.S * Cb, Cb))) return rc;
        if ((rc = copy_launch(b.pe_split, tables, pe, res, c->dtype, stream))) return rc;
      }
      a.kind = SM_ATT_FULL;
      const int64_t per = b.nwin * hb * b.S * d;
      int64_t* st[4] = {a.q_stride, a.k_stride, a.v_stride, a.o_stride};
      for (int k = 0; k < 4; ++k) { st[k][0] = hb * b.S * d; st[k][1] = b.S * d; st[k][2] = d; }
      if ((rc = attention_checked(a, parts, parts + per, parts + 2 * per, res, nullptr, stream, "sm_cswin_attention"))) return rc;
      if ((rc = copy_launch(b.merge, tables, res, merged[i], c->dtype, stream))) return rc;
    }
  }
  if (el) {
    // the two halves as one launch when they have one shape (square grids), else one after the other
    const Branch &b0 = plan->br[0], &b1 = plan->br[1];
    void* p0[4] = {(void*)(src + b0.q.base), (void*)(src + b0.k.base), (void*)(src + b0.v.base), dst};
    void* p1[4] = {(void*)(src + b1.q.base), (void*)(src + b1.k.base), (void*)(src + b1.v.base), dst + Cb};
    if (b0.nwin == b1.nwin && b0.S == b1.S) return attention_stripe_pair_checked(el_desc[0], p0, el_desc[1], p1, stream, "sm_cswin_attention");
    if ((rc = attention_checked(el_desc[0], p0[0], p0[1], p0[2], p0[3], nullptr, stream, "sm_cswin_attention"))) return rc;
    return attention_checked(el_desc[1], p1[0], p1[1], p1[2], p1[3], nullptr, stream, "sm_cswin_attention");
  }
  {
    char label[96];
    snprintf(label, sizeof(label), "concat_bf16[%lld,%lld]", (long long)(B * L), (long long)C);
    Timed tm(label, stream);
    if (int e = launch_concat2_cols(merged[0], merged[1], out, B * L, (int)(Cb * dtype_size(c->dtype)), stream))
      return fail(SM_ERR_DEVICE, "sm_cswin_attention: concat launch failed (hip error %d)", e);
    count_copy();
  }
  return SM_OK;
}
}  // namespace

// ---------------------------------------------------------------------------
// sm_cswin_block
// ---------------------------------------------------------------------------
namespace {

sm_cswin_cfg attn_cfg(const sm_cswin_block_cfg& c) { return sm_cswin_cfg{c.dtype, c.B, c.H, c.W, c.C, c.heads, c.sw}; }
int check_block(const sm_cswin_block_cfg* c, const char* who) {
  if (!c) return fail(SM_ERR_INVALID_ARG, "%s: null configuration", who);
  const sm_cswin_cfg a = attn_cfg(*c);
  if (int rc = check_cfg(&a, who)) return rc;
  if (c->C % 16) return fail(SM_ERR_SHAPE, "%s: C must be a multiple of 16", who);
  if (c->mlp_ratio < 1 || c->mlp_ratio > 8 || !(c->eps > 0.f)) return fail(SM_ERR_SHAPE, "%s: bad MLP ratio or epsilon", who);
  return SM_OK;
}
size_t token_bytes(const sm_cswin_block_cfg& c) { return align256((size_t)c.B * c.H * c.W * c.C * dtype_size(c.dtype)); }
// q | k | v (3 units), attention output, x1, a normalised copy, the MLP's hidden tensor
size_t block_act_bytes(const sm_cswin_block_cfg& c) { return (6 + (size_t)c.mlp_ratio) * token_bytes(c); }

int norm_rows(const void* x, const void* g, const void* b, void* y, int64_t rows, int C, float eps, int dt, void* stream) {
  NormArgs a; std::memset(&a, 0, sizeof(a));
  a.x = x; a.gamma = g; a.beta = b; a.y = y; a.rows = rows; a.C = C; a.eps = eps; a.rms = 0; a.dtype = dt; a.nseg = 1;
  a.load = identity_rows(C); a.store = identity_rows(C);
  return norm_checked(a, stream, "sm_cswin_block(norm)");
}
// ln_g != null: LayerNorm of A's rows folded into the load
int linear_rows(const void* A, const void* W, const void* bias, const void* res, void* Cc, int64_t M, int N, int K, int dt, int act,
                void* stream, const void* ln_g = nullptr, const void* ln_b = nullptr, float eps = 0.f) {
  GemmArgs g; std::memset(&g, 0, sizeof(g));
  g.A = A; g.W = W; g.bias = bias; g.residual = res; g.C = Cc; g.M = M; g.N = N; g.K = K; g.dtype = dt; g.act = act; g.ldw = K;
  if (ln_g) { g.norm = 1; g.norm_gamma = ln_g; g.norm_beta = ln_b; g.norm_eps = eps; }
  g.a_rows = identity_rows(K); g.c_rows = identity_rows(N);
  return gemm_checked(g, stream, "sm_cswin_block(linear)");
}
// the norm is folded into the Linear while the Linear has few column tiles (it is repeated per column tile)
bool fold(int n_cols) { return n_cols <= 512; }

}  // namespace

extern "C" size_t sm_cswin_block_workspace_bytes(const sm_cswin_block_cfg* c, int mode) {
  if (check_block(c, "sm_cswin_block_workspace_bytes") != SM_OK) return 0;
  const sm_cswin_cfg a = attn_cfg(*c);
  const size_t inner = sm_cswin_attention_workspace_bytes(&a, mode);
  if (inner == 0) return 0;
  return block_act_bytes(*c) + inner;
}

extern "C" int sm_cswin_block(const sm_cswin_block_cfg* c, const sm_cswin_weights* wt, const void* x, void* y, void* ws, size_t ws_bytes,
                              int mode, void* stream) {
  int rc = check_block(c, "sm_cswin_block");
  if (rc) return rc;
  if (!wt || !x || !y || !ws) return fail(SM_ERR_INVALID_ARG, "sm_cswin_block: null pointer");
  if (mode != SM_ELIDED && mode != SM_EXPLICIT) return fail(SM_ERR_INVALID_ARG, "sm_cswin_block: unknown mode %d", mode);
  const void* need_w[] = {wt->ln1_g, wt->ln1_b, wt->wqkv, wt->bqkv, wt->lepe_w, wt->lepe_b, wt->wproj, wt->bproj, wt->ln2_g, wt->ln2_b, wt->w1, wt->b1, wt->w2, wt->b2};
  for (const void* p : need_w) if (!p || !aligned16(p)) return fail(SM_ERR_INVALID_ARG, "sm_cswin_block: a weight is null or misaligned");
  if (!aligned16(x) || !aligned16(y) || !aligned16(ws)) return fail(SM_ERR_INVALID_ARG, "sm_cswin_block: pointers must be 16-byte aligned");
  const sm_cswin_cfg acfg = attn_cfg(*c);
  const size_t inner = sm_cswin_attention_workspace_bytes(&acfg, mode);
  if (inner == 0) return SM_ERR_UNSUPPORTED;          // message set by the query
  const size_t act = block_act_bytes(*c);
  if (ws_bytes < act + inner) return fail(SM_ERR_WORKSPACE, "sm_cswin_block: workspace of %zu bytes, %zu needed", ws_bytes, act + inner);
  count_reset();
  const int64_t T = (int64_t)c->B * c->H * c->W;
  const int C = c->C, Hd = c->mlp_ratio * C, dt = c->dtype;
  const size_t tc = token_bytes(*c);
  char* base = (char*)ws;
  void* qkv = base; void* att = base + 3 * tc; void* x1 = base + 4 * tc; void* nbuf = base + 5 * tc; void* hid = base + 6 * tc;
  void* inner_ws = base + act;

  // LayerNorm + fused q | k | v Linear
  if (wt->qkv_packed && lin32_supported(3 * C, C, dt)) {
    Lin32Args a; std::memset(&a, 0, sizeof(a));
    a.X = x; a.Wp = wt->qkv_packed; a.bias = wt->bqkv; a.Y = qkv; a.M = T; a.N = 3 * C; a.K = C; a.act = SM_ACT_NONE;
    a.norm = 1; a.norm_eps = c->eps; a.norm_gamma = wt->ln1_g; a.norm_beta = wt->ln1_b;
    a.x_rows = identity_rows(C); a.y_rows = identity_rows(3 * C);
    if ((rc = lin32_checked(a, stream, "sm_cswin_block(ln1+qkv)"))) return rc;
  } else if (fold(3 * C)) {
    if ((rc = linear_rows(x, wt->wqkv, wt->bqkv, nullptr, qkv, T, 3 * C, C, dt, SM_ACT_NONE, stream, wt->ln1_g, wt->ln1_b, c->eps))) return rc;
  } else {
    if ((rc = norm_rows(x, wt->ln1_g, wt->ln1_b, nbuf, T, C, c->eps, dt, stream))) return rc;
    if ((rc = linear_rows(nbuf, wt->wqkv, wt->bqkv, nullptr, qkv, T, 3 * C, C, dt, SM_ACT_NONE, stream))) return rc;
  }
  // every layout operator of the block: elided or explicit
  if ((rc = cswin_attention_impl(&acfg, qkv, wt->lepe_w, wt->lepe_b, att, inner_ws, inner, mode, stream, false))) return rc;
  // output Linear + residual + LayerNorm + MLP + residual
  if (wt->proj_packed && wt->mlp_packed && mlp_proj_supported(C, Hd, dt)) {
    MlpArgs a; std::memset(&a, 0, sizeof(a));
    a.X = att; a.Wp = wt->mlp_packed; a.b1 = wt->b1; a.b2 = wt->b2; a.Y = y; a.M = T; a.C = C; a.Hd = Hd;
    a.norm = 1; a.norm_eps = c->eps; a.norm_gamma = wt->ln2_g; a.norm_beta = wt->ln2_b;
    a.Wproj_p = wt->proj_packed; a.bproj = wt->bproj; a.resid0 = x;
    a.x_rows = identity_rows(C); a.y_rows = identity_rows(C);
    return mlp_checked(a, stream, "sm_cswin_block(proj+mlp)");
  }
  if ((rc = linear_rows(att, wt->wproj, wt->bproj, x, x1, T, C, C, dt, SM_ACT_NONE, stream))) return rc;
  if (wt->mlp_packed && mlp_fused_supported(C, Hd, dt)) {
    MlpArgs a; std::memset(&a, 0, sizeof(a));
    a.X = x1; a.Wp = wt->mlp_packed; a.b1 = wt->b1; a.b2 = wt->b2; a.residual = x1; a.Y = y; a.M = T; a.C = C; a.Hd = Hd;
    a.norm = 1; a.norm_eps = c->eps; a.norm_gamma = wt->ln2_g; a.norm_beta = wt->ln2_b;
    a.x_rows = identity_rows(C); a.y_rows = identity_rows(C);
    return mlp_checked(a, stream, "sm_cswin_block(mlp)");
  }
  if (fold(Hd)) {
    if ((rc = linear_rows(x1, wt->w1, wt->b1, nullptr, hid, T, Hd, C, dt, SM_ACT_GELU, stream, wt->ln2_g, wt->ln2_b, c->eps))) return rc;
  } else {
    if ((rc = norm_rows(x1, wt->ln2_g, wt->ln2_b, nbuf, T, C, c->eps, dt, stream))) return rc;
    if ((rc = linear_rows(nbuf, wt->w1, wt->b1, nullptr, hid, T, Hd, C, dt, SM_ACT_GELU, stream))) return rc;
  }
  return linear_rows(hid, wt->w2, wt->b2, x1, y, T, C, Hd, dt, SM_ACT_NONE, stream);
}
