// C ABI of the single operators: validation and map compilation, then one launch.
#include <cstring>
#include "common.h"
#include "index_map.h"
#include "kernels.h"

using namespace sm;

namespace sm {

// row program of a map whose view has `rows * inner` elements and last dimension `inner`
int rows_of(const sm_map* m, int64_t rows, int64_t inner, int64_t identity_ld, RowProg* out, const char* who) {
  if (!m) { *out = identity_rows(identity_ld); return SM_OK; }
  if (m->numel() != rows * inner || m->shape.back() != inner)
    return fail(SM_ERR_SHAPE, "%s: map has %lld elements / last dimension %lld, operand needs %lld x %lld", who,
                (long long)m->numel(), (long long)m->shape.back(), (long long)rows, (long long)inner);
  std::string err;
  if (!m->compile_rows(out, &err)) return fail(SM_ERR_UNSUPPORTED, "%s: %s", who, err.c_str());
  return SM_OK;
}

int norm_checked(NormArgs& a, void* stream, const char* who) {
  if (a.rows == 0 && a.C >= 1 && dtype_ok(a.dtype)) return SM_OK;      // nothing to do: no pointer is looked at, nothing is launched
  if (!a.x || !a.gamma || !a.y) return fail(SM_ERR_INVALID_ARG, "%s: null pointer", who);
  if (!dtype_ok(a.dtype)) return fail(SM_ERR_INVALID_ARG, "%s: unknown dtype", who);
  const int vec = a.dtype == SM_F32 ? 4 : 8;
  if (a.rows < 0 || a.C < 1 || a.nseg < 1 || a.C % a.nseg) return fail(SM_ERR_SHAPE, "%s: bad shape", who);
  if (a.C % vec || (a.C / a.nseg) % vec) return fail(SM_ERR_SHAPE, "%s: C (and C / segments) must be a multiple of %d", who, vec);
  if (a.C / vec > 512) return fail(SM_ERR_UNSUPPORTED, "%s: C = %d exceeds %d", who, a.C, 512 * vec);
  if (!aligned16(a.x) || !aligned16(a.y) || !aligned16(a.gamma) || (a.beta && !aligned16(a.beta)))
    return fail(SM_ERR_INVALID_ARG, "%s: pointers must be 16-byte aligned", who);
  char label[96];
  snprintf(label, sizeof(label), "%s_%s[%lld,%d]%s", a.rms ? "rmsnorm" : "layernorm", a.dtype == SM_F32 ? "f32" : "bf16", (long long)a.rows, a.C, a.nseg > 1 ? "+gather" : (a.store.identity ? "" : "+scatter"));
  Timed tm(label, stream);
  int rc = launch_norm(a, stream);
  if (rc) return fail(SM_ERR_DEVICE, "%s: launch failed (hip error %d)", who, rc);
  count_compute();
  return SM_OK;
}

int gemm_checked(GemmArgs& g, void* stream, const char* who) {
  if (g.M == 0 && g.N >= 1 && g.K >= 1 && dtype_ok(g.dtype)) return SM_OK;      // no rows: nothing is launched
  if (!g.A || !g.W || !g.C) return fail(SM_ERR_INVALID_ARG, "%s: null pointer", who);
  if (!dtype_ok(g.dtype)) return fail(SM_ERR_INVALID_ARG, "%s: unknown dtype", who);
  const int vec = g.dtype == SM_F32 ? 4 : 8;
  if (g.M < 0 || g.N < 1 || g.K < 1) return fail(SM_ERR_SHAPE, "%s: bad shape", who);
  if (g.K % vec || g.ldw % vec) return fail(SM_ERR_SHAPE, "%s: K and the pitch of W must be multiples of %d", who, vec);
  if (g.act < SM_ACT_NONE || g.act > SM_ACT_GEGLU) return fail(SM_ERR_INVALID_ARG, "%s: unknown activation", who);
  const bool gated = g.act == SM_ACT_SWIGLU || g.act == SM_ACT_GEGLU;
  if (gated && (g.N % 64)) return fail(SM_ERR_SHAPE, "%s: gated activations need N / 2 to be a multiple of 32", who);
  if (g.c_cols_on && (g.c_transposed || g.act == SM_ACT_SWIGLU || g.act == SM_ACT_GEGLU)) return fail(SM_ERR_UNSUPPORTED, "%s: column-splitting store with a gated activation or transposed store", who);
  if (g.a_gran > 0 && (g.act != SM_ACT_NONE || g.rope_cols)) return fail(SM_ERR_UNSUPPORTED, "%s: activation or RoPE with an unfolded A operand", who);
  if (g.act != SM_ACT_NONE && g.rope_cols) return fail(SM_ERR_UNSUPPORTED, "%s: RoPE goes with no activation (the RoPE epilogue applies none)", who);
  if (g.C2 && (g.residual || g.c_transposed || g.c_cols_on || gated || !aligned16(g.C2)))
    return fail(SM_ERR_UNSUPPORTED, "%s: a second (column-major) copy goes with a plain store only", who);
  if (g.norm) {
    if (g.norm != 1 && g.norm != 2) return fail(SM_ERR_INVALID_ARG, "%s: unknown norm %d", who, g.norm);
    if (gated || g.rope_cols || g.a_gran > 0) return fail(SM_ERR_UNSUPPORTED, "%s: a folded norm goes with activation none or GELU only, without RoPE or an unfolded A", who);
    if (!g.norm_gamma || !aligned16(g.norm_gamma) || (g.norm_beta && !aligned16(g.norm_beta)))
      return fail(SM_ERR_INVALID_ARG, "%s: folded norm needs a 16-byte aligned gamma (and beta, if given)", who);
    if (!(g.norm_eps > 0.f)) return fail(SM_ERR_INVALID_ARG, "%s: folded norm needs eps > 0", who);
  }
  if (g.rope_cols) {
    if (g.rope_dim < 64 || g.rope_dim % 64 || g.rope_cols % g.rope_dim || g.rope_cols > g.N || g.rope_seq < 1)
      return fail(SM_ERR_SHAPE, "%s: RoPE needs head size a multiple of 64 and whole heads", who);
  }
  if (g.c_transposed && (g.c_batch_rows < 1 || g.M % g.c_batch_rows)) return fail(SM_ERR_SHAPE, "%s: bad transposed-store batch", who);
  if (!aligned16(g.A) || !aligned16(g.W) || !aligned16(g.C) || (g.bias && !aligned16(g.bias)) || (g.residual && !aligned16(g.residual)))
    return fail(SM_ERR_INVALID_ARG, "%s: pointers must be 16-byte aligned", who);
  if ((int64_t)g.N * g.ldw > INT32_MAX * 16LL) return fail(SM_ERR_UNSUPPORTED, "%s: weight too large", who);
  char label[128];
  snprintf(label, sizeof(label), "%sgemm_%s[%lld,%d,%d]%s%s%s", g.norm == 1 ? "ln+" : (g.norm == 2 ? "rms+" : ""), g.dtype == SM_F32 ? "f32" : "bf16", (long long)g.M, g.N, g.K,
           g.act == SM_ACT_GELU ? "+gelu" : (g.act ? "+glu" : ""), g.residual ? "+res" : "", g.c_rows.identity ? "" : (g.C2 ? "+copy2" : "+scatter"));
  if (g.C2 && g.c_rows.identity) { const size_t n = strlen(label); snprintf(label + n, sizeof(label) - n, "+copy2"); }
  Timed tm(label, stream);
  int rc = launch_gemm(g, stream);
  if (rc) return fail(SM_ERR_DEVICE, "%s: launch failed (hip error %d)", who, rc);
  count_compute();
  return SM_OK;
}

namespace {
int attention_validate(const sm_attention_desc& d, const void* q, const void* k, const void* v, void* o, const void* table, const char* who) {
  if (!q || !k || !v || !o) return fail(SM_ERR_INVALID_ARG, "%s: null pointer", who);
  if (!dtype_ok(d.dtype)) return fail(SM_ERR_INVALID_ARG, "%s: unknown dtype", who);
  if (d.kind < SM_ATT_FULL || d.kind > SM_ATT_STRIPE) return fail(SM_ERR_INVALID_ARG, "%s: unknown kind", who);
  if (d.nb < 1 || d.heads < 1 || d.nq < 1 || d.nk < 1 || d.d < 1) return fail(SM_ERR_SHAPE, "%s: bad shape", who);
  const int vec = d.dtype == SM_F32 ? 4 : 8;
  if (d.d % vec || d.d > 128) return fail(SM_ERR_SHAPE, "%s: head size must be a multiple of %d and <= 128", who, vec);
  for (int i = 0; i < 3; ++i)
    if (d.q_stride[i] % vec || d.k_stride[i] % vec || d.v_stride[i] % vec || d.o_stride[i] % 4)
      return fail(SM_ERR_SHAPE, "%s: strides must keep 16-byte alignment", who);
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return fail(SM_ERR_INVALID_ARG, "%s: pointers must be 16-byte aligned", who);
  if (d.kind == SM_ATT_CAUSAL && d.nq != d.nk) return fail(SM_ERR_SHAPE, "%s: causal attention needs nq == nk", who);
  if (d.kind == SM_ATT_WINDOW) {
    if (!table) return fail(SM_ERR_INVALID_ARG, "%s: window attention needs the relative-position table", who);
    if (d.window < 1 || d.nq != d.window * d.window || d.nk != d.nq) return fail(SM_ERR_SHAPE, "%s: window attention needs nq == nk == window^2", who);
    if (d.H < d.window || d.W < d.window || d.H % d.window || d.W % d.window) return fail(SM_ERR_SHAPE, "%s: grid %d x %d is not a multiple of the window %d", who, d.H, d.W, d.window);
    if (d.shift < 0 || d.shift >= d.window) return fail(SM_ERR_SHAPE, "%s: shift out of range", who);
    if (d.nq > 64) return fail(SM_ERR_UNSUPPORTED, "%s: window attention supports windows of at most 64 tokens", who);
    if (d.nb % ((d.H / d.window) * (d.W / d.window))) return fail(SM_ERR_SHAPE, "%s: batch is not a whole number of images", who);
  }
  if (d.accumulate && (d.kind == SM_ATT_WINDOW || d.dtype != SM_BF16 || !(d.scale > 0.f)))
    return fail(SM_ERR_UNSUPPORTED, "%s: accumulating into O needs a bf16 full, causal or stripe attention with a positive scale", who);
  if (d.kind == SM_ATT_STRIPE) {
    if (d.dtype != SM_BF16 || d.d > 32 || !(d.scale > 0.f)) return fail(SM_ERR_UNSUPPORTED, "%s: stripe attention needs bf16, a head size <= 32 and a positive scale", who);
    if (d.nq != d.nk || d.nq > 65536) return fail(SM_ERR_SHAPE, "%s: stripe attention needs nq == nk <= 65536", who);
    if (d.stripes < 1 || d.run < 1 || d.nb % d.stripes || d.nq % d.run) return fail(SM_ERR_SHAPE, "%s: batch must be whole images of `stripes` stripes, a stripe whole runs", who);
    for (int i = 0; i < 2; ++i)
      if (d.q_stripe[i] % vec || d.k_stripe[i] % vec || d.v_stripe[i] % vec || d.o_stripe[i] % 4)
        return fail(SM_ERR_SHAPE, "%s: stripe strides must keep 16-byte alignment", who);
  }
  if (d.dtype == SM_F32) {
    if (d.kind != SM_ATT_WINDOW) return fail(SM_ERR_UNSUPPORTED, "%s: fp32 supports window attention only", who);
    if (d.nq > 64 || d.d > 64) return fail(SM_ERR_UNSUPPORTED, "%s: fp32 window attention needs window^2 <= 64 and head size <= 64", who);
  }
  return SM_OK;
}
}  // namespace

int attention_checked(const sm_attention_desc& d, const void* q, const void* k, const void* v, void* o, const void* table,
                      void* stream, const char* who) {
  if (int rc = attention_validate(d, q, k, v, o, table, who)) return rc;
  char label[128];
  snprintf(label, sizeof(label), "attention_%s_%s[%d,%d,%d,%d,%d]%s", d.kind == SM_ATT_WINDOW ? "window" : (d.kind == SM_ATT_CAUSAL ? "causal" : (d.kind == SM_ATT_STRIPE ? "stripe" : "full")),
           d.dtype == SM_F32 ? "f32" : "bf16", d.nb, d.heads, d.nq, d.nk, d.d, d.accumulate ? "+acc" : "");
  Timed tm(label, stream);
  int rc = launch_attention(d, q, k, v, o, table, stream);
  if (rc) return fail(SM_ERR_DEVICE, "%s: launch failed (hip error %d)", who, rc);
  count_compute();
  return SM_OK;
}

// two stripe attentions of one shape (the halves of a cross-shaped window attention) as one launch; p0 / p1: {q, k, v, o}
int attention_stripe_pair_checked(const sm_attention_desc& d0, void* const* p0, const sm_attention_desc& d1, void* const* p1,
                                  void* stream, const char* who) {
  if (int rc = attention_validate(d0, p0[0], p0[1], p0[2], p0[3], nullptr, who)) return rc;
  if (int rc = attention_validate(d1, p1[0], p1[1], p1[2], p1[3], nullptr, who)) return rc;
  if (d0.kind != SM_ATT_STRIPE || d1.kind != SM_ATT_STRIPE || d0.nb != d1.nb || d0.heads != d1.heads || d0.nq != d1.nq || d0.d != d1.d ||
      d0.scale != d1.scale || d0.accumulate != d1.accumulate)
    return fail(SM_ERR_SHAPE, "%s: the two attentions of a pair must be stripe attentions of one shape", who);
  char label[128];
  snprintf(label, sizeof(label), "attention_stripe_bf16[%d,%d,%d,%d,%d]%s", 2 * d0.nb, d0.heads, d0.nq, d0.nk, d0.d, d0.accumulate ? "+acc" : "");
  Timed tm(label, stream);
  const void* c0[4] = {p0[0], p0[1], p0[2], p0[3]};
  const void* c1[4] = {p1[0], p1[1], p1[2], p1[3]};
  int rc = launch_attention_stripe_pair(d0, c0, d1, c1, stream);
  if (rc) return fail(SM_ERR_DEVICE, "%s: launch failed (hip error %d)", who, rc);
  count_compute();
  return SM_OK;
}

}  // namespace sm

extern "C" int sm_norm(const void* x, const void* gamma, const void* beta, void* y, int64_t rows, int C, float eps,
                       int rms, int dtype, const sm_map* store_map, void* stream) {
  NormArgs a; std::memset(&a, 0, sizeof(a));
  a.x = x; a.gamma = gamma; a.beta = beta; a.y = y; a.rows = rows; a.C = C; a.eps = eps; a.rms = rms; a.dtype = dtype; a.nseg = 1;
  a.load = identity_rows(C);
  int rc = rows_of(store_map, rows, C, C, &a.store, "sm_norm");
  if (rc) return rc;
  return norm_checked(a, stream, "sm_norm");
}

extern "C" int sm_groupnorm(const void* x, const void* gamma, const void* beta, void* y, int B, int C, int HW, int G,
                            float eps, int tokens_out, int dtype, void* stats_scratch, void* stream) {
  if (!x || !gamma || !beta || !y) return fail(SM_ERR_INVALID_ARG, "sm_groupnorm: null pointer");
  if (!dtype_ok(dtype)) return fail(SM_ERR_INVALID_ARG, "sm_groupnorm: unknown dtype");
  if (B < 1 || C < 1 || HW < 1 || G < 1 || C % G) return fail(SM_ERR_SHAPE, "sm_groupnorm: bad shape");
  if (stats_scratch && (!aligned16(x) || !aligned16(y))) return fail(SM_ERR_INVALID_ARG, "sm_groupnorm: pointers must be 16-byte aligned");
  GroupNormArgs a{x, gamma, beta, y, B, C, HW, G, eps, tokens_out, dtype, (float*)stats_scratch};
  Timed tm("groupnorm", stream);
  int rc = launch_groupnorm(a, stream);
  if (rc) return fail(SM_ERR_DEVICE, "sm_groupnorm: launch failed (hip error %d)", rc);
  count_compute(groupnorm_launches(a));
  return SM_OK;
}

namespace sm {
int lin32_checked(Lin32Args& a, void* stream, const char* who) {
  if (!lin32_supported(a.N, a.K, SM_BF16)) return fail(SM_ERR_UNSUPPORTED, "%s: no packed-weight kernel for N = %d, K = %d", who, a.N, a.K);
  if (a.M < 0) return fail(SM_ERR_SHAPE, "%s: negative row count", who);
  if (a.act != SM_ACT_NONE && a.act != SM_ACT_GELU) return fail(SM_ERR_UNSUPPORTED, "%s: packed weights go with activation none or GELU", who);
  if (a.norm != 0 && a.norm != 1) return fail(SM_ERR_UNSUPPORTED, "%s: packed weights go with no norm or LayerNorm", who);
  if (a.M == 0) return SM_OK;
  if (!a.X || !a.Wp || !a.Y) return fail(SM_ERR_INVALID_ARG, "%s: null pointer", who);
  if (!aligned16(a.X) || !aligned16(a.Wp) || !aligned16(a.Y) || (a.bias && !aligned16(a.bias)) || (a.residual && !aligned16(a.residual)))
    return fail(SM_ERR_INVALID_ARG, "%s: pointers must be 16-byte aligned", who);
  if (a.norm) {
    if (!a.norm_gamma || !a.norm_beta || !aligned16(a.norm_gamma) || !aligned16(a.norm_beta))
      return fail(SM_ERR_INVALID_ARG, "%s: folded LayerNorm needs 16-byte aligned gamma and beta", who);
    if (!(a.norm_eps > 0.f)) return fail(SM_ERR_INVALID_ARG, "%s: folded LayerNorm needs eps > 0", who);
  }
  if ((a.M + 31) / 32 > 0x7fffffff) return fail(SM_ERR_SHAPE, "%s: too many rows", who);
  char label[128];
  std::snprintf(label, sizeof label, "%spgemm_bf16[%lld,%d,%d]%s%s%s", a.norm ? "ln+" : "", (long long)a.M, a.N, a.K,
                a.act == SM_ACT_GELU ? "+gelu" : "", a.residual ? "+res" : "", a.y_rows.identity ? "" : "+scatter");
  Timed tm(label, stream);
  const int rc = launch_lin32(a, stream);
  if (rc) return fail(SM_ERR_DEVICE, "%s: launch failed (hip error %d)", who, rc);
  count_compute(1);
  return SM_OK;
}
}  // namespace sm

extern "C" int sm_linear_pack_supported(int N, int K, int dtype) { return sm::lin32_supported(N, K, dtype) ? 1 : 0; }

extern "C" int sm_linear_pack(const void* W, int N, int K, int dtype, void* packed, void* stream) {
  if (!dtype_ok(dtype)) return fail(SM_ERR_INVALID_ARG, "sm_linear_pack: unknown dtype");
  if (!sm::lin32_supported(N, K, dtype)) return fail(SM_ERR_UNSUPPORTED, "sm_linear_pack: no packed-weight kernel for N = %d, K = %d, dtype %d", N, K, dtype);
  if (!W || !packed) return fail(SM_ERR_INVALID_ARG, "sm_linear_pack: null pointer");
  if (!aligned16(W) || !aligned16(packed)) return fail(SM_ERR_INVALID_ARG, "sm_linear_pack: pointers must be 16-byte aligned");
  Timed tm("linear_pack", stream);
  const int rc = launch_lin_pack(W, N, K, packed, stream);
  if (rc) return fail(SM_ERR_DEVICE, "sm_linear_pack: launch failed (hip error %d)", rc);
  return SM_OK;
}

extern "C" int sm_decode_pack(const void* W, int N, int K, int dtype, void* packed, void* stream) {
  if (dtype != SM_BF16) return fail(SM_ERR_UNSUPPORTED, "sm_decode_pack: bf16 only");
  if (N < 32 || N % 32 || K < 16 || K % 16) return fail(SM_ERR_SHAPE, "sm_decode_pack: N must be a multiple of 32 and K of 16 (N = %d, K = %d)", N, K);
  if (!W || !packed) return fail(SM_ERR_INVALID_ARG, "sm_decode_pack: null pointer");
  if (!aligned16(W) || !aligned16(packed)) return fail(SM_ERR_INVALID_ARG, "sm_decode_pack: pointers must be 16-byte aligned");
  Timed tm("decode_pack", stream);
  const int rc = launch_lin_pack(W, N, K, packed, stream);
  if (rc) return fail(SM_ERR_DEVICE, "sm_decode_pack: launch failed (hip error %d)", rc);
  return SM_OK;
}

extern "C" int sm_linear(const sm_linear_desc* d, const void* A, const void* W, const void* bias, const void* residual,
                         void* C, const sm_map* a_map, const sm_map* c_map, void* stream) {
  if (!d) return fail(SM_ERR_INVALID_ARG, "sm_linear: null descriptor");
  if (d->w_packed) {
    if (!dtype_ok(d->dtype)) return fail(SM_ERR_INVALID_ARG, "sm_linear: unknown dtype");
    if (!sm::lin32_supported(d->N, d->K, d->dtype)) return fail(SM_ERR_UNSUPPORTED, "sm_linear: no packed-weight kernel for N = %d, K = %d, dtype %d", d->N, d->K, d->dtype);
    if (d->rope_cols || d->c_transposed) return fail(SM_ERR_UNSUPPORTED, "sm_linear: packed weights go without RoPE and transposed stores");
    Lin32Args a; std::memset(&a, 0, sizeof(a));
    a.X = A; a.Wp = W; a.bias = bias; a.residual = residual; a.Y = C; a.M = d->M; a.N = d->N; a.K = d->K; a.act = d->act;
    a.norm = d->norm; a.norm_eps = d->norm_eps; a.norm_gamma = d->norm_gamma; a.norm_beta = d->norm_beta;
    int rc = rows_of(a_map, d->M, d->K, d->K, &a.x_rows, "sm_linear(A)");
    if (rc) return rc;
    rc = rows_of(c_map, d->M, d->N, d->N, &a.y_rows, "sm_linear(C)");
    if (rc) return rc;
    return lin32_checked(a, stream, "sm_linear");
  }
  GemmArgs g; std::memset(&g, 0, sizeof(g));
  g.A = A; g.W = W; g.bias = bias; g.residual = residual; g.C = C;
  g.M = d->M; g.N = d->N; g.K = d->K; g.dtype = d->dtype; g.act = d->act;
  g.rope_cols = d->rope_cols; g.rope_dim = d->rope_dim; g.rope_seq = d->rope_seq; g.rope_base = d->rope_base;
  g.c_transposed = d->c_transposed; g.c_batch_rows = d->c_batch_rows; g.ldw = d->K;
  g.norm = d->norm; g.norm_eps = d->norm_eps; g.norm_gamma = d->norm_gamma; g.norm_beta = d->norm_beta;
  const int n_out = (d->act == SM_ACT_SWIGLU || d->act == SM_ACT_GEGLU) ? d->N / 2 : d->N;
  int rc = rows_of(a_map, d->M, d->K, d->K, &g.a_rows, "sm_linear(A)");
  if (rc == SM_ERR_UNSUPPORTED && a_map) {
    // K contiguous only in granules of 4 (an unfold), or not at all (a transposed operand read in place, one element
    // per load: correct, and as slow as Sec. 3.2.2 says a sub-optimal read is): separable row + column programs
    std::string err;
    if (d->K % 4 == 0 && a_map->compile_rows_cols(4, &g.a_rows, &g.a_cols, &err)) g.a_gran = 4;
    else if (a_map->compile_rows_cols(1, &g.a_rows, &g.a_cols, &err)) g.a_gran = 1;
    else return fail(SM_ERR_UNSUPPORTED, "sm_linear(A): %s", err.c_str());
    rc = SM_OK;
  }
  if (rc) return rc;
  if (d->c_transposed && c_map) return fail(SM_ERR_UNSUPPORTED, "sm_linear: transposed store with a row map");
  rc = rows_of(c_map, d->M, n_out, n_out, &g.c_rows, "sm_linear(C)");
  if (rc == SM_ERR_UNSUPPORTED && c_map) {
    // the store splits the column dimension (e.g. into heads): separable row + column programs
    std::string err;
    // (in granules of one 16-byte vector when the split keeps them whole, else per element)
    const int vec = d->dtype == SM_F32 ? 4 : 8;
    g.c_gran = vec;
    if (!c_map->compile_rows_cols(vec, &g.c_rows, &g.c_cols, &err)) {
      g.c_gran = 1;
      if (!c_map->compile_rows_cols(1, &g.c_rows, &g.c_cols, &err)) return fail(SM_ERR_UNSUPPORTED, "sm_linear(C): %s", err.c_str());
    }
    g.c_cols_on = 1;
    rc = SM_OK;
  }
  if (rc) return rc;
  return gemm_checked(g, stream, "sm_linear");
}

namespace sm {
int mlp_checked(MlpArgs& a, void* stream, const char* who) {
  if (!mlp_fused_supported(a.C, a.Hd, SM_BF16)) return fail(SM_ERR_UNSUPPORTED, "%s: no fused MLP kernel for C = %d, hidden = %d", who, a.C, a.Hd);
  if (a.M < 0) return fail(SM_ERR_SHAPE, "%s: negative row count", who);
  if (a.norm != 0 && a.norm != 1) return fail(SM_ERR_INVALID_ARG, "%s: unknown norm %d", who, a.norm);
  if (a.M == 0) return SM_OK;
  if (!a.X || !a.Wp || !a.b1 || !a.b2 || !a.Y) return fail(SM_ERR_INVALID_ARG, "%s: null pointer", who);
  if (!aligned16(a.X) || !aligned16(a.Wp) || !aligned16(a.b1) || !aligned16(a.b2) || !aligned16(a.Y) || (a.residual && !aligned16(a.residual)))
    return fail(SM_ERR_INVALID_ARG, "%s: pointers must be 16-byte aligned", who);
  if (a.norm) {
    if (!a.norm_gamma || !a.norm_beta || !aligned16(a.norm_gamma) || !aligned16(a.norm_beta))
      return fail(SM_ERR_INVALID_ARG, "%s: folded LayerNorm needs 16-byte aligned gamma and beta", who);
    if (!(a.norm_eps > 0.f)) return fail(SM_ERR_INVALID_ARG, "%s: folded LayerNorm needs eps > 0", who);
  }
  if (a.Wproj_p) {
    if (!mlp_proj_supported(a.C, a.Hd, SM_BF16)) return fail(SM_ERR_UNSUPPORTED, "%s: projection + MLP does not fit the LDS for C = %d, hidden = %d", who, a.C, a.Hd);
    if (!a.bproj || !a.resid0 || !aligned16(a.Wproj_p) || !aligned16(a.bproj) || !aligned16(a.resid0))
      return fail(SM_ERR_INVALID_ARG, "%s: the fused projection needs 16-byte aligned packed weight, bias and residual", who);
  }
  if (a.Y2 && (!a.ln2_gamma || !a.ln2_beta || !aligned16(a.Y2) || !aligned16(a.ln2_gamma) || !aligned16(a.ln2_beta) || !(a.ln2_eps > 0.f)))
    return fail(SM_ERR_INVALID_ARG, "%s: the second (normalised) output needs 16-byte aligned output, gamma, beta and eps > 0", who);
  if (a.Wq_p && (!a.Wproj_p || !a.Y2 || !a.bq || !aligned16(a.Wq_p) || !aligned16(a.bq) || a.Hd < 3 * a.C))
    return fail(SM_ERR_INVALID_ARG, "%s: the following Linear needs the fused projection, the normalised output's arguments, a 16-byte aligned packed weight and bias, and hidden >= 3 C", who);
  if ((a.M + 31) / 32 > 0x7fffffff) return fail(SM_ERR_SHAPE, "%s: too many rows", who);
  char label[96];
  std::snprintf(label, sizeof label, "%s%smlp_bf16[%lld,%d,%d]%s", a.Wproj_p ? "proj+" : "", a.norm ? "ln+" : "", (long long)a.M, a.Hd, a.C,
                a.Wq_p ? "+ln+qkv" : (a.Y2 ? "+ln" : ""));
  Timed tm(label, stream);
  const int rc = launch_mlp_fused(a, stream);
  if (rc) return fail(SM_ERR_DEVICE, "%s: launch failed (hip error %d)", who, rc);
  count_compute(1);
  return SM_OK;
}
}  // namespace sm

extern "C" int sm_mlp_fused_supported(int C, int hidden, int dtype) { return sm::mlp_fused_supported(C, hidden, dtype) ? 1 : 0; }
extern "C" int sm_mlp_proj_supported(int C, int hidden, int dtype) { return sm::mlp_proj_supported(C, hidden, dtype) ? 1 : 0; }

extern "C" int sm_mlp_pack(const void* W1, const void* W2, int C, int hidden, int dtype, void* packed, void* stream) {
  if (!dtype_ok(dtype)) return fail(SM_ERR_INVALID_ARG, "sm_mlp_pack: unknown dtype");
  if (!sm::mlp_fused_supported(C, hidden, dtype)) return fail(SM_ERR_UNSUPPORTED, "sm_mlp_pack: no fused MLP kernel for C = %d, hidden = %d, dtype %d", C, hidden, dtype);
  if (!W1 || !W2 || !packed) return fail(SM_ERR_INVALID_ARG, "sm_mlp_pack: null pointer");
  if (!aligned16(W1) || !aligned16(W2) || !aligned16(packed)) return fail(SM_ERR_INVALID_ARG, "sm_mlp_pack: pointers must be 16-byte aligned");
  Timed tm("mlp_pack", stream);
  const int rc = launch_mlp_pack(W1, W2, C, hidden, packed, stream);
  if (rc) return fail(SM_ERR_DEVICE, "sm_mlp_pack: launch failed (hip error %d)", rc);
  return SM_OK;
}

extern "C" int sm_mlp_fused(const sm_mlp_desc* d, const void* X, const void* packed, const void* b1, const void* b2,
                            const void* residual, void* Y, const sm_map* x_map, const sm_map* y_map, void* stream) {
  if (!d) return fail(SM_ERR_INVALID_ARG, "sm_mlp_fused: null descriptor");
  if (!dtype_ok(d->dtype)) return fail(SM_ERR_INVALID_ARG, "sm_mlp_fused: unknown dtype");
  if (!sm::mlp_fused_supported(d->C, d->hidden, d->dtype))
    return fail(SM_ERR_UNSUPPORTED, "sm_mlp_fused: no kernel for C = %d, hidden = %d, dtype %d", d->C, d->hidden, d->dtype);
  MlpArgs a; std::memset(&a, 0, sizeof(a));
  a.X = X; a.Wp = packed; a.b1 = b1; a.b2 = b2; a.residual = residual; a.Y = Y; a.M = d->M; a.C = d->C; a.Hd = d->hidden;
  a.norm = d->norm; a.norm_eps = d->norm_eps; a.norm_gamma = d->norm_gamma; a.norm_beta = d->norm_beta;
  a.Wproj_p = d->proj_packed; a.bproj = d->proj_bias; a.resid0 = d->proj_residual;
  int rc = rows_of(x_map, d->M, d->C, d->C, &a.x_rows, "sm_mlp_fused(X)");
  if (rc) return rc;
  rc = rows_of(y_map, d->M, d->C, d->C, &a.y_rows, "sm_mlp_fused(Y)");
  if (rc) return rc;
  return mlp_checked(a, stream, "sm_mlp_fused");
}

extern "C" int sm_attention(const sm_attention_desc* d, const void* q, const void* k, const void* v, void* o,
                            const void* rpb_table, void* stream) {
  if (!d) return fail(SM_ERR_INVALID_ARG, "sm_attention: null descriptor");
  return attention_checked(*d, q, k, v, o, rpb_table, stream, "sm_attention");
}

extern "C" int sm_linear_autotune(const sm_linear_desc* d, const void* A, const void* W, const void* bias, const void* residual,
                                  void* C, int iters, void* stream, int* tile_rows, int* stages, float* best_us, float* default_us) {
  if (!d || !tile_rows || !stages || !best_us || !default_us) return fail(SM_ERR_INVALID_ARG, "sm_linear_autotune: null pointer");
  if (iters < 1 || iters > 1000) return fail(SM_ERR_INVALID_ARG, "sm_linear_autotune: iters must be 1..1000");
  if (d->w_packed || d->norm || d->c_transposed) return fail(SM_ERR_UNSUPPORTED, "sm_linear_autotune: the plain tiled Linear only (no packed weight, folded norm or transposed store)");
  // one ordinary, fully checked call first: bad arguments are refused here and nothing below runs on them
  int rc = sm_linear(d, A, W, bias, residual, C, nullptr, nullptr, stream);
  if (rc) return rc;
  GemmArgs g; std::memset(&g, 0, sizeof(g));
  g.A = A; g.W = W; g.bias = bias; g.residual = residual; g.C = C;
  g.M = d->M; g.N = d->N; g.K = d->K; g.dtype = d->dtype; g.act = d->act;
  g.rope_cols = d->rope_cols; g.rope_dim = d->rope_dim; g.rope_seq = d->rope_seq; g.rope_base = d->rope_base; g.ldw = d->K;
  const int n_out = (d->act == SM_ACT_SWIGLU || d->act == SM_ACT_GEGLU) ? d->N / 2 : d->N;
  g.a_rows = identity_rows(d->K); g.c_rows = identity_rows(n_out);
  rc = sm::gemm_autotune(g, iters, stream, tile_rows, stages, best_us, default_us);
  if (rc == -2) { *tile_rows = *stages = 0; *best_us = *default_us = 0.f; return SM_OK; }      // a shape with one variant: nothing to choose
  if (rc) return fail(SM_ERR_DEVICE, "sm_linear_autotune: timing failed (hip error %d)", rc);
  return SM_OK;
}
extern "C" void sm_linear_autotune_clear(void) { sm::gemm_autotune_clear(); }

extern "C" int sm_gemm_tuning(int tile_rows, int stages) {
  if (sm::gemm_tuning(tile_rows, stages)) return sm::fail(SM_ERR_INVALID_ARG, "sm_gemm_tuning: tile_rows must be 0, 64, 128 or 256 and stages 0 or 2..4");
  return SM_OK;
}

extern "C" int sm_timing_calibrate(int n, void* stream) {
  if (n < 1 || n > 1024) return sm::fail(SM_ERR_INVALID_ARG, "sm_timing_calibrate: n must be 1..1024");
  for (int i = 0; i < n; ++i) { sm::Timed tm("empty_pair", stream); }
  for (int i = 0; i < n; ++i) {
    sm::Timed tm("empty_kernel", stream);
    const int rc = sm::launch_empty(stream);
    if (rc) return sm::fail(SM_ERR_DEVICE, "sm_timing_calibrate: launch failed (hip error %d)", rc);
  }
  return SM_OK;
}
