// C ABI of the index-map composer and of sm_gather_mapped.
#include <cstring>
#include <vector>
#include "common.h"
#include "index_map.h"
#include "kernels.h"

using namespace sm;

extern "C" int sm_map_create(const sm_tensor_desc* src, const sm_view_op* chain, int n, sm_map** out) {
  if (!src || !out || n < 0 || (n > 0 && !chain)) return fail(SM_ERR_INVALID_ARG, "sm_map_create: null argument");
  if (src->rank < 1 || src->rank > SM_MAX_RANK) return fail(SM_ERR_INVALID_ARG, "sm_map_create: rank %d out of range", src->rank);
  std::vector<int64_t> shape(src->shape, src->shape + src->rank);
  std::string err;
  int rc = map_create(shape, chain, n, out, &err);
  if (rc != SM_OK) set_error("sm_map_create: %s", err.c_str());
  return rc;
}

extern "C" int sm_map_compose(const sm_map* inner, const sm_map* outer, sm_map** out) {
  if (!inner || !outer || !out) return fail(SM_ERR_INVALID_ARG, "sm_map_compose: null argument");
  if (outer->src_shape != inner->shape) return fail(SM_ERR_SHAPE, "sm_map_compose: outer's source shape differs from inner's view shape");
  std::vector<sm_view_op> chain = inner->chain;
  chain.insert(chain.end(), outer->chain.begin(), outer->chain.end());
  std::string err;
  int rc = map_create(inner->src_shape, chain.data(), (int)chain.size(), out, &err);
  if (rc != SM_OK) set_error("sm_map_compose: %s", err.c_str());
  return rc;
}

extern "C" int sm_map_rank(const sm_map* m) { return m ? (int)m->shape.size() : SM_ERR_INVALID_ARG; }
extern "C" int sm_map_shape(const sm_map* m, int64_t* shape) {
  if (!m || !shape) return fail(SM_ERR_INVALID_ARG, "sm_map_shape: null argument");
  for (size_t k = 0; k < m->shape.size(); ++k) shape[k] = m->shape[k];
  return SM_OK;
}
extern "C" int64_t sm_map_numel(const sm_map* m) { return m ? m->numel() : SM_ERR_INVALID_ARG; }
extern "C" int sm_map_cost(const sm_map* m, int* n_divmod, int* n_raw) {
  if (!m) return fail(SM_ERR_INVALID_ARG, "sm_map_cost: null map");
  if (n_divmod) *n_divmod = m->n_divmod();
  if (n_raw) *n_raw = m->n_divmod_raw;
  return SM_OK;
}
extern "C" int sm_map_eval_host(const sm_map* m, int64_t* offsets, int64_t n) {
  if (!m || !offsets) return fail(SM_ERR_INVALID_ARG, "sm_map_eval_host: null argument");
  if (n != m->numel()) return fail(SM_ERR_SHAPE, "sm_map_eval_host: n = %lld, map has %lld elements", (long long)n, (long long)m->numel());
  m->eval(offsets);
  return SM_OK;
}
extern "C" int sm_map_affine(const sm_map* m, int64_t* base, int64_t* strides) {
  if (!m || !base || !strides) return fail(SM_ERR_INVALID_ARG, "sm_map_affine: null argument");
  return m->affine(base, strides) ? 1 : 0;
}
extern "C" void sm_map_destroy(sm_map* m) { delete m; }

namespace sm {
// largest power-of-two vector (in elements, <= 16 bytes) the map moves as a whole
int map_vector_width(const sm_map& m, int esize) {
  for (int v = 16 / esize; v > 1; v >>= 1)
    if (m.inner_contiguous(v)) return v;
  return 1;
}
}  // namespace sm

extern "C" int sm_gather_mapped(const sm_map* m, const void* src, void* dst, int dtype, int on_device, void* stream) {
  if (m && m->numel() == 0) return SM_OK;                    // an empty view: nothing to move
  if (!m || !src || !dst) return fail(SM_ERR_INVALID_ARG, "sm_gather_mapped: null argument");
  if (!dtype_ok(dtype)) return fail(SM_ERR_INVALID_ARG, "sm_gather_mapped: unknown dtype %d", dtype);
  const int es = (int)dtype_size(dtype);
  const int64_t n = m->numel();
  if (!on_device) {
    std::vector<int64_t> off(n);
    m->eval(off.data());
    const char* s = (const char*)src; char* d = (char*)dst;
    for (int64_t o = 0; o < n; ++o) std::memcpy(d + o * es, s + off[o] * es, es);
    return SM_OK;
  }
  if (!aligned16(src) || !aligned16(dst)) return fail(SM_ERR_INVALID_ARG, "sm_gather_mapped: device pointers must be 16-byte aligned");
  MapProg prog; std::string err;
  if (!m->compile(&prog, &err)) return fail(SM_ERR_UNSUPPORTED, "sm_gather_mapped: %s", err.c_str());
  int64_t src_n = 1; for (auto s : m->src_shape) src_n *= s;
  if (src_n > INT32_MAX || n > (int64_t)INT32_MAX * 8) return fail(SM_ERR_UNSUPPORTED, "sm_gather_mapped: tensor exceeds 32-bit indexing");
  int rc = launch_gather(prog, n, map_vector_width(*m, es), src, dst, es, stream);
  if (rc) return fail(SM_ERR_DEVICE, "sm_gather_mapped: launch failed (hip error %d)", rc);
  count_copy();
  return SM_OK;
}

// Human-readable form of the simplified map ("i0, i1, ..." are the view indices).
static std::string affine_str(const sm_map* m, const Affine& a);
static std::string atom_str(const sm_map* m, int id) {
  const Atom& t = m->atoms[id];
  if (t.kind == ATOM_VAR) return "i" + std::to_string(t.var);
  std::string s = "(" + affine_str(m, t.arg) + ")";
  if (t.div > 1) s += " // " + std::to_string(t.div);
  if (t.mod > 0) s = "(" + s + ") % " + std::to_string(t.mod);
  return "(" + s + ")";
}
static std::string affine_str(const sm_map* m, const Affine& a) {
  std::string s;
  for (auto& t : a.terms) {
    if (!s.empty()) s += " + ";
    if (t.second != 1) s += std::to_string(t.second) + "*";
    s += atom_str(m, t.first);
  }
  if (a.c0 || s.empty()) s += (s.empty() ? "" : " + ") + std::to_string(a.c0);
  return s;
}
extern "C" int sm_map_describe(const sm_map* m, char* buf, int n) {
  if (!m || !buf || n < 1) return fail(SM_ERR_INVALID_ARG, "sm_map_describe: bad argument");
  std::string s = affine_str(m, m->offset);
  snprintf(buf, n, "%s", s.c_str());
  return SM_OK;
}
