#include "copy_plan.h"
#include <cstdio>
#include "common.h"
#include "kernels.h"

namespace sm {

bool make_copy(const std::vector<int64_t>& src, const std::vector<sm_view_op>& chain, int esize, TableRegion* tables, Copy* out, std::string* err) {
  sm_map* m = nullptr;
  if (map_create(src, chain.data(), (int)chain.size(), &m, err) != SM_OK) return false;
  bool ok = m->compile(&out->prog, err);
  out->numel = m->numel();
  out->vec = map_vector_width(*m, esize);
  out->by_rows = false;
  const int64_t inner = m->shape.back();
  std::string why;
  // rows of at least one 16-byte vector whose start keeps the vector alignment
  if (ok && out->vec * esize == 16 && inner % out->vec == 0 && inner <= INT32_MAX && m->inner_contiguous((int)inner) &&
      m->compile_rows(&out->rows, &why)) {
    out->n_rows = out->numel / inner;
    out->inner = (int)inner;
    int64_t src_numel = 1;
    for (auto e : src) src_numel *= e;
    tables->add(&out->rows, out->n_rows, src_numel);
    out->by_rows = out->rows.identity || out->rows.table_off;
  }
  delete m;
  return ok;
}

int copy_launch(const Copy& cp, const void* region, const void* src, void* dst, int dtype, void* stream, const void* addend) {
  char label[64];
  snprintf(label, sizeof(label), "copy_%s[%lld]%s", dtype == SM_F32 ? "f32" : "bf16", (long long)cp.numel, addend ? "+add" : "");
  Timed tm(label, stream);
  int rc;
  if (cp.by_rows) rc = launch_gather_rows(bound(cp.rows, region), cp.n_rows, cp.inner, src, addend, dst, dtype, stream);
  else rc = addend ? launch_gather_add(cp.prog, cp.numel, cp.vec, src, addend, dst, dtype, stream)
                   : launch_gather(cp.prog, cp.numel, cp.vec, src, dst, (int)dtype_size(dtype), stream);
  if (rc) return fail(SM_ERR_DEVICE, "copy kernel launch failed (hip error %d)", rc);
  count_copy();
  return SM_OK;
}

}  // namespace sm
