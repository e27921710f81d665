// Per-row offset tables of compiled row programs: the composed index map of paper Sec. 3.2.1 evaluated once per
// call by a small kernel, into the caller's workspace, instead of once per row inside every kernel of the chain.
#include <cstdint>
#include <cstdio>
#include "common.h"
#include "index_map.h"
#include "kernels.h"

namespace sm {

void TableRegion::add(RowProg* p, int64_t n_rows, int64_t src_numel) {
  p->table = nullptr;
  p->table_off = 0;
  if (p->identity || n_rows <= 0 || src_numel > INT32_MAX) return;     // kernels interpret the program
  p->table_off = (int64_t)bytes + 1;
  items.push_back({*p, n_rows, bytes});
  bytes += ((size_t)n_rows * sizeof(int32_t) + 255) & ~(size_t)255;
}

int fill_tables(const TableRegion& r, void* region, void* stream, uint64_t which) {
  for (size_t i = 0; i < r.items.size(); ++i) {
    if (i < 64 && !((which >> i) & 1)) continue;
    const auto& it = r.items[i];
    char label[48];
    snprintf(label, sizeof(label), "fill_row_table[%lld]", (long long)it.n_rows);
    Timed tm(label, stream);
    const int rc = launch_fill_rows(it.prog, it.n_rows, (int32_t*)((char*)region + it.off), stream);
    if (rc) return fail(SM_ERR_DEVICE, "row-table fill kernel launch failed (hip error %d)", rc);
  }
  return SM_OK;
}

}  // namespace sm
