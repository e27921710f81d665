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

// as few launches as the packed programs allow: a batch takes up to FILL_MAX_JOBS tables / FILL_MAX_WORDS words
int TableFiller::flush() {
  if (b_.n_jobs == 0) return SM_OK;
  char label[48];
  snprintf(label, sizeof(label), "fill_row_tables[%d]", b_.n_jobs);
  Timed tm(label, stream_);
  const int rc = launch_fill_batch(b_, stream_);
  b_.n_jobs = 0; b_.total_blocks = 0; used_ = 0;
  return rc ? fail(SM_ERR_DEVICE, "row-table fill kernel launch failed (hip error %d)", rc) : (int)SM_OK;
}
int TableFiller::add(const TableRegion& r, void* region, uint64_t which) {
  int rc;
  for (size_t i = 0; i < r.items.size(); ++i) {
    if (i < 64 && !((which >> i) & 1)) continue;
    const auto& it = r.items[i];
    int32_t* dst = (int32_t*)((char*)region + it.off);
    if (it.n_rows >= (1LL << 31) - 256) return fail(SM_ERR_SHAPE, "row-offset table of %lld rows", (long long)it.n_rows);
    int n = b_.n_jobs < FILL_MAX_JOBS ? fill_pack(it.prog, b_.words + used_, FILL_MAX_WORDS - used_) : -1;
    if (n < 0) {                                          // batch full: start another one
      if ((rc = flush())) return rc;
      n = fill_pack(it.prog, b_.words, FILL_MAX_WORDS);
    }
    if (n < 0) {                                          // a program too long for the packed form: a launch of its own
      char label[48];
      snprintf(label, sizeof(label), "fill_row_table[%lld]", (long long)it.n_rows);
      Timed tm(label, stream_);
      const int lrc = launch_fill_rows(it.prog, it.n_rows, dst, stream_);
      if (lrc) return fail(SM_ERR_DEVICE, "row-table fill kernel launch failed (hip error %d)", lrc);
      continue;
    }
    const int j = b_.n_jobs++;
    b_.dst[j] = (int64_t)(intptr_t)dst; b_.n_rows[j] = (int32_t)it.n_rows; b_.first_block[j] = b_.total_blocks; b_.word_off[j] = used_;
    b_.total_blocks += (int32_t)((it.n_rows + 255) / 256);
    used_ += n;
  }
  return SM_OK;
}
int fill_tables(const TableRegion& r, void* region, void* stream, uint64_t which) {
  TableFiller f(stream);
  const int rc = f.add(r, region, which);
  return rc ? rc : f.flush();
}

}  // namespace sm
