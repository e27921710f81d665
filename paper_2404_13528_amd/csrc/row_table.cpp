// Per-row offset tables of compiled row programs (the composed index map of paper Sec. 3.2.1 evaluated once,
// when a plan is built, instead of once per row and kernel launch).
#include <hip/hip_runtime_api.h>
#include <cstdint>
#include <string>
#include <vector>
#include "index_map.h"

namespace sm {

bool attach_row_table(RowProg* p, int64_t n_rows, std::string* err) {
  p->table = nullptr;
  if (p->identity || n_rows <= 0) return true;
  std::vector<int32_t> host((size_t)n_rows);
  for (int64_t r = 0; r < n_rows; ++r) {
    const int64_t off = eval_rows_host(*p, r);
    if (off < 0 || off > INT32_MAX) return true;         // kernels fall back to interpreting the program
    host[(size_t)r] = (int32_t)off;
  }
  void* dev = nullptr;
  if (hipMalloc(&dev, host.size() * sizeof(int32_t)) != hipSuccess) { *err = "out of device memory for a row-offset table"; return false; }
  if (hipMemcpy(dev, host.data(), host.size() * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess) {
    (void)hipFree(dev);
    *err = "copy of a row-offset table to the device failed";
    return false;
  }
  p->table = (const int32_t*)dev;
  return true;
}

}  // namespace sm
