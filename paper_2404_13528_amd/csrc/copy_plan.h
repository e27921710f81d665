// One materialised layout transformation of an explicit-transpose chain (paper Sec. 2.2): compiled once per
// plan, launched as a copy kernel.  Where the last view axis stays contiguous in the source the copy moves whole
// rows through a per-row offset table; otherwise every vector goes through the full map program.
#pragma once
#include <cstdint>
#include <string>
#include <vector>
#include "index_map.h"

namespace sm {

struct Copy {
  MapProg prog; int64_t numel; int vec;      // general form: one map evaluation per vector of `vec` elements
  bool by_rows; RowProg rows; int64_t n_rows; int inner;   // row form: rows of `inner` contiguous elements
};

// tables: the region the copy's row-offset table gets a slot in
bool make_copy(const std::vector<int64_t>& src, const std::vector<sm_view_op>& chain, int esize, TableRegion* tables, Copy* out, std::string* err);
// dst = src gathered through the copy's map (+ addend, element-wise, when given); counts as one copy kernel.
// region: where `tables` was filled for this call
int copy_launch(const Copy& cp, const void* region, const void* src, void* dst, int dtype, void* stream, const void* addend = nullptr);

}  // namespace sm
