// Strided [B, h, S, d] views of attention operands, taken from the planned load / store maps (Sec. 3.2.1: the
// eliminated Reshape / Transpose / Slice run of an operand is the address expression of the consumer's load).
#pragma once
#include <cstdint>
#include <string>
#include "graph_build.h"

namespace sm {
struct View4 { int64_t base; int64_t stride[3]; };      // element offset of (b, hh, s, 0) = base + b*stride[0] + hh*stride[1] + s*stride[2]
// operand `slot` of operator `op`: its planned load map (looking through element-wise operators fused into the
// producer), or the natural layout of the tensor it reads
bool plan_operand_view(const sm_plan* plan, const GraphB& g, int op, int slot, View4* v, std::string* err);
bool plan_output_view(const sm_plan* plan, const GraphB& g, int op, View4* v, std::string* err);
}  // namespace sm
