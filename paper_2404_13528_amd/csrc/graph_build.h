// Small builder of operator graphs (sm_tensor_desc / sm_op_desc arrays) used by
// the block executors to describe their chain to sm_layout_plan in the explicit
// form a model exporter produces: one operator per Reshape, Transpose, Roll,
// Slice, bias add, activation and residual add.
#pragma once
#include <string>
#include <vector>
#include "../../include/smartmem.h"

namespace sm {

struct GraphB {
  std::vector<sm_tensor_desc> tensors;
  std::vector<sm_op_desc> ops;
  std::vector<std::string> names;

  int tensor(std::initializer_list<int64_t> shape) { return tensor(std::vector<int64_t>(shape)); }
  int tensor(const std::vector<int64_t>& shape) {
    sm_tensor_desc t{}; t.rank = (int)shape.size();
    for (size_t i = 0; i < shape.size(); ++i) t.shape[i] = shape[i];
    tensors.push_back(t);
    return (int)tensors.size() - 1;
  }
  std::vector<int64_t> shape(int t) const { return std::vector<int64_t>(tensors[t].shape, tensors[t].shape + tensors[t].rank); }
  int op(int kind, std::vector<int> ins, const std::vector<int64_t>& out_shape, const char* name, std::vector<int64_t> attr = {}) {
    sm_op_desc o{}; o.kind = kind; o.n_in = (int)ins.size();
    for (size_t i = 0; i < ins.size(); ++i) o.in[i] = ins[i];
    o.out = tensor(out_shape);
    o.n_attr = (int)attr.size();
    for (size_t i = 0; i < attr.size(); ++i) o.attr[i] = attr[i];
    ops.push_back(o); names.push_back(name);
    return o.out;
  }
  int find(const std::string& name) const { for (size_t i = 0; i < names.size(); ++i) if (names[i] == name) return (int)i; return -1; }
  int reshape(int t, std::vector<int64_t> s) { return op(SM_OP_RESHAPE, {t}, s, "reshape"); }
  int transpose(int t, std::vector<int64_t> perm) {
    std::vector<int64_t> in = shape(t), out(perm.size());
    for (size_t i = 0; i < perm.size(); ++i) out[i] = in[perm[i]];
    return op(SM_OP_TRANSPOSE, {t}, out, "transpose", perm);
  }
  int roll(int t, int64_t axis, int64_t shift) { return op(SM_OP_ROLL, {t}, shape(t), "roll", {axis, shift}); }
  int slice(int t, int64_t axis, int64_t a, int64_t b) {
    std::vector<int64_t> s = shape(t); s[axis] = b - a;
    return op(SM_OP_SLICE, {t}, s, "slice", {axis, a, b, 1});
  }
  int linear(int t, int64_t n_out, const char* name, bool bias) {
    std::vector<int64_t> s = shape(t); s.back() = n_out;
    int y = op(SM_OP_MATMUL, {t}, s, name, {(int64_t)s.size() - 1});
    if (bias) y = op(SM_OP_BIAS, {y}, s, "bias");
    return y;
  }
};

}  // namespace sm
