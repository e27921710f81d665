// View chains of the layout transformations in the supported operator chains,
// written as the operators a model exporter emits (Reshape, Transpose, Roll,
// Slice).  The composer folds each chain into one index map.
#pragma once
#include <vector>
#include "../../include/smartmem.h"

namespace sm { namespace chains {

inline sm_view_op reshape(std::initializer_list<int64_t> s) {
  sm_view_op v{}; v.kind = SM_VIEW_RESHAPE; v.n = (int)s.size(); int i = 0; for (auto x : s) v.arg[i++] = x; return v;
}
inline sm_view_op permute(std::initializer_list<int64_t> p) {
  sm_view_op v{}; v.kind = SM_VIEW_PERMUTE; v.n = (int)p.size(); int i = 0; for (auto x : p) v.arg[i++] = x; return v;
}
inline sm_view_op roll(int64_t axis, int64_t r) { sm_view_op v{}; v.kind = SM_VIEW_ROLL; v.n = 2; v.arg[0] = axis; v.arg[1] = r; return v; }
inline sm_view_op slice(int64_t axis, int64_t a, int64_t b) { sm_view_op v{}; v.kind = SM_VIEW_SLICE; v.n = 4; v.arg[0] = axis; v.arg[1] = a; v.arg[2] = b; v.arg[3] = 1; return v; }

// [B,H,W,C] -> roll both spatial axes
inline std::vector<sm_view_op> roll2(int64_t r) { return {roll(1, r), roll(2, r)}; }
// [B,H,W,C] -> [B*nW, w*w, C], cyclic shift by -s first
inline std::vector<sm_view_op> window_partition(int64_t B, int64_t H, int64_t W, int64_t C, int64_t w, int64_t s) {
  std::vector<sm_view_op> c;
  if (s) { c.push_back(roll(1, -s)); c.push_back(roll(2, -s)); }
  c.push_back(reshape({B, H / w, w, W / w, w, C}));
  c.push_back(permute({0, 1, 3, 2, 4, 5}));
  c.push_back(reshape({B * (H / w) * (W / w), w * w, C}));
  return c;
}
// [B*nW, w*w, C] -> [B,H,W,C], cyclic shift by +s afterwards
inline std::vector<sm_view_op> window_reverse(int64_t B, int64_t H, int64_t W, int64_t C, int64_t w, int64_t s) {
  std::vector<sm_view_op> c{reshape({B, H / w, W / w, w, w, C}), permute({0, 1, 3, 2, 4, 5}), reshape({B, H, W, C})};
  if (s) { c.push_back(roll(1, s)); c.push_back(roll(2, s)); }
  return c;
}
// [B_, N, 3*h*d] -> [3, B_, h, N, d]
inline std::vector<sm_view_op> qkv_split(int64_t B_, int64_t N, int64_t h, int64_t d) {
  return {reshape({B_, N, 3, h, d}), permute({2, 0, 3, 1, 4})};
}
// [B, S, h*d] -> [B, h, S, d] and back
inline std::vector<sm_view_op> head_split(int64_t B, int64_t S, int64_t h, int64_t d) { return {reshape({B, S, h, d}), permute({0, 2, 1, 3})}; }
inline std::vector<sm_view_op> head_merge(int64_t B, int64_t S, int64_t h, int64_t d) { return {permute({0, 2, 1, 3}), reshape({B, S, h * d})}; }
// [B,H,W,C] -> [B, H/2, W/2, 4C], channel block k = 2*dw + dh
inline std::vector<sm_view_op> patch_merge(int64_t B, int64_t H, int64_t W, int64_t C) {
  return {reshape({B, H / 2, 2, W / 2, 2, C}), permute({0, 1, 3, 4, 2, 5}), reshape({B, H / 2, W / 2, 4 * C})};
}
// NCHW image -> [B, (H/p)*(W/p), Cin*p*p], column order (c, py, px)
inline std::vector<sm_view_op> patch_embed(int64_t B, int64_t Cin, int64_t H, int64_t W, int64_t p) {
  return {reshape({B, Cin, H / p, p, W / p, p}), permute({0, 2, 4, 1, 3, 5}), reshape({B, (H / p) * (W / p), Cin * p * p})};
}
inline std::vector<sm_view_op> nchw_to_tokens(int64_t B, int64_t C, int64_t HW) { return {reshape({B, C, HW}), permute({0, 2, 1})}; }
inline std::vector<sm_view_op> tokens_to_nchw(int64_t B, int64_t C, int64_t H, int64_t W) { return {permute({0, 2, 1}), reshape({B, C, H, W})}; }

}}  // namespace sm::chains
