// Device-side helpers: bf16 conversion, index-program evaluation, wave reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>
#include "index_map.h"

namespace sm {

typedef unsigned short bf16_t;     // raw bits

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((unsigned)v) << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {   // round to nearest even
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int VEC = 4;     // elements per 16 bytes
  __device__ static float ld(const float* p) { return *p; }
  __device__ static void st(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int VEC = 8;
  __device__ static float ld(const bf16_t* p) { return bf2f(*p); }
  __device__ static void st(bf16_t* p, float v) { *p = f2bf(v); }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// bf16 outputs: erf(x / sqrt 2) as an odd polynomial of degree 13 on the clamped argument (|error| < 1.4e-4, i.e.
// |GELU error| < 2.6e-4, a fifteenth of a bf16 ulp at 1): seven FMAs and no transcendental instruction
__device__ __forceinline__ float gelu_poly(float x) {
  const float xc = __builtin_amdgcn_fmed3f(x, -3.8183766f, 3.8183766f);
  const float u = xc * xc;
  float p = 7.157552710e-08f;
  p = fmaf(p, u, -4.470385145e-06f);
  p = fmaf(p, u, 1.201538955e-04f);
  p = fmaf(p, u, -1.853696382e-03f);
  p = fmaf(p, u, 1.859850362e-02f);
  p = fmaf(p, u, -1.313855874e-01f);
  p = fmaf(p, u, 7.973302013e-01f);
  const float hx = 0.5f * x;
  return fmaf(hx, p * xc, hx);
}

// value of atom list for one variable assignment; vars[] are the view indices
template <int NV>
__device__ __forceinline__ void eval_atoms(const ProgAtom* atoms, int n_atoms, const int* vars, int* val) {
  for (int i = 0; i < n_atoms; ++i) {
    const ProgAtom& a = atoms[i];
    int x = a.c0;
    for (int t = 0; t < a.nterm; ++t) {
      int id = a.t_atom[t];
      x += a.t_coef[t] * (id < 0 ? vars[~id] : val[id]);
    }
    if (a.div > 1) x = (int)(__umulhi((unsigned)x, a.div_mul) >> a.div_sh);
    if (a.mod > 1) x -= (int)(__umulhi((unsigned)x, a.mod_mul) >> a.mod_sh) * a.mod;
    else if (a.mod == 1) x = 0;
    val[i] = x;
  }
}

// Kernel arguments live in the constant kernarg segment.  Reading a large by-value argument through
// this pointer keeps dynamically indexed fields (the index programs) in scalar loads instead of a
// private copy.  The first explicit argument of a kernel starts at offset 0 of the segment.
#define SM_KARG __attribute__((address_space(4)))
template <typename Args>
__device__ __forceinline__ const SM_KARG Args* kernarg_ptr() { return (const SM_KARG Args*)__builtin_amdgcn_kernarg_segment_ptr(); }

// Atom values live in a 16-wide register vector indexed by wave-uniform ids taken from the kernarg segment, so
// the evaluation touches no scratch memory.
typedef int i32x16 __attribute__((ext_vector_type(16)));
__device__ __forceinline__ int64_t eval_rows_k(const SM_KARG RowProg* p, int64_t r) {
  if (p->identity) return r * p->ld;
  if (p->table) return (int64_t)p->table[r];          // evaluated when the plan was built
  i32x16 val = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  const int n = p->n_atoms;
  for (int i = 0; i < n; ++i) {
    const SM_KARG ProgAtom* a = &p->atoms[i];
    int x = a->c0;
    const int nt = a->nterm;
    for (int t = 0; t < nt; ++t) {
      const int id = a->t_atom[t];
      x += a->t_coef[t] * (id < 0 ? (int)r : val[id & 15]);
    }
    if (a->div > 1) x = (int)(__umulhi((unsigned)x, a->div_mul) >> a->div_sh);
    if (a->mod > 1) x -= (int)(__umulhi((unsigned)x, a->mod_mul) >> a->mod_sh) * a->mod;
    else if (a->mod == 1) x = 0;
    val[i & 15] = x;
  }
  int64_t off = p->c0;
  const int nt = p->nterm;
  for (int t = 0; t < nt; ++t) {
    const int id = p->t_atom[t];
    off += p->t_coef[t] * (int64_t)(id < 0 ? (int)r : val[id & 15]);
  }
  return off;
}

// Offset of one view element under a full map program (vars = view indices), register-resident like eval_rows_k.
typedef int i32x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ int64_t eval_map_k(const SM_KARG MapProg* p, i32x8 vars) {
  i32x16 val = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  const int n = p->n_atoms;
  for (int i = 0; i < n; ++i) {
    const SM_KARG ProgAtom* a = &p->atoms[i];
    int x = a->c0;
    const int nt = a->nterm;
    for (int t = 0; t < nt; ++t) {
      const int id = a->t_atom[t];
      x += a->t_coef[t] * (id < 0 ? vars[(~id) & 7] : val[id & 15]);
    }
    if (a->div > 1) x = (int)(__umulhi((unsigned)x, a->div_mul) >> a->div_sh);
    if (a->mod > 1) x -= (int)(__umulhi((unsigned)x, a->mod_mul) >> a->mod_sh) * a->mod;
    else if (a->mod == 1) x = 0;
    val[i & 15] = x;
  }
  int64_t off = p->c0;
  const int nt = p->nterm;
  for (int t = 0; t < nt; ++t) {
    const int id = p->t_atom[t];
    off += p->t_coef[t] * (int64_t)(id < 0 ? vars[(~id) & 7] : val[id & 15]);
  }
  return off;
}

// view multi-index of flat vector index o (last axis counted in vectors of `vec` elements)
__device__ __forceinline__ i32x8 unflatten_k(const SM_KARG MapProg* p, int64_t o, int vec) {
  i32x8 vars = {0, 0, 0, 0, 0, 0, 0, 0};
  const int rank = p->rank;
  int64_t rem = o;
  for (int k = rank - 1; k >= 0; --k) {
    int ext = p->shape[k];
    if (k == rank - 1) ext /= vec;
    const int64_t qd = rem / ext;
    vars[k & 7] = (int)(rem - qd * ext) * (k == rank - 1 ? vec : 1);
    rem = qd;
  }
  return vars;
}

__device__ __forceinline__ int64_t eval_rows(const RowProg& p, int64_t r) {
  if (p.identity) return r * p.ld;
  int val[PROG_MAX_ATOMS];
  int vars[1] = {(int)r};
  eval_atoms<1>(p.atoms, p.n_atoms, vars, val);
  int64_t off = p.c0;
  for (int t = 0; t < p.nterm; ++t) {
    int id = p.t_atom[t];
    off += p.t_coef[t] * (int64_t)(id < 0 ? vars[0] : val[id]);
  }
  return off;
}

}  // namespace sm
