// out[o] = in[map(o)]: the materialised form of an eliminated layout
// transformation (paper Sec. 2.2 "explicit" transformations; Sec. 3.2.1 folds
// them into index computation instead).  One thread per vector of `vec`
// consecutive view elements along the last axis; the host guarantees that the
// map moves such vectors as a whole (unit stride, no // or % on the last axis
// finer than vec, aligned offsets).
#include "device_common.h"
#include "kernels.h"

namespace sm {

template <typename V>
__global__ __launch_bounds__(256) void gather_kernel(MapProg p, int64_t nvec, int vec, const V* __restrict__ src, V* __restrict__ dst) {
  int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= nvec) return;
  const SM_KARG MapProg* pk = kernarg_ptr<MapProg>();        // p is the first argument
  const int64_t off = eval_map_k(pk, unflatten_k(pk, o, vec));
  dst[o] = src[off / vec];
}

// dst[o] = src[map(o)] + addend[o]: the last copy of an explicit chain fused with the residual Add that follows it.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void gather_add_kernel(MapProg p, int64_t nvec, const T* __restrict__ src, const T* __restrict__ addend, T* __restrict__ dst) {
  int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= nvec) return;
  const SM_KARG MapProg* pk = kernarg_ptr<MapProg>();        // p is the first argument
  const int64_t off = eval_map_k(pk, unflatten_k(pk, o, VEC));
  struct alignas(sizeof(T) * VEC) Pack { T v[VEC]; };
  const Pack a = *(const Pack*)(src + off), b = *(const Pack*)(addend + o * VEC);
  Pack r;
#pragma unroll
  for (int e = 0; e < VEC; ++e) Elem<T>::st(&r.v[e], Elem<T>::ld(&a.v[e]) + Elem<T>::ld(&b.v[e]));
  *(Pack*)(dst + o * VEC) = r;
}

// Row form: one thread per 16-byte vector; the row's source offset comes from the row program (one table word
// per row once the plan has attached its table), the position inside the row is plain arithmetic.
template <typename T, bool ADD>
__global__ __launch_bounds__(256) void gather_rows_kernel(RowProg rows, int64_t nvec, int vpr, unsigned vpr_mul, unsigned vpr_sh,
                                                          const T* __restrict__ src, const T* __restrict__ addend, T* __restrict__ dst) {
  constexpr int VEC = Elem<T>::VEC;
  const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= nvec) return;
  const SM_KARG RowProg* pk = kernarg_ptr<RowProg>();        // rows is the first argument
  // o < 2^31 vectors (checked by the launcher): row = o / vpr by multiplication
  const unsigned r = vpr == 1 ? (unsigned)o : (__umulhi((unsigned)o, vpr_mul) >> vpr_sh);
  const unsigned c = (unsigned)o - r * (unsigned)vpr;
  const int64_t off = eval_rows_k(pk, (int64_t)r) + (int64_t)c * VEC;
  typedef unsigned int v4 __attribute__((ext_vector_type(4)));
  v4 a = *(const v4*)(src + off);
  if (ADD) {
    const v4 b = *(const v4*)(addend + o * VEC);
    if constexpr (VEC == 8) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float lo = __uint_as_float(a[e] << 16) + __uint_as_float(b[e] << 16);
        const float hi = __uint_as_float(a[e] & 0xffff0000u) + __uint_as_float(b[e] & 0xffff0000u);
        a[e] = (unsigned)f2bf(lo) | ((unsigned)f2bf(hi) << 16);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) a[e] = __float_as_uint(__uint_as_float(a[e]) + __uint_as_float(b[e]));
    }
  }
  *(v4*)(dst + o * VEC) = a;
}

int launch_gather_rows(const RowProg& rows, int64_t n_rows, int inner, const void* src, const void* addend, void* dst, int dtype, void* stream) {
  const int vec = dtype == SM_F32 ? 4 : 8;
  const int vpr = inner / vec;
  const int64_t nvec = n_rows * vpr;
  if (nvec == 0) return 0;
  if (nvec >= (1LL << 31)) return (int)hipErrorInvalidValue;
  unsigned mul = 0, sh = 0;
  magic(vpr, &mul, &sh);
  dim3 grid((unsigned)((nvec + 255) / 256)), block(256);
  hipStream_t s = (hipStream_t)stream;
  if (dtype == SM_F32) {
    if (addend) gather_rows_kernel<float, true><<<grid, block, 0, s>>>(rows, nvec, vpr, mul, sh, (const float*)src, (const float*)addend, (float*)dst);
    else gather_rows_kernel<float, false><<<grid, block, 0, s>>>(rows, nvec, vpr, mul, sh, (const float*)src, (const float*)addend, (float*)dst);
  } else {
    if (addend) gather_rows_kernel<bf16_t, true><<<grid, block, 0, s>>>(rows, nvec, vpr, mul, sh, (const bf16_t*)src, (const bf16_t*)addend, (bf16_t*)dst);
    else gather_rows_kernel<bf16_t, false><<<grid, block, 0, s>>>(rows, nvec, vpr, mul, sh, (const bf16_t*)src, (const bf16_t*)addend, (bf16_t*)dst);
  }
  return (int)hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_rows_kernel(RowProg prog, int64_t n_rows, int32_t* __restrict__ table) {
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_rows) return;
  table[r] = (int32_t)eval_rows_k(kernarg_ptr<RowProg>(), r);      // prog is the first argument; its own table is null
}
int launch_fill_rows(const RowProg& prog, int64_t n_rows, int32_t* table, void* stream) {
  if (n_rows <= 0) return 0;
  if (n_rows >= (1LL << 31)) return (int)hipErrorInvalidValue;
  RowProg p = prog;
  p.table = nullptr;
  fill_rows_kernel<<<dim3((unsigned)((n_rows + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(p, n_rows, table);
  return (int)hipGetLastError();
}

// packed program: [n_atoms, nterm, c0 lo, c0 hi], per atom [div, mod, c0, nterm, div_mul, div_sh, mod_mul, mod_sh,
// nterm x (t_atom, t_coef)], then nterm x (t_atom, coef lo, coef hi)
int fill_pack(const RowProg& p, int32_t* w, int room) {
  int n = 4;
  for (int i = 0; i < p.n_atoms; ++i) n += 8 + 2 * p.atoms[i].nterm;
  n += 3 * p.nterm;
  if (n > room) return -1;
  int o = 0;
  w[o++] = p.n_atoms; w[o++] = p.nterm; w[o++] = (int32_t)(uint32_t)(p.c0 & 0xffffffff); w[o++] = (int32_t)(p.c0 >> 32);
  for (int i = 0; i < p.n_atoms; ++i) {
    const ProgAtom& a = p.atoms[i];
    w[o++] = a.div; w[o++] = a.mod; w[o++] = a.c0; w[o++] = a.nterm;
    w[o++] = (int32_t)a.div_mul; w[o++] = (int32_t)a.div_sh; w[o++] = (int32_t)a.mod_mul; w[o++] = (int32_t)a.mod_sh;
    for (int t = 0; t < a.nterm; ++t) { w[o++] = a.t_atom[t]; w[o++] = a.t_coef[t]; }
  }
  for (int t = 0; t < p.nterm; ++t) { w[o++] = p.t_atom[t]; w[o++] = (int32_t)(uint32_t)(p.t_coef[t] & 0xffffffff); w[o++] = (int32_t)(p.t_coef[t] >> 32); }
  return o;
}
__global__ __launch_bounds__(256) void fill_batch_kernel(FillBatch b) {
  const SM_KARG FillBatch* bk = kernarg_ptr<FillBatch>();
  int job = 0;
  for (int j = 1; j < bk->n_jobs; ++j) if ((int)blockIdx.x >= bk->first_block[j]) job = j;       // wave-uniform
  const int64_t r = (int64_t)((int)blockIdx.x - bk->first_block[job]) * 256 + threadIdx.x;
  if (r >= bk->n_rows[job]) return;
  const SM_KARG int32_t* w = bk->words + bk->word_off[job];
  const int n_atoms = w[0], nterm = w[1];
  int64_t off = (int64_t)(uint32_t)w[2] | ((int64_t)w[3] << 32);
  i32x16 val = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  int o = 4;
  for (int i = 0; i < n_atoms; ++i) {
    const int div = w[o], mod = w[o + 1], nt = w[o + 3];
    int x = w[o + 2];
    const unsigned div_mul = (unsigned)w[o + 4], div_sh = (unsigned)w[o + 5], mod_mul = (unsigned)w[o + 6], mod_sh = (unsigned)w[o + 7];
    o += 8;
    for (int t = 0; t < nt; ++t) {
      const int id = w[o + 2 * t];
      x += w[o + 2 * t + 1] * (id < 0 ? (int)r : val[id & 15]);
    }
    o += 2 * nt;
    if (div > 1) x = (int)(__umulhi((unsigned)x, div_mul) >> div_sh);
    if (mod > 1) x -= (int)(__umulhi((unsigned)x, mod_mul) >> mod_sh) * mod;
    else if (mod == 1) x = 0;
    val[i & 15] = x;
  }
  for (int t = 0; t < nterm; ++t) {
    const int id = w[o + 3 * t];
    const int64_t coef = (int64_t)(uint32_t)w[o + 3 * t + 1] | ((int64_t)w[o + 3 * t + 2] << 32);
    off += coef * (int64_t)(id < 0 ? (int)r : val[id & 15]);
  }
  ((int32_t*)bk->dst[job])[r] = (int32_t)off;
}
int launch_fill_batch(const FillBatch& b, void* stream) {
  if (b.n_jobs <= 0 || b.total_blocks <= 0) return 0;
  fill_batch_kernel<<<dim3((unsigned)b.total_blocks), dim3(256), 0, (hipStream_t)stream>>>(b);
  return (int)hipGetLastError();
}

__global__ void empty_kernel() {}
int launch_empty(void* stream) {
  empty_kernel<<<dim3(1), dim3(64), 0, (hipStream_t)stream>>>();
  return (int)hipGetLastError();
}

int launch_gather_add(const MapProg& prog, int64_t numel, int vec_elems, const void* src, const void* addend, void* dst, int dtype, void* stream) {
  if (numel == 0) return 0;
  const int64_t nvec = numel / vec_elems;
  dim3 grid((unsigned)((nvec + 255) / 256)), block(256);
  hipStream_t s = (hipStream_t)stream;
#define GA(T, V) gather_add_kernel<T, V><<<grid, block, 0, s>>>(prog, nvec, (const T*)src, (const T*)addend, (T*)dst)
  if (dtype == SM_F32) { if (vec_elems == 4) GA(float, 4); else if (vec_elems == 2) GA(float, 2); else GA(float, 1); }
  else { if (vec_elems == 8) GA(bf16_t, 8); else if (vec_elems == 4) GA(bf16_t, 4); else if (vec_elems == 2) GA(bf16_t, 2); else GA(bf16_t, 1); }
#undef GA
  return (int)hipGetLastError();
}

// Concat along the last axis: out [rows, 2 * cv] = [a [rows, cv] | b [rows, cv]], cv in 16-byte vectors
__global__ __launch_bounds__(256) void concat2_cols_kernel(const uint4* __restrict__ a, const uint4* __restrict__ b, uint4* __restrict__ out,
                                                           int cv, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int64_t r = i / (2 * cv);
  const int c = (int)(i - r * 2 * cv);
  out[i] = c < cv ? a[r * cv + c] : b[r * cv + c - cv];
}
int launch_concat2_cols(const void* a, const void* b, void* out, int64_t rows, int cols_bytes, void* stream) {
  const int cv = cols_bytes / 16;
  const int64_t total = rows * 2 * cv;
  if (total == 0) return 0;
  concat2_cols_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>((const uint4*)a, (const uint4*)b, (uint4*)out, cv, total);
  return (int)hipGetLastError();
}

int launch_gather(const MapProg& prog, int64_t numel, int vec_elems, const void* src, void* dst, int esize, void* stream) {
  if (numel == 0) return 0;
  int64_t nvec = numel / vec_elems;
  dim3 grid((unsigned)((nvec + 255) / 256)), block(256);
  hipStream_t s = (hipStream_t)stream;
  int bytes = vec_elems * esize;
  if (bytes == 16) gather_kernel<uint4><<<grid, block, 0, s>>>(prog, nvec, vec_elems, (const uint4*)src, (uint4*)dst);
  else if (bytes == 8) gather_kernel<uint2><<<grid, block, 0, s>>>(prog, nvec, vec_elems, (const uint2*)src, (uint2*)dst);
  else if (bytes == 4) gather_kernel<uint32_t><<<grid, block, 0, s>>>(prog, nvec, vec_elems, (const uint32_t*)src, (uint32_t*)dst);
  else gather_kernel<uint16_t><<<grid, block, 0, s>>>(prog, nvec, vec_elems, (const uint16_t*)src, (uint16_t*)dst);
  return (int)hipGetLastError();
}

}  // namespace sm
