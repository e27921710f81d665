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
