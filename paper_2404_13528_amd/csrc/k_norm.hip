// LayerNorm / RMSNorm / GroupNorm / token mean: HBM-bound, one pass over the
// data, fp32 statistics with wavefront-shuffle reductions.  The row kernels
// read and write through row programs, so that a following or preceding
// layout transformation (window partition / reverse, cyclic roll, patch-merge
// gather) costs only address arithmetic (paper Sec. 3.2.1; LayerNorm is
// ILD & Variable in Table 3: its output layout is free to choose).
#include "device_common.h"
#include "kernels.h"

namespace sm {

template <typename T> struct Vec16;
template <> struct Vec16<float> { typedef float4 type; };
template <> struct Vec16<bf16_t> { typedef uint4 type; };

template <typename T>
__device__ __forceinline__ void unpack(const typename Vec16<T>::type& v, float* f);
template <>
__device__ __forceinline__ void unpack<float>(const float4& v, float* f) { f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w; }
template <>
__device__ __forceinline__ void unpack<bf16_t>(const uint4& v, float* f) {
  const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) { f[2 * i] = __uint_as_float(w[i] << 16); f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
}
template <typename T>
__device__ __forceinline__ typename Vec16<T>::type pack(const float* f);
template <>
__device__ __forceinline__ float4 pack<float>(const float* f) { return make_float4(f[0], f[1], f[2], f[3]); }
template <>
__device__ __forceinline__ uint4 pack<bf16_t>(const float* f) {
  unsigned w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) w[i] = (unsigned)f2bf(f[2 * i]) | ((unsigned)f2bf(f[2 * i + 1]) << 16);
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// Each wave owns RPW consecutive logical rows; lane l owns 16-byte chunks l, l+64, ... of each.  All loads
// of the wave's rows are issued before the first reduction, so several rows are in flight per lane.
template <typename T, int MAXCH, int RPW>
__global__ __launch_bounds__(256) void norm_rows_kernel(NormArgs a) {
  constexpr int VEC = Elem<T>::VEC;
  typedef typename Vec16<T>::type V;
  const SM_KARG NormArgs* ak = kernarg_ptr<NormArgs>();
  const int lane = threadIdx.x & 63;
  const int64_t row0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW;
  if (row0 >= a.rows) return;
  // The kernel-argument fields used below, read together and pinned in scalar registers: fetched where they are used
  // they cost one scalar load and one wait each, strung out by the branches between them, before the first data load.
#define SM_PIN(x) asm volatile("" : "+s"(x))
  int l_ident = a.load.identity, s_ident = a.store.identity, nseg = a.nseg, n_ch = a.C, rms = a.rms;
  int64_t n_rows = a.rows, l_ld = a.load.ld, s_ld = a.store.ld;
  const int32_t* l_tab = a.load.table;
  const int32_t* s_tab = a.store.table;
  float eps = a.eps;
  SM_PIN(l_ident); SM_PIN(s_ident); SM_PIN(nseg); SM_PIN(n_ch); SM_PIN(rms); SM_PIN(n_rows); SM_PIN(l_ld); SM_PIN(s_ld);
  SM_PIN(l_tab); SM_PIN(s_tab); SM_PIN(eps);
#undef SM_PIN
  const int nchunk = n_ch / VEC;
  const int seg_chunks = nchunk / nseg;
  const T* x = (const T*)a.x;
  // row offsets first.  With offset tables all lookups of the wave's rows (load and store side) are in flight together;
  // the index programs, where there is no table, are evaluated out of line before any data register is live.
  int64_t seg_off[RPW], out_off[RPW];
  int lt[RPW], st[RPW];
#pragma unroll
  for (int r = 0; r < RPW; ++r) {
    const int64_t row = min(row0 + r, n_rows - 1);          // a clamped duplicate row is computed and not stored
    const int64_t li = row * nseg + min(lane, nseg - 1);    // segment base offsets: lane j < nseg evaluates segment j, broadcast below
    if (l_ident) seg_off[r] = li * l_ld;
    else if (l_tab) lt[r] = l_tab[li];
    else seg_off[r] = eval_rows_k(&ak->load, li);
    if (s_ident) out_off[r] = row * s_ld;
    else if (s_tab) st[r] = s_tab[row];
    else out_off[r] = eval_rows_k(&ak->store, row);
  }
#pragma unroll
  for (int r = 0; r < RPW; ++r) {
    if (!l_ident && l_tab) seg_off[r] = (int64_t)lt[r];
    if (!s_ident && s_tab) out_off[r] = (int64_t)st[r];
  }
  float v[RPW][MAXCH][VEC];
  float sum[RPW];
#pragma unroll
  for (int r = 0; r < RPW; ++r) {
    const int64_t my_seg = seg_off[r];
    sum[r] = 0.f;
#pragma unroll
    for (int i = 0; i < MAXCH; ++i) {
      const int ch = lane + 64 * i;
      const int seg = ch < nchunk ? ch / seg_chunks : 0;
      const int64_t base = __shfl(my_seg, seg, 64);
      if (ch < nchunk) {
        V raw = *(const V*)(x + base + (int64_t)(ch - seg * seg_chunks) * VEC);
        unpack<T>(raw, v[r][i]);
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[r][i][e] = 0.f;
      }
    }
  }
  // gamma and beta ride along with the data loads instead of waiting behind the reductions
  const T* g = (const T*)a.gamma;
  const T* bta = (const T*)a.beta;
  V graw[MAXCH], braw[MAXCH];
#pragma unroll
  for (int i = 0; i < MAXCH; ++i) {
    const int ch = min(lane + 64 * i, nchunk - 1);
    graw[i] = *(const V*)(g + ch * VEC);
    braw[i] = *(const V*)((!rms && bta ? bta : g) + ch * VEC);
  }
  float mean[RPW], rstd[RPW];
#pragma unroll
  for (int r = 0; r < RPW; ++r) {
#pragma unroll
    for (int i = 0; i < MAXCH; ++i)
#pragma unroll
      for (int e = 0; e < VEC; ++e) sum[r] += v[r][i][e];
  }
#pragma unroll
  for (int r = 0; r < RPW; ++r) mean[r] = rms ? 0.f : wave_sum(sum[r]) / (float)n_ch;
#pragma unroll
  for (int r = 0; r < RPW; ++r) {
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < MAXCH; ++i)
      if (lane + 64 * i < nchunk) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) { const float dlt = v[r][i][e] - mean[r]; ss += dlt * dlt; }
      }
    sum[r] = ss;
  }
#pragma unroll
  for (int r = 0; r < RPW; ++r) rstd[r] = rsqrtf(wave_sum(sum[r]) / (float)n_ch + eps);
  T* y = (T*)a.y;
#pragma unroll
  for (int i = 0; i < MAXCH; ++i) {
    const int ch = lane + 64 * i;
    if (ch >= nchunk) continue;
    float gg[VEC], bb[VEC];
    unpack<T>(graw[i], gg);
    if (!rms && bta) unpack<T>(braw[i], bb);
    else {
#pragma unroll
      for (int e = 0; e < VEC; ++e) bb[e] = 0.f;
    }
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
      const int64_t row = row0 + r;
      if (row >= n_rows) continue;
      const int64_t obase = out_off[r];
      float o[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) o[e] = (v[r][i][e] - mean[r]) * rstd[r] * gg[e] + bb[e];
      *(V*)(y + obase + (int64_t)ch * VEC) = pack<T>(o);
    }
  }
}

// Rows of at most LPR 16-byte chunks (LPR = 16 or 32 lanes per row): 64 / LPR rows side by side in a wave, RPL such groups
// per wave one after the other; the statistics are sums over the LPR lanes of a row (DPP row operations, and one
// cross-row-of-16 exchange when LPR = 32).  One segment per row; the same row maps as norm_rows_kernel.
__device__ __forceinline__ float norm_sum16(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));      // xor 1
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));      // xor 2
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));     // mirror within 8
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));     // mirror within 16
  return v;
}
template <typename T, int LPR, int RPL>
__global__ __launch_bounds__(256) void norm_short_rows_kernel(NormArgs a) {
  constexpr int VEC = Elem<T>::VEC, RPP = 64 / LPR;      // rows per pass of the wave
  typedef typename Vec16<T>::type V;
  const SM_KARG NormArgs* ak = kernarg_ptr<NormArgs>();
  const int lane = threadIdx.x & 63, sub = lane / LPR, ch = lane % LPR;
  const int64_t row0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * (RPP * RPL);
  if (row0 >= a.rows) return;
  const int nchunk = a.C / VEC;
  const bool on = ch < nchunk;
  const T* x = (const T*)a.x;
  int64_t in_off[RPL], out_off[RPL];
  float v[RPL][VEC];
#pragma unroll
  for (int r = 0; r < RPL; ++r) {
    const int64_t row = min(row0 + r * RPP + sub, a.rows - 1);      // a clamped duplicate row is computed and not stored
    in_off[r] = a.load.identity ? row * a.load.ld : eval_rows_k(&ak->load, row);
    out_off[r] = a.store.identity ? row * a.store.ld : eval_rows_k(&ak->store, row);
  }
#pragma unroll
  for (int r = 0; r < RPL; ++r) {
    if (on) { V raw = *(const V*)(x + in_off[r] + (int64_t)ch * VEC); unpack<T>(raw, v[r]); }
    else {
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[r][e] = 0.f;
    }
  }
  const T* g = (const T*)a.gamma;
  const T* bta = (const T*)a.beta;
  float gg[VEC], bb[VEC];
  { V graw = *(const V*)(g + min(ch, nchunk - 1) * VEC); unpack<T>(graw, gg); }
  if (!a.rms && bta) { V braw = *(const V*)(bta + min(ch, nchunk - 1) * VEC); unpack<T>(braw, bb); }
  else {
#pragma unroll
    for (int e = 0; e < VEC; ++e) bb[e] = 0.f;
  }
  T* y = (T*)a.y;
#pragma unroll
  for (int r = 0; r < RPL; ++r) {
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < VEC; ++e) s += v[r][e];
    s = norm_sum16(s);
    if (LPR == 32) s += __shfl_xor(s, 16, 64);
    const float mean = a.rms ? 0.f : s / (float)a.C;
    float ss = 0.f;
    if (on) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) { const float d = v[r][e] - mean; ss += d * d; }
    }
    ss = norm_sum16(ss);
    if (LPR == 32) ss += __shfl_xor(ss, 16, 64);
    const float rstd = rsqrtf(ss / (float)a.C + a.eps);
    if (on && row0 + r * RPP + sub < a.rows) {
      float o[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) o[e] = (v[r][e] - mean) * rstd * gg[e] + bb[e];
      *(V*)(y + out_off[r] + (int64_t)ch * VEC) = pack<T>(o);
    }
  }
}

template <typename T>
static int norm_dispatch(const NormArgs& a, hipStream_t s) {
  constexpr int VEC = Elem<T>::VEC;
  const int nchunk = a.C / VEC;
  dim3 block(256);
  // short rows (one segment): several rows side by side in a wave instead of lanes without a chunk
  if (a.nseg == 1 && nchunk <= 16) norm_short_rows_kernel<T, 16, 2><<<dim3((unsigned)((a.rows + 31) / 32)), block, 0, s>>>(a);
  else if (a.nseg == 1 && nchunk <= 32) norm_short_rows_kernel<T, 32, 2><<<dim3((unsigned)((a.rows + 15) / 16)), block, 0, s>>>(a);
  else if (nchunk <= 64) norm_rows_kernel<T, 1, 2><<<dim3((unsigned)((a.rows + 7) / 8)), block, 0, s>>>(a);
  else if (nchunk <= 128) norm_rows_kernel<T, 2, 1><<<dim3((unsigned)((a.rows + 3) / 4)), block, 0, s>>>(a);
  else if (nchunk <= 256) norm_rows_kernel<T, 4, 1><<<dim3((unsigned)((a.rows + 3) / 4)), block, 0, s>>>(a);
  else norm_rows_kernel<T, 8, 1><<<dim3((unsigned)((a.rows + 3) / 4)), block, 0, s>>>(a);
  return (int)hipGetLastError();
}

int launch_norm(const NormArgs& a, void* stream) {
  if (a.rows == 0) return 0;
  return a.dtype == SM_F32 ? norm_dispatch<float>(a, (hipStream_t)stream) : norm_dispatch<bf16_t>(a, (hipStream_t)stream);
}

// ---- GroupNorm over NCHW: one workgroup per (image, group); the group's
// channels are one contiguous run of cpg*HW elements.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}

template <typename T>
__global__ __launch_bounds__(512) void groupnorm_kernel(GroupNormArgs a) {
  __shared__ float red[8];
  const int b = blockIdx.x / a.G, g = blockIdx.x % a.G;
  const int cpg = a.C / a.G;
  const int64_t n = (int64_t)cpg * a.HW;
  const T* x = (const T*)a.x + ((int64_t)b * a.C + (int64_t)g * cpg) * a.HW;
  float s = 0.f;
  for (int64_t i = threadIdx.x; i < n; i += blockDim.x) s += Elem<T>::ld(x + i);
  const float mean = block_sum(s, red) / (float)n;
  float ss = 0.f;
  for (int64_t i = threadIdx.x; i < n; i += blockDim.x) { float d = Elem<T>::ld(x + i) - mean; ss += d * d; }
  const float rstd = rsqrtf(block_sum(ss, red) / (float)n + a.eps);
  const T* gm = (const T*)a.gamma; const T* bt = (const T*)a.beta;
  T* y = (T*)a.y;
  if (!a.tokens_out) {
    T* yo = y + ((int64_t)b * a.C + (int64_t)g * cpg) * a.HW;
    for (int64_t i = threadIdx.x; i < n; i += blockDim.x) {
      const int c = g * cpg + (int)(i / a.HW);
      Elem<T>::st(yo + i, (Elem<T>::ld(x + i) - mean) * rstd * Elem<T>::ld(gm + c) + Elem<T>::ld(bt + c));
    }
  } else {
    // token-major store [B, HW, C]: thread per token, cpg adjacent channels each
    for (int t = threadIdx.x; t < a.HW; t += blockDim.x) {
      T* yo = y + ((int64_t)b * a.HW + t) * a.C + g * cpg;
      for (int c = 0; c < cpg; ++c) {
        const int cc = g * cpg + c;
        Elem<T>::st(yo + c, (Elem<T>::ld(x + (int64_t)c * a.HW + t) - mean) * rstd * Elem<T>::ld(gm + cc) + Elem<T>::ld(bt + cc));
      }
    }
  }
}

// ---- GroupNorm in two kernels (the caller provides scratch for the statistics): every CU takes part, all
// global accesses are 16-byte vectors, and the token-major store goes through an LDS transpose so that it writes
// whole token rows.
template <typename T>
__global__ __launch_bounds__(512) void gn_stats_kernel(GroupNormArgs a) {
  __shared__ float red[8];
  constexpr int VEC = Elem<T>::VEC;
  typedef typename Vec16<T>::type V;
  const int cpg = a.C / a.G;
  const int64_t nv = (int64_t)cpg * a.HW / VEC;                 // the group is one contiguous run of cpg * HW elements
  const V* x = (const V*)((const T*)a.x + (int64_t)blockIdx.x * cpg * a.HW);
  float s = 0.f;
  for (int64_t i = threadIdx.x; i < nv; i += blockDim.x) {
    float f[VEC];
    unpack<T>(x[i], f);
#pragma unroll
    for (int e = 0; e < VEC; ++e) s += f[e];
  }
  const float mean = block_sum(s, red) / (float)(nv * VEC);
  float ss = 0.f;
  for (int64_t i = threadIdx.x; i < nv; i += blockDim.x) {      // second pass over data that is in L2 by now
    float f[VEC];
    unpack<T>(x[i], f);
#pragma unroll
    for (int e = 0; e < VEC; ++e) { const float d = f[e] - mean; ss += d * d; }
  }
  const float var = block_sum(ss, red) / (float)(nv * VEC);
  if (threadIdx.x == 0) { a.stats[2 * blockIdx.x] = mean; a.stats[2 * blockIdx.x + 1] = rsqrtf(var + a.eps); }
}

// channel-major in, channel-major out: one thread per 16-byte vector
template <typename T>
__global__ __launch_bounds__(256) void gn_apply_nchw_kernel(GroupNormArgs a) {
  constexpr int VEC = Elem<T>::VEC;
  typedef typename Vec16<T>::type V;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int vpc = a.HW / VEC;                                   // vectors per channel
  if (i >= (int64_t)a.B * a.C * vpc) return;
  const int64_t bc = i / vpc;                                   // image * C + channel
  const int c = (int)(bc % a.C), b = (int)(bc / a.C);
  const int g = c / (a.C / a.G);
  const float mean = a.stats[2 * (b * a.G + g)], rstd = a.stats[2 * (b * a.G + g) + 1];
  const float ga = Elem<T>::ld((const T*)a.gamma + c) * rstd, be = Elem<T>::ld((const T*)a.beta + c) - mean * ga;
  float f[VEC];
  unpack<T>(((const V*)a.x)[i], f);
#pragma unroll
  for (int e = 0; e < VEC; ++e) f[e] = fmaf(f[e], ga, be);
  ((V*)a.y)[i] = pack<T>(f);
}

// channel-major in, token-major out: a workgroup owns TT tokens of one image, all channels
template <typename T, int TT>
__global__ __launch_bounds__(256) void gn_apply_tokens_kernel(GroupNormArgs a) {
  constexpr int VEC = Elem<T>::VEC;
  typedef typename Vec16<T>::type V;
  extern __shared__ __align__(16) unsigned char gn_lds[];
  T* tile = (T*)gn_lds;                                          // [TT][C + VEC]
  const int pitch = a.C + VEC;
  const int b = blockIdx.y, t0 = blockIdx.x * TT;
  const int cpg = a.C / a.G;
  constexpr int TV = TT / VEC;                                   // vectors per channel inside the tile
  const T* x = (const T*)a.x + (int64_t)b * a.C * a.HW;
  for (int p = threadIdx.x; p < a.C * TV; p += 256) {
    const int c = p / TV, tv = p - c * TV;
    const int t = t0 + tv * VEC;
    if (t >= a.HW) continue;                                     // HW is a multiple of VEC: a vector is inside or outside
    const int g = c / cpg;
    const float mean = a.stats[2 * (b * a.G + g)], rstd = a.stats[2 * (b * a.G + g) + 1];
    const float ga = Elem<T>::ld((const T*)a.gamma + c) * rstd, be = Elem<T>::ld((const T*)a.beta + c) - mean * ga;
    float f[VEC];
    unpack<T>(*(const V*)(x + (int64_t)c * a.HW + t), f);
#pragma unroll
    for (int e = 0; e < VEC; ++e) Elem<T>::st(tile + (tv * VEC + e) * pitch + c, fmaf(f[e], ga, be));
  }
  __syncthreads();
  const int cv = a.C / VEC;                                      // vectors per token row
  T* y = (T*)a.y + ((int64_t)b * a.HW + t0) * a.C;
  for (int p = threadIdx.x; p < TT * cv; p += 256) {
    const int t = p / cv, c8 = p - t * cv;
    if (t0 + t >= a.HW) break;
    *(V*)(y + (int64_t)t * a.C + c8 * VEC) = *(const V*)(tile + t * pitch + c8 * VEC);
  }
}

static bool groupnorm_split(const GroupNormArgs& a) {
  const int vec = a.dtype == SM_F32 ? 4 : 8;
  const size_t es = a.dtype == SM_F32 ? 4 : 2;
  return a.stats && a.HW % vec == 0 && a.C % vec == 0 && (size_t)32 * (a.C + vec) * es <= 160 * 1024;
}
int groupnorm_launches(const GroupNormArgs& a) { return groupnorm_split(a) ? 2 : 1; }

template <typename T>
static int groupnorm_split_launch(const GroupNormArgs& a, hipStream_t s) {
  constexpr int VEC = Elem<T>::VEC;
  gn_stats_kernel<T><<<dim3((unsigned)(a.B * a.G)), dim3(512), 0, s>>>(a);
  if (!a.tokens_out) {
    const int64_t nv = (int64_t)a.B * a.C * (a.HW / VEC);
    gn_apply_nchw_kernel<T><<<dim3((unsigned)((nv + 255) / 256)), dim3(256), 0, s>>>(a);
    return (int)hipGetLastError();
  }
  const size_t row = (size_t)(a.C + VEC) * sizeof(T);
  if (64 * row <= 160 * 1024) {
    const size_t smem = 64 * row;
    static size_t granted = 0;
    if (smem > granted) {
      const hipError_t e = hipFuncSetAttribute((const void*)gn_apply_tokens_kernel<T, 64>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      if (e != hipSuccess) return (int)e;
      granted = smem;
    }
    gn_apply_tokens_kernel<T, 64><<<dim3((unsigned)((a.HW + 63) / 64), (unsigned)a.B), dim3(256), smem, s>>>(a);
  } else {
    const size_t smem = 32 * row;
    static size_t granted = 0;
    if (smem > granted) {
      const hipError_t e = hipFuncSetAttribute((const void*)gn_apply_tokens_kernel<T, 32>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      if (e != hipSuccess) return (int)e;
      granted = smem;
    }
    gn_apply_tokens_kernel<T, 32><<<dim3((unsigned)((a.HW + 31) / 32), (unsigned)a.B), dim3(256), smem, s>>>(a);
  }
  return (int)hipGetLastError();
}

int launch_groupnorm(const GroupNormArgs& a, void* stream) {
  if (groupnorm_split(a)) return a.dtype == SM_F32 ? groupnorm_split_launch<float>(a, (hipStream_t)stream) : groupnorm_split_launch<bf16_t>(a, (hipStream_t)stream);
  dim3 grid((unsigned)(a.B * a.G)), block(512);
  if (a.dtype == SM_F32) groupnorm_kernel<float><<<grid, block, 0, (hipStream_t)stream>>>(a);
  else groupnorm_kernel<bf16_t><<<grid, block, 0, (hipStream_t)stream>>>(a);
  return (int)hipGetLastError();
}

// ---- mean over tokens: x [B, L, C] -> y [B, C]
template <typename T>
__global__ __launch_bounds__(256) void mean_tokens_kernel(const T* x, T* y, int L, int C) {
  const int b = blockIdx.y;
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= C) return;
  float s = 0.f;
  const T* p = x + (int64_t)b * L * C + c;
  for (int t = 0; t < L; ++t) s += Elem<T>::ld(p + (int64_t)t * C);
  Elem<T>::st(y + (int64_t)b * C + c, s / (float)L);
}

int launch_mean_tokens(const void* x, void* y, int B, int L, int C, int dtype, void* stream) {
  dim3 grid((unsigned)((C + 255) / 256), (unsigned)B), block(256);
  if (dtype == SM_F32) mean_tokens_kernel<float><<<grid, block, 0, (hipStream_t)stream>>>((const float*)x, (float*)y, L, C);
  else mean_tokens_kernel<bf16_t><<<grid, block, 0, (hipStream_t)stream>>>((const bf16_t*)x, (bf16_t*)y, L, C);
  return (int)hipGetLastError();
}

// ---- Reduce (sum), fp32 accumulation.  reduce_last: one wave per row of n contiguous elements (the reduction
// dimension innermost: 16-byte loads when the row length allows).  reduce_first: one thread per inner element,
// walking the outermost dimension (coalesced across threads, strided per thread).
template <typename T>
__global__ __launch_bounds__(256) void reduce_last_kernel(const T* __restrict__ x, T* __restrict__ y, int64_t rows, int n) {
  constexpr int VEC = Elem<T>::VEC;
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const T* p = x + r * n;
  float s = 0.f;
  if (n % VEC == 0) {
    typedef unsigned int v4 __attribute__((ext_vector_type(4)));
    for (int c = lane * VEC; c < n; c += 64 * VEC) {
      const v4 v = *(const v4*)(p + c);
      if constexpr (VEC == 8) {
#pragma unroll
        for (int e = 0; e < 4; ++e) s += __uint_as_float(v[e] << 16) + __uint_as_float(v[e] & 0xffff0000u);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) s += __uint_as_float(v[e]);
      }
    }
  } else {
    for (int c = lane; c < n; c += 64) s += Elem<T>::ld(p + c);
  }
  s = wave_sum(s);
  if (lane == 0) Elem<T>::st(y + r, s);
}
template <typename T>
__global__ __launch_bounds__(256) void reduce_first_kernel(const T* __restrict__ x, T* __restrict__ y, int n_outer, int64_t inner) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= inner) return;
  float s = 0.f;
  for (int o = 0; o < n_outer; ++o) s += Elem<T>::ld(x + (int64_t)o * inner + i);
  Elem<T>::st(y + i, s);
}
int launch_reduce_last(const void* x, void* y, int64_t rows, int n, int dtype, void* stream) {
  if (rows <= 0) return 0;
  dim3 grid((unsigned)((rows + 3) / 4)), block(256);
  if (dtype == SM_F32) reduce_last_kernel<float><<<grid, block, 0, (hipStream_t)stream>>>((const float*)x, (float*)y, rows, n);
  else reduce_last_kernel<bf16_t><<<grid, block, 0, (hipStream_t)stream>>>((const bf16_t*)x, (bf16_t*)y, rows, n);
  return (int)hipGetLastError();
}
int launch_reduce_first(const void* x, void* y, int n_outer, int64_t inner, int dtype, void* stream) {
  if (inner <= 0) return 0;
  dim3 grid((unsigned)((inner + 255) / 256)), block(256);
  if (dtype == SM_F32) reduce_first_kernel<float><<<grid, block, 0, (hipStream_t)stream>>>((const float*)x, (float*)y, n_outer, inner);
  else reduce_first_kernel<bf16_t><<<grid, block, 0, (hipStream_t)stream>>>((const bf16_t*)x, (bf16_t*)y, n_outer, inner);
  return (int)hipGetLastError();
}

}  // namespace sm
