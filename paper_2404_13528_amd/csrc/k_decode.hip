// Kernels of a decode step (one new token per sequence against a key / value cache; the paper's decoder-only
// workload, Pythia, Table 7, at its memory-bound end).  With at most 32 tokens every Linear is a matrix-vector
// product bound by the stream of its weights from HBM, so the three kernels here are built around that stream:
//
//  * the weights are read in MFMA-fragment order (packed once by launch_lin_pack: fragment (slice, step) is 1 KiB
//    contiguous in lane order; Sec. 3.2.2's rule that a producer writes what its consumer reads best, applied to
//    constants), every wave-load is one fully used 1 KiB run, and a 32 x 32 x 16 MFMA per fragment forms the products
//    for all (up to 32) tokens at once: the matrix core is idle most of the time and costs nothing;
//  * a slice of 32 output features is split along K over the waves of a workgroup (and, for the output kernel, over
//    workgroups); partial sums meet in LDS (and, across workgroups, in a small fp32 buffer summed by the workgroup
//    that arrives last: a counter per slice, no waiting anywhere, every order of arrival gives the same sum order);
//  * the layout operators of the step are addresses of these kernels' loads and stores: the query / key / value
//    Slices and Permutes and the Concat behind the cache are the store of the first kernel (the new key / value row
//    goes straight to position L of the cache), the head merge is the store of the attention kernel.
#include <atomic>
#include "device_common.h"
#include "kernels.h"

namespace sm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 dc_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float dc_f32x16;
typedef unsigned int dc_u32x4 __attribute__((ext_vector_type(4)));

constexpr int DC_PF = 8;       // weight fragments in flight per wave

__device__ __forceinline__ void dc_unpack8(dc_u32x4 v, float* f) {
#pragma unroll
  for (int e = 0; e < 4; ++e) { f[2 * e] = __uint_as_float(v[e] << 16); f[2 * e + 1] = __uint_as_float(v[e] & 0xffff0000u); }
}
__device__ __forceinline__ float dc_load_f32(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// true in exactly one workgroup per counter: the one whose increment is the n-th.  Everything the workgroup stored
// before the call is visible to the workgroup that gets `true` (release before the increment, acquire after it).
__device__ __forceinline__ bool dc_arrived_last(int* counter, int n, int* flag_lds) {
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) *flag_lds = (atomicAdd(counter, 1) == n - 1);
  __syncthreads();
  const bool last = *flag_lds != 0;
  if (last) __threadfence();
  return last;
}

// acc += sum over steps k in [k0, k1) of W-fragment(k) x activation-fragment(k): two register sets of DC_PF fragments
// each, one being consumed while the other is in flight (loads past the end re-read the last step, their products are
// formed with a zero operand).
template <bool XG, class WL, class XL>
__device__ __forceinline__ void dc_stream(int k0, int k1, WL wl, XL xl, dc_f32x16& acc) {
  if (k0 >= k1) return;
  const dc_u32x4 zero = {0u, 0u, 0u, 0u};
  dc_u32x4 wa[DC_PF], xa[DC_PF], wb[DC_PF], xb[DC_PF];
#pragma unroll
  for (int i = 0; i < DC_PF; ++i) { const int k = min(k0 + i, k1 - 1); wa[i] = wl(k); xa[i] = xl(k); }
  for (int kk = k0; kk < k1; kk += 2 * DC_PF) {
#pragma unroll
    for (int i = 0; i < DC_PF; ++i) { const int k = min(kk + DC_PF + i, k1 - 1); wb[i] = wl(k); xb[i] = xl(k); }
#pragma unroll
    for (int i = 0; i < DC_PF; ++i)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(dc_bf16x8, wa[i]), __builtin_bit_cast(dc_bf16x8, kk + i < k1 ? xa[i] : zero), acc, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < DC_PF; ++i) { const int k = min(kk + 2 * DC_PF + i, k1 - 1); wa[i] = wl(k); xa[i] = xl(k); }
#pragma unroll
    for (int i = 0; i < DC_PF; ++i)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(dc_bf16x8, wb[i]), __builtin_bit_cast(dc_bf16x8, kk + DC_PF + i < k1 ? xb[i] : zero), acc, 0, 0, 0);
    // issue order as written: a set's loads together, then the other set's products
#pragma unroll
    for (int rep = 0; rep < 2; ++rep) {
      __builtin_amdgcn_sched_group_barrier(0x020, XG ? 2 * DC_PF : DC_PF, 0);
      if (!XG) __builtin_amdgcn_sched_group_barrier(0x100, DC_PF, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, DC_PF, 0);
    }
  }
}

// ---------------------------------------------------------------------------------------------------------------
// First kernel: [q | k | v] = LayerNorm-1(x) . Wqkv^T + bqkv with the rotary embedding on the first `rot` features of
// every query and key head, and hid = GELU(LayerNorm-2(x) . W1^T + b1): the two Linears that depend on x alone
// (parallel residual), one launch.  A workgroup owns 64 consecutive output features (two slices of 32) so that both
// members of a rotary pair (i, i + rot/2), rot/2 <= 32, are in the same workgroup; eight waves: slice = wave / 4,
// K quarter = wave % 4.
__global__ __launch_bounds__(512) void decode_in_kernel(DecodeInArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char dc_smem[];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, l32 = lane & 31, hf = lane >> 5;
  const int B = a.B, E = a.E;
  const int pitch = E + 8;                                          // elements: rows 16 bytes apart modulo the banks
  bf16_t* xs = (bf16_t*)dc_smem;                                    // [B][pitch] normalised x
  float* red = (float*)(dc_smem + (size_t)B * pitch * 2);           // [8 waves][32 rows][B]
  float* vals = red + 8 * 32 * B;                                   // [64 rows][B]
  if (blockIdx.x == 0) for (int i = tid; i < a.n_counters; i += 512) a.counters[i] = 0;
  const int n0 = blockIdx.x * 64;
  const bool fc1 = n0 >= 3 * E;
  const bf16_t* gam = fc1 ? a.ln2_g : a.ln1_g;
  const bf16_t* bet = fc1 ? a.ln2_b : a.ln1_b;
  // LayerNorm of the tokens this workgroup needs (all of them), two-pass statistics, bf16 result in LDS
  for (int b = w; b < B; b += 8) {
    const bf16_t* xr = a.x + (int64_t)b * E;
    float f[8], s = 0.f;
    for (int c = lane; c < E / 8; c += 64) {
      dc_unpack8(*(const dc_u32x4*)(xr + 8 * c), f);
#pragma unroll
      for (int e = 0; e < 8; ++e) s += f[e];
    }
    const float mean = wave_sum(s) / (float)E;
    s = 0.f;
    for (int c = lane; c < E / 8; c += 64) {
      dc_unpack8(*(const dc_u32x4*)(xr + 8 * c), f);
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float dlt = f[e] - mean; s = fmaf(dlt, dlt, s); }
    }
    const float rstd = rsqrtf(wave_sum(s) / (float)E + a.eps);
    for (int c = lane; c < E / 8; c += 64) {
      float g[8], bt[8];
      dc_unpack8(*(const dc_u32x4*)(xr + 8 * c), f);
      dc_unpack8(*(const dc_u32x4*)(gam + 8 * c), g);
      dc_unpack8(*(const dc_u32x4*)(bet + 8 * c), bt);
      bf16_t* o = xs + (size_t)b * pitch + 8 * c;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = f2bf(fmaf((f[e] - mean) * rstd, g[e], bt[e]));
    }
  }
  __syncthreads();
  // the wave's K quarter of its slice
  const int KS = E / 16, per = (KS + 3) / 4;
  const int k0 = (w & 3) * per, k1 = min(KS, k0 + per);
  const int slice = (fc1 ? (n0 - 3 * E) : n0) / 32 + (w >> 2);
  const dc_u32x4* wp = (const dc_u32x4*)(fc1 ? a.w1_p_ : a.wqkv_p_) + (int64_t)slice * KS * 64 + lane;
  const unsigned char* xl = (const unsigned char*)xs + (size_t)min(l32, B - 1) * pitch * 2 + hf * 16;
  dc_f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  dc_stream<false>(k0, k1, [&](int k) { return wp[(int64_t)k * 64]; }, [&](int k) { return *(const dc_u32x4*)(xl + (size_t)k * 32); }, acc);
  if (l32 < B) {
#pragma unroll
    for (int i = 0; i < 16; ++i) red[(w * 32 + (i / 4) * 8 + hf * 4 + (i & 3)) * B + l32] = acc[i];
  }
  __syncthreads();
  const bf16_t* bias = fc1 ? a.b1 : a.bqkv;
  for (int idx = tid; idx < 64 * B; idx += 512) {
    const int r = idx / B, b = idx - r * B, s4 = (r >> 5) * 4, rr = r & 31;
    float v = bf2f(bias[(fc1 ? n0 - 3 * E : n0) + r]);
#pragma unroll
    for (int p = 0; p < 4; ++p) v += red[((s4 + p) * 32 + rr) * B + b];
    vals[idx] = v;
  }
  __syncthreads();
  for (int idx = tid; idx < 64 * B; idx += 512) {
    const int r = idx / B, b = idx - r * B;
    float v = vals[idx];
    if (fc1) {
      v = 0.5f * v * (1.f + erff(v * 0.70710678118654752f));
      a.hid[(int64_t)b * a.F + (n0 - 3 * E) + r] = f2bf(v);
    } else {
      const int n = n0 + r, d = a.d, hh = n / (3 * d), rem = n - hh * 3 * d, t = rem / d, e = rem - t * d;
      if (t < 2 && e < a.rot) {                                   // rotary pair (i, i + rot/2) at position L
        const int half = a.rot >> 1, i = e < half ? e : e - half;
        const float other = vals[(e < half ? r + half : r - half) * B + b];
        const double ang = (double)a.L * exp2(-2.0 * (double)i / (double)a.rot * log2((double)a.rope_base));
        const float c = (float)cos(ang), s = (float)sin(ang);
        v = e < half ? v * c - other * s : v * c + other * s;
      }
      a.dst[t][(int64_t)b * a.dst_b[t] + (int64_t)hh * a.dst_h[t] + e] = f2bf(v);
    }
  }
}

// ---------------------------------------------------------------------------------------------------------------
// Attention of one query per (sequence, head) over n_keys cached tokens, keys split over gridDim.x workgroups.
// A key row (D elements) is read by D / 8 adjacent lanes, 16 bytes each, so one wave-load covers 512 / D whole
// rows; a lane keeps its eight query features in registers.  Scores go to LDS, the softmax of the chunk is taken
// there, and the value rows are accumulated per lane (its eight features, its share of the keys) without any exchange
// until the end.  Every workgroup leaves (max, sum, unnormalised output) in `part`; the one that arrives last for its
// (sequence, head) merges them and stores the output row.
template <int D>
__global__ __launch_bounds__(256) void decode_attn_kernel(DecodeAttnArgs a) {
  constexpr int LPK = D / 8, KPL = 64 / LPK, U = 4;
  extern __shared__ __attribute__((aligned(16))) unsigned char dc_smem[];
  float* sc = (float*)dc_smem;                                     // [chunk] scores, then probabilities
  __shared__ float s_red[4][D];
  __shared__ float s_w[8];
  __shared__ int s_flag;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lk = lane % LPK, kq = lane / LPK;
  const int bh = blockIdx.y, b = bh / a.h, hh = bh - b * a.h, split = blockIdx.x, nsplit = gridDim.x;
  const int chunk = (a.n_keys + nsplit - 1) / nsplit;
  const int t0 = split * chunk, t1 = min(a.n_keys, t0 + chunk), n = max(0, t1 - t0);
  const bf16_t* Kp = a.K + (int64_t)b * a.kv_b + (int64_t)hh * a.kv_h + 8 * lk;
  const bf16_t* Vp = a.V + (int64_t)b * a.kv_b + (int64_t)hh * a.kv_h + 8 * lk;
  float qf[8];
  dc_unpack8(*(const dc_u32x4*)(a.q + (int64_t)b * a.q_b + (int64_t)hh * a.q_h + 8 * lk), qf);
#pragma unroll
  for (int e = 0; e < 8; ++e) qf[e] *= a.scale_log2e;
  const int nit = (n + 4 * KPL - 1) / (4 * KPL);
  for (int it0 = 0; it0 < nit; it0 += U) {
    dc_u32x4 kv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int key = t0 + ((it0 + u) * 4 + w) * KPL + kq;
      kv[u] = key < t1 ? *(const dc_u32x4*)(Kp + (int64_t)key * D) : dc_u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int key = t0 + ((it0 + u) * 4 + w) * KPL + kq;
      float kf[8], dot = 0.f;
      dc_unpack8(kv[u], kf);
#pragma unroll
      for (int e = 0; e < 8; ++e) dot = fmaf(qf[e], kf[e], dot);
#pragma unroll
      for (int o = LPK / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
      if (lk == 0 && key < t1) sc[key - t0] = dot;
    }
  }
  __syncthreads();
  float m = -INFINITY;
  for (int i = tid; i < n; i += 256) m = fmaxf(m, sc[i]);
  m = wave_max(m);
  if (lane == 0) s_w[w] = m;
  __syncthreads();
  m = fmaxf(fmaxf(s_w[0], s_w[1]), fmaxf(s_w[2], s_w[3]));
  float l = 0.f;
  for (int i = tid; i < n; i += 256) { const float p = exp2f(sc[i] - m); sc[i] = p; l += p; }
  l = wave_sum(l);
  if (lane == 0) s_w[4 + w] = l;
  __syncthreads();
  l = (s_w[4] + s_w[5]) + (s_w[6] + s_w[7]);
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  for (int it0 = 0; it0 < nit; it0 += U) {
    dc_u32x4 vv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int key = t0 + ((it0 + u) * 4 + w) * KPL + kq;
      vv[u] = key < t1 ? *(const dc_u32x4*)(Vp + (int64_t)key * D) : dc_u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int key = t0 + ((it0 + u) * 4 + w) * KPL + kq;
      const float p = key < t1 ? sc[key - t0] : 0.f;
      float vf[8];
      dc_unpack8(vv[u], vf);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = fmaf(p, vf[e], acc[e]);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
#pragma unroll
    for (int o = LPK; o < 64; o <<= 1) acc[e] += __shfl_xor(acc[e], o, 64);
  }
  if (kq == 0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) s_red[w][8 * lk + e] = acc[e];
  }
  __syncthreads();
  float* part = a.part + ((int64_t)bh * nsplit + split) * (D + 2);
  if (tid < D) part[tid] = (s_red[0][tid] + s_red[1][tid]) + (s_red[2][tid] + s_red[3][tid]);
  if (tid == 0) { part[D] = m; part[D + 1] = l; }
  if (!dc_arrived_last(a.counters + bh, nsplit, &s_flag)) return;
  if (tid < D) {
    const float* p0 = a.part + (int64_t)bh * nsplit * (D + 2);
    float M = -INFINITY;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, dc_load_f32(p0 + (int64_t)s * (D + 2) + D));
    float o = 0.f, ls = 0.f;
    for (int s = 0; s < nsplit; ++s) {
      const float ms = dc_load_f32(p0 + (int64_t)s * (D + 2) + D);
      const float f = ms == -INFINITY ? 0.f : exp2f(ms - M);
      o = fmaf(f, dc_load_f32(p0 + (int64_t)s * (D + 2) + tid), o);
      ls = fmaf(f, dc_load_f32(p0 + (int64_t)s * (D + 2) + D + 1), ls);
    }
    a.o[(int64_t)b * a.o_b + (int64_t)hh * a.o_h + tid] = f2bf(o / ls);
  }
}

// ---------------------------------------------------------------------------------------------------------------
// Last kernel: y = x + bdense + b2 + Wdense . o + W2 . hid: one matrix-vector product over the concatenated reduction
// dimension E + F.  Grid (E / 32 slices, K splits); the activation fragments come straight from global memory (they
// are a few KB and stay in the caches), the partial sums of a workgroup go to `part`, and the workgroup that arrives
// last for its slice adds them up in split order, adds the biases and the residual and stores y.
__global__ __launch_bounds__(256) void decode_out_kernel(DecodeOutArgs a) {
  __shared__ float red[4 * 32 * 32];
  __shared__ int s_flag;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, l32 = lane & 31, hf = lane >> 5;
  const int B = a.B, E = a.E, F = a.F, slice = blockIdx.x, ks = blockIdx.y, nks = gridDim.y;
  const int KE = E / 16, KT = (E + F) / 16;
  const int per = (KT + nks - 1) / nks, g0 = min(KT, ks * per), g1 = min(KT, g0 + per);
  const int perw = (g1 - g0 + 3) / 4, k0 = min(g1, g0 + w * perw), k1 = min(g1, k0 + perw);
  const int tok = min(l32, B - 1);
  const dc_u32x4* wd = (const dc_u32x4*)a.wdense_p_ + (int64_t)slice * KE * 64 + lane;
  const dc_u32x4* w2 = (const dc_u32x4*)a.w2_p_ + (int64_t)slice * (KT - KE) * 64 + lane;
  const bf16_t* xo = a.o + (int64_t)tok * E + 8 * hf;
  const bf16_t* xh = a.hid + (int64_t)tok * F + 8 * hf;
  auto wfrag = [&](int k) -> dc_u32x4 { return k < KE ? wd[(int64_t)k * 64] : w2[(int64_t)(k - KE) * 64]; };
  auto xfrag = [&](int k) -> dc_u32x4 { return k < KE ? *(const dc_u32x4*)(xo + 16 * k) : *(const dc_u32x4*)(xh + 16 * (k - KE)); };
  dc_f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  dc_stream<true>(k0, k1, wfrag, xfrag, acc);
  if (l32 < B) {
#pragma unroll
    for (int i = 0; i < 16; ++i) red[(w * 32 + (i / 4) * 8 + hf * 4 + (i & 3)) * B + l32] = acc[i];
  }
  __syncthreads();
  for (int idx = tid; idx < 32 * B; idx += 256) {
    const int r = idx / B, b = idx - r * B;
    const float v = (red[(0 * 32 + r) * B + b] + red[(1 * 32 + r) * B + b]) + (red[(2 * 32 + r) * B + b] + red[(3 * 32 + r) * B + b]);
    a.part[((int64_t)ks * B + b) * E + slice * 32 + r] = v;
  }
  if (!dc_arrived_last(a.counters + slice, nks, &s_flag)) return;
  for (int idx = tid; idx < 32 * B; idx += 256) {
    const int b = idx >> 5, r = idx & 31, n = slice * 32 + r;
    float v = bf2f(a.bdense[n]) + bf2f(a.b2[n]);
    for (int s = 0; s < nks; ++s) v += dc_load_f32(a.part + ((int64_t)s * B + b) * E + n);
    a.y[(int64_t)b * E + n] = f2bf(v + bf2f(a.x[(int64_t)b * E + n]));
  }
}

// ---------------------------------------------------------------------------------------------------------------
// Explicit chain only: the Concat behind the cache as a copy, out[bh][t] = t < L ? cache[bh][t] : fresh[bh], rows of
// d elements in 16-byte vectors.
__global__ void decode_concat_kernel(const dc_u32x4* cache, int64_t cache_bh, const dc_u32x4* fresh, dc_u32x4* out, int L, int dv, int64_t total) {
  const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= total) return;
  const int c = (int)(o % dv);
  const int64_t row = o / dv;
  const int t = (int)(row % (L + 1));
  const int64_t bh = row / (L + 1);
  out[o] = t < L ? cache[bh * cache_bh + (int64_t)t * dv + c] : fresh[bh * dv + c];
}

size_t decode_in_smem(int B, int E) { return (size_t)B * (E + 8) * 2 + (size_t)(8 * 32 + 64) * B * 4; }

int launch_decode_in(const DecodeInArgs& a, void* stream) {
  const size_t smem = decode_in_smem(a.B, a.E);
  static std::atomic<size_t> allowed{0};
  if (smem > allowed.load()) {
    const hipError_t e = hipFuncSetAttribute((const void*)decode_in_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return (int)e;
    allowed.store(smem);
  }
  decode_in_kernel<<<dim3((unsigned)((3 * a.E + a.F) / 64)), dim3(512), smem, (hipStream_t)stream>>>(a);
  return (int)hipGetLastError();
}

int launch_decode_attn(const DecodeAttnArgs& a, int nsplit, void* stream) {
  const int chunk = (a.n_keys + nsplit - 1) / nsplit;
  const size_t smem = (size_t)chunk * 4;
  const dim3 grid((unsigned)nsplit, (unsigned)(a.B * a.h));
  switch (a.d) {
    case 64: decode_attn_kernel<64><<<grid, dim3(256), smem, (hipStream_t)stream>>>(a); break;
    case 128: decode_attn_kernel<128><<<grid, dim3(256), smem, (hipStream_t)stream>>>(a); break;
    case 256: decode_attn_kernel<256><<<grid, dim3(256), smem, (hipStream_t)stream>>>(a); break;
    default: return (int)hipErrorInvalidValue;
  }
  return (int)hipGetLastError();
}

int launch_decode_out(const DecodeOutArgs& a, int nks, void* stream) {
  decode_out_kernel<<<dim3((unsigned)(a.E / 32), (unsigned)nks), dim3(256), 0, (hipStream_t)stream>>>(a);
  return (int)hipGetLastError();
}

int launch_decode_concat(const void* cache, int64_t cache_bh_elems, const void* fresh, void* out, int BH, int L, int d, void* stream) {
  const int dv = d / 8;
  const int64_t total = (int64_t)BH * (L + 1) * dv;
  decode_concat_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(
      (const dc_u32x4*)cache, cache_bh_elems / 8, (const dc_u32x4*)fresh, (dc_u32x4*)out, L, dv, total);
  return (int)hipGetLastError();
}

}  // namespace sm
