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
#include <algorithm>
#include <atomic>
#include "device_common.h"
#include "kernels.h"

namespace sm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 dc_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float dc_f32x16;
typedef unsigned int dc_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int dc_u32x2 __attribute__((ext_vector_type(2)));

constexpr int DC_CNT_STRIDE = 64;   // ints between two arrival counters: one counter per 256 bytes, so that the
                                    // increments of different slices / heads do not queue up on one cache line
constexpr int DC_PF = 8;       // weight fragments per register set of a wave (two sets)
constexpr int DC_PF_IN = 8;    // the same in the first kernel: a wave's whole stream at E = 2048 is requested up front
constexpr int DC_ATTN_NIT = 4; // key rows (and value rows) a lane of the attention kernel holds

__device__ __forceinline__ void dc_unpack8(dc_u32x4 v, float* f) {
#pragma unroll
  for (int e = 0; e < 4; ++e) { f[2 * e] = __uint_as_float(v[e] << 16); f[2 * e + 1] = __uint_as_float(v[e] & 0xffff0000u); }
}
__device__ __forceinline__ float dc_load_f32(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

__device__ __forceinline__ void dc_store_f32(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// true in exactly one workgroup per counter: the one whose increment is the n-th.  The partial results a workgroup
// hands over are written with dc_store_f32 (device-scope stores that go through to memory) and read with dc_load_f32:
// once the wave's stores have completed (vmcnt 0) and the workgroup has met at the barrier, the increment can only be
// observed after them.  No cache write-back is involved: a release fence here would flush the L2 once per workgroup.
__device__ __forceinline__ bool dc_arrived_last(int* counter, int n, int* flag_lds) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) *flag_lds = (__hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n - 1);
  __syncthreads();
  const bool last = *flag_lds != 0;
  if (last) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  return last;
}

// The weight stream of one wave: steps k in [k0, k1) of a slice, fragment k at wp[k * 64] (this lane's 16 bytes).  Two
// register sets of DC_PF fragments.  dc_preload issues both sets' first loads (before the activation tile is ready, so
// that the prologue's latency and the first weights overlap); dc_consume forms acc += W(k) x X(k) for all steps,
// reloading a set right after the products that read it.  X fragments come from LDS: step k at xl + (k - kbase) * 32
// bytes.  Loads past the end re-read the last step and their products are formed with a zero operand.
template <int PF> struct DcSets { dc_u32x4 a[PF], b[PF]; };
template <int PF>
__device__ __forceinline__ void dc_preload(DcSets<PF>& f, const dc_u32x4* wp, int k0, int k1) {
  if (k0 >= k1) return;
#pragma unroll
  for (int i = 0; i < PF; ++i) f.a[i] = wp[(int64_t)min(k0 + i, k1 - 1) * 64];
#pragma unroll
  for (int i = 0; i < PF; ++i) f.b[i] = wp[(int64_t)min(k0 + PF + i, k1 - 1) * 64];
}
template <int PF>
__device__ __forceinline__ void dc_consume(DcSets<PF>& f, const dc_u32x4* wp, const unsigned char* xl, int kbase, int k0, int k1, dc_f32x16& acc) {
  if (k0 >= k1) return;
  const dc_u32x4 zero = {0u, 0u, 0u, 0u};
  for (int kk = k0; kk < k1; kk += 2 * PF) {
    dc_u32x4 x[PF];
#pragma unroll
    for (int i = 0; i < PF; ++i) x[i] = *(const dc_u32x4*)(xl + (size_t)(min(kk + i, k1 - 1) - kbase) * 32);
#pragma unroll
    for (int i = 0; i < PF; ++i)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(dc_bf16x8, f.a[i]), __builtin_bit_cast(dc_bf16x8, kk + i < k1 ? x[i] : zero), acc, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < PF; ++i) f.a[i] = wp[(int64_t)min(kk + 2 * PF + i, k1 - 1) * 64];
#pragma unroll
    for (int i = 0; i < PF; ++i) x[i] = *(const dc_u32x4*)(xl + (size_t)(min(kk + PF + i, k1 - 1) - kbase) * 32);
#pragma unroll
    for (int i = 0; i < PF; ++i)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(dc_bf16x8, f.b[i]), __builtin_bit_cast(dc_bf16x8, kk + PF + i < k1 ? x[i] : zero), acc, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < PF; ++i) f.b[i] = wp[(int64_t)min(kk + 3 * PF + i, k1 - 1) * 64];
    // issue order as written
#pragma unroll
    for (int rep = 0; rep < 2; ++rep) {
      __builtin_amdgcn_sched_group_barrier(0x100, PF, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, PF, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, PF, 0);
    }
  }
}

// cos and sin of position x theta_i, theta_i = base^(-2 i / rot): the angle in revolutions, its fraction to the hardware
__device__ __forceinline__ void dc_rope_cs(int pos, int i, int rot, float base, float* c, float* s) {
  const float rev = (float)pos * (exp2f(-2.f * (float)i / (float)rot * log2f(base)) * 0.15915494309189535f);
  const float f = __builtin_amdgcn_fractf(rev);
  *c = __builtin_amdgcn_cosf(f); *s = __builtin_amdgcn_sinf(f);
}

// ---------------------------------------------------------------------------------------------------------------
// First kernel: [q | k | v] = LayerNorm-1(x) . Wqkv^T + bqkv with the rotary embedding on the first `rot` features of
// every query and key head, and hid = GELU(LayerNorm-2(x) . W1^T + b1): the two Linears that depend on x alone
// (parallel residual), one launch.  A workgroup owns 64 consecutive output features (two slices of 32) so that both
// members of a rotary pair (i, i + rot/2), rot/2 <= 32, are in the same workgroup; eight waves: slice = wave / 4,
// K quarter = wave % 4.
template <int MAXP>      // 16-byte pieces of a token row per lane: E <= 512 MAXP
__global__ __launch_bounds__(512) void decode_in_kernel(DecodeInArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char dc_smem[];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, l32 = lane & 31, hf = lane >> 5;
  const int B = a.B, E = a.E;
  const int pitch = E + 8;                                          // elements: rows 16 bytes apart modulo the banks
  bf16_t* xs = (bf16_t*)dc_smem;                                    // [B][pitch] normalised x
  float* red = (float*)(dc_smem + (size_t)B * pitch * 2);           // [8 waves][32 rows][B]
  float* vals = red + 8 * 32 * B;                                   // [64 rows][B]
  if (blockIdx.x == 0) for (int i = tid; i < a.n_counters; i += 512) a.counters[i * DC_CNT_STRIDE] = 0;
  const int n0 = blockIdx.x * 64;
  const bool fc1 = n0 >= 3 * E;
  const bf16_t* gam = fc1 ? a.ln2_g : a.ln1_g;
  const bf16_t* bet = fc1 ? a.ln2_b : a.ln1_b;
  // the wave's K quarter of its slice; its first weight fragments are requested before anything else
  const int KS = E / 16, per = (KS + 3) / 4;
  const int k0 = (w & 3) * per, k1 = min(KS, k0 + per);
  const int slice = (fc1 ? (n0 - 3 * E) : n0) / 32 + (w >> 2);
  const dc_u32x4* wp = (const dc_u32x4*)(fc1 ? a.w1_p_ : a.wqkv_p_) + (int64_t)slice * KS * 64 + lane;
  constexpr int PFI = MAXP <= 4 ? DC_PF_IN : DC_PF;
  DcSets<PFI> fr;
  if constexpr (MAXP <= 4) dc_preload(fr, wp, k0, k1);      // long rows need the registers for the LayerNorm first
  // LayerNorm of the tokens this workgroup needs (all of them), two-pass statistics, bf16 result in LDS
  for (int b = w; b < B; b += 8) {                  // one load round trip: the row, gamma and beta requested together
    const bf16_t* xr = a.x + (int64_t)b * E;
    const int nch = E / 8;
    dc_u32x4 xv[MAXP], gv[MAXP], bv[MAXP];      // gv / bv hold one piece at a time when MAXP > 4
#pragma unroll
    for (int j = 0; j < MAXP; ++j) {
      const int c = lane + 64 * j;
      if (c < nch) {
        xv[j] = *(const dc_u32x4*)(xr + 8 * c);
        if constexpr (MAXP <= 4) { gv[j] = *(const dc_u32x4*)(gam + 8 * c); bv[j] = *(const dc_u32x4*)(bet + 8 * c); }
      }
    }
    float f[8], s = 0.f;
#pragma unroll
    for (int j = 0; j < MAXP; ++j) {
      if (lane + 64 * j < nch) {
        dc_unpack8(xv[j], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) s += f[e];
      }
    }
    const float mean = wave_sum(s) / (float)E;
    s = 0.f;
#pragma unroll
    for (int j = 0; j < MAXP; ++j) {
      if (lane + 64 * j < nch) {
        dc_unpack8(xv[j], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) { const float dlt = f[e] - mean; s = fmaf(dlt, dlt, s); }
      }
    }
    const float rstd = rsqrtf(wave_sum(s) / (float)E + a.eps);
#pragma unroll
    for (int j = 0; j < MAXP; ++j) {
      const int c = lane + 64 * j;
      if (c < nch) {
        float g[8], bt[8];
        if constexpr (MAXP > 4) { gv[j] = *(const dc_u32x4*)(gam + 8 * c); bv[j] = *(const dc_u32x4*)(bet + 8 * c); }      // long rows: registers go to x
        dc_unpack8(xv[j], f); dc_unpack8(gv[j], g); dc_unpack8(bv[j], bt);
        dc_u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          o[e] = (unsigned)f2bf(fmaf((f[2 * e] - mean) * rstd, g[2 * e], bt[2 * e])) | ((unsigned)f2bf(fmaf((f[2 * e + 1] - mean) * rstd, g[2 * e + 1], bt[2 * e + 1])) << 16);
        *(dc_u32x4*)(xs + (size_t)b * pitch + 8 * c) = o;
      }
    }
  }
  if constexpr (MAXP > 4) dc_preload(fr, wp, k0, k1);
  __syncthreads();
  const unsigned char* xl = (const unsigned char*)xs + (size_t)min(l32, B - 1) * pitch * 2 + hf * 16;
  dc_f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  dc_consume(fr, wp, xl, 0, k0, k1, acc);
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
        float c, s;
        dc_rope_cs(a.L, i, a.rot, a.rope_base, &c, &s);
        v = e < half ? v * c - other * s : v * c + other * s;
      }
      a.dst[t][(int64_t)b * a.dst_b[t] + (int64_t)hh * a.dst_h[t] + e] = f2bf(v);
    }
  }
}

// ---------------------------------------------------------------------------------------------------------------
// Attention of one query per (sequence, head) over n_keys cached tokens, the keys split over gridDim.x workgroups
// (equal shares of whole blocks of 4 waves x DC_ATTN_NIT x 4 keys).  A key row (D elements) is read by 16 adjacent
// lanes (one DPP row), D / 16 elements each in 16-byte pieces (8-byte for D = 64), so a wave-load covers four rows in
// runs of 256 bytes and the dot product's cross-lane sum is four DPP adds (no LDS traffic).  A lane keeps its query
// features in registers and holds the value rows of exactly the keys whose scores it ends up with (the reduction
// leaves a key's score in every lane of its row), so a wave runs its own online softmax over its keys with no LDS and
// no barrier: blocks of DC_ATTN_NIT key rows and value rows per lane, two register sets, one in flight while the
// other is consumed.  At the end the four waves merge through LDS, the workgroup leaves (max, sum, unnormalised
// output) in `part`, and the one that arrives last for its (sequence, head) merges the workgroups.
template <int D> struct DcRow;      // a lane's share of a key / value row: D / 16 elements
template <> struct DcRow<256> { dc_u32x4 p[2]; };
template <> struct DcRow<128> { dc_u32x4 p[1]; };
template <> struct DcRow<64> { dc_u32x2 p[1]; };
template <int D> __device__ __forceinline__ DcRow<D> dc_row_load(const bf16_t* row, int lk) {
  DcRow<D> r;
  if constexpr (D == 256) { r.p[0] = *(const dc_u32x4*)(row + 8 * lk); r.p[1] = *(const dc_u32x4*)(row + 128 + 8 * lk); }
  else if constexpr (D == 128) r.p[0] = *(const dc_u32x4*)(row + 8 * lk);
  else r.p[0] = *(const dc_u32x2*)(row + 4 * lk);
  return r;
}
// the lane's D / 16 features as floats, in the order element e of piece j
template <int D> __device__ __forceinline__ void dc_row_unpack(const DcRow<D>& r, float* f) {
  if constexpr (D == 256) { dc_unpack8(r.p[0], f); dc_unpack8(r.p[1], f + 8); }
  else if constexpr (D == 128) { dc_unpack8(r.p[0], f); }
  else {
#pragma unroll
    for (int e = 0; e < 2; ++e) { f[2 * e] = __uint_as_float(r.p[0][e] << 16); f[2 * e + 1] = __uint_as_float(r.p[0][e] & 0xffff0000u); }
  }
}
// feature index of float i of dc_row_unpack for lane lk of a row
template <int D> __device__ __forceinline__ int dc_row_feature(int lk, int i) {
  if constexpr (D == 256) return (i >> 3) * 128 + 8 * lk + (i & 7);
  else if constexpr (D == 128) return 8 * lk + i;
  else return 4 * lk + i;
}
// sum over the 16 lanes of a DPP row, result in every lane: xor 1, xor 2 (quad permutes), then the mirrors of 8 and 16
__device__ __forceinline__ float dc_row_sum16(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));
  return v;
}

template <int D>
struct DcKV { DcRow<D> k[DC_ATTN_NIT], v[DC_ATTN_NIT]; };

// row u of a block: key0 + 16 u (four waves x four rows of lanes).  Rows past the end re-read the last key (no
// branch around a load, so that the loads of one set stay in flight while the other set is consumed); their scores
// are masked.
template <int D>
__device__ __forceinline__ void dc_attn_load(DcKV<D>& r, const bf16_t* Kp, const bf16_t* Vp, int lk, int key0, int t1) {
#pragma unroll
  for (int u = 0; u < DC_ATTN_NIT; ++u) r.k[u] = dc_row_load<D>(Kp + (int64_t)min(key0 + 16 * u, t1 - 1) * D, lk);
#pragma unroll
  for (int u = 0; u < DC_ATTN_NIT; ++u) r.v[u] = dc_row_load<D>(Vp + (int64_t)min(key0 + 16 * u, t1 - 1) * D, lk);
}

template <int D>
__device__ __forceinline__ void dc_attn_block(const DcKV<D>& r, const float* qf, int key0, int t1, float& m, float& l, float* acc) {
  constexpr int NF = D / 16;
  float s[DC_ATTN_NIT], mb = -INFINITY;
#pragma unroll
  for (int u = 0; u < DC_ATTN_NIT; ++u) {
    float kf[NF], dot = 0.f;
    dc_row_unpack<D>(r.k[u], kf);
#pragma unroll
    for (int e = 0; e < NF; ++e) dot = fmaf(qf[e], kf[e], dot);
    dot = dc_row_sum16(dot);
    s[u] = key0 + 16 * u < t1 ? dot : -INFINITY;
    mb = fmaxf(mb, s[u]);
  }
  mb = fmaxf(mb, __shfl_xor(mb, 16, 64));
  mb = fmaxf(mb, __shfl_xor(mb, 32, 64));
  const float mn = fmaxf(m, mb);
  if (mn == -INFINITY) return;                       // no valid key in this block for the whole wave (wave-uniform)
  const float f = exp2f(m - mn);                     // 0 when m was -inf
  m = mn; l *= f;
#pragma unroll
  for (int e = 0; e < NF; ++e) acc[e] *= f;
#pragma unroll
  for (int u = 0; u < DC_ATTN_NIT; ++u) {
    const float p = exp2f(s[u] - mn);                // 0 for masked keys
    float vf[NF];
    dc_row_unpack<D>(r.v[u], vf);
    l += p;
#pragma unroll
    for (int e = 0; e < NF; ++e) acc[e] = fmaf(p, vf[e], acc[e]);
  }
}

template <int D>
__global__ __launch_bounds__(256) void decode_attn_kernel(DecodeAttnArgs a) {
  constexpr int NF = D / 16, BLOCK = 16 * DC_ATTN_NIT;
  __shared__ float s_red[4][D + 2];
  __shared__ int s_flag;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lk = lane & 15, kq = lane >> 4;
  const int bh = blockIdx.y, b = bh / a.h, hh = bh - b * a.h, split = blockIdx.x, nsplit = gridDim.x;
  // blocks are dealt to the workgroups of a (sequence, head) in turn, so that at any time they read one contiguous
  // stretch of the cache together (a softmax does not care about the order of its keys)
  const int t1 = a.n_keys, stride = nsplit * BLOCK;
  const bf16_t* Kp = a.K + (int64_t)b * a.kv_b + (int64_t)hh * a.kv_h;
  const bf16_t* Vp = a.V + (int64_t)b * a.kv_b + (int64_t)hh * a.kv_h;
  const DcRow<D> qv = dc_row_load<D>(a.q + (int64_t)b * a.q_b + (int64_t)hh * a.q_h, lk);
  const int first = split * BLOCK + 4 * w + kq;      // this lane's key in row u = 0 of the workgroup's first block
  DcKV<D> ra, rb;
  dc_attn_load<D>(ra, Kp, Vp, lk, first, t1);
  float qf[NF], acc[NF], m = -INFINITY, l = 0.f;
  dc_row_unpack<D>(qv, qf);
#pragma unroll
  for (int e = 0; e < NF; ++e) { qf[e] *= a.scale_log2e; acc[e] = 0.f; }
  for (int base = split * BLOCK; base < t1; base += 2 * stride) {
    const int kb = base + 4 * w + kq;
    dc_attn_load<D>(rb, Kp, Vp, lk, kb + stride, t1);
    dc_attn_block<D>(ra, qf, kb, t1, m, l, acc);
    dc_attn_load<D>(ra, Kp, Vp, lk, kb + 2 * stride, t1);
    dc_attn_block<D>(rb, qf, kb + stride, t1, m, l, acc);
  }
  // the wave's four rows of lanes hold disjoint keys: sums over the rows; then the four waves through LDS
#pragma unroll
  for (int o = 16; o < 64; o <<= 1) {
    l += __shfl_xor(l, o, 64);
#pragma unroll
    for (int e = 0; e < NF; ++e) acc[e] += __shfl_xor(acc[e], o, 64);
  }
  if (kq == 0) {
#pragma unroll
    for (int e = 0; e < NF; ++e) s_red[w][dc_row_feature<D>(lk, e)] = acc[e];
    if (lk == 0) { s_red[w][D] = m; s_red[w][D + 1] = l; }
  }
  __syncthreads();
  float* part = a.part + ((int64_t)bh * nsplit + split) * (D + 2);
  {
    const float M = fmaxf(fmaxf(s_red[0][D], s_red[1][D]), fmaxf(s_red[2][D], s_red[3][D]));
    float f[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) f[i] = s_red[i][D] == -INFINITY ? 0.f : exp2f(s_red[i][D] - M);
    if (tid < D) dc_store_f32(part + tid, (f[0] * s_red[0][tid] + f[1] * s_red[1][tid]) + (f[2] * s_red[2][tid] + f[3] * s_red[3][tid]));
    if (tid == 0) {
      dc_store_f32(part + D, M);
      dc_store_f32(part + D + 1, (f[0] * s_red[0][D + 1] + f[1] * s_red[1][D + 1]) + (f[2] * s_red[2][D + 1] + f[3] * s_red[3][D + 1]));
    }
  }
  if (!dc_arrived_last(a.counters + bh * DC_CNT_STRIDE, nsplit, &s_flag)) return;
  if (tid < D) {      // the partial results are read eight workgroups at a time (independent loads, one round trip)
    const float* p0 = a.part + (int64_t)bh * nsplit * (D + 2);
    float M = -INFINITY;
    for (int s0 = 0; s0 < nsplit; s0 += 8) {
      float ms[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) ms[i] = dc_load_f32(p0 + (int64_t)min(s0 + i, nsplit - 1) * (D + 2) + D);
#pragma unroll
      for (int i = 0; i < 8; ++i) M = fmaxf(M, ms[i]);
    }
    float o = 0.f, ls = 0.f;
    for (int s0 = 0; s0 < nsplit; s0 += 8) {
      float ms[8], os[8], lv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float* ps = p0 + (int64_t)min(s0 + i, nsplit - 1) * (D + 2);
        ms[i] = dc_load_f32(ps + D); os[i] = dc_load_f32(ps + tid); lv[i] = dc_load_f32(ps + D + 1);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float f = (s0 + i >= nsplit || ms[i] == -INFINITY) ? 0.f : exp2f(ms[i] - M);
        o = fmaf(f, os[i], o);
        ls = fmaf(f, lv[i], ls);
      }
    }
    a.o[(int64_t)b * a.o_b + (int64_t)hh * a.o_h + tid] = f2bf(o / ls);
  }
}

// ---------------------------------------------------------------------------------------------------------------
// Last kernel: y = x + bdense + b2 + Wdense . o + W2 . hid: one matrix-vector product over the concatenated reduction
// dimension E + F.  Grid (E / 32 slices, K splits); a workgroup copies its K range of the activation rows into LDS
// (after requesting its first weight fragments), its partial sums go to `part`, and the workgroup that arrives last
// for its slice adds them up in split order, adds the biases and the residual and stores y.
__global__ __launch_bounds__(256) void decode_out_kernel(DecodeOutArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char dc_smem[];
  __shared__ float red[4 * 32 * 32];
  __shared__ int s_flag;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, l32 = lane & 31, hf = lane >> 5;
  const int B = a.B, E = a.E, F = a.F, slice = blockIdx.x, nks = gridDim.y;
  // splits [0, n_dense) walk Wdense (activation o), the others W2 (activation hid): no split straddles the two
  const bool dense = (int)blockIdx.y < a.n_dense;
  const int ks = dense ? blockIdx.y : blockIdx.y - a.n_dense, nk = dense ? a.n_dense : nks - a.n_dense;
  const int KM = (dense ? E : F) / 16;
  const int per = (KM + nk - 1) / nk, g0 = min(KM, ks * per), g1 = min(KM, g0 + per);
  const int perw = (g1 - g0 + 3) / 4, k0 = min(g1, g0 + w * perw), k1 = min(g1, k0 + perw);
  const dc_u32x4* wp = (const dc_u32x4*)(dense ? a.wdense_p_ : a.w2_p_) + (int64_t)slice * KM * 64 + lane;
  DcSets<DC_PF> fr;
  dc_preload(fr, wp, k0, k1);
  // the workgroup's K range of the activation rows into LDS
  const int pitch = a.per_max * 16 + 8;
  bf16_t* xs = (bf16_t*)dc_smem;
  const bf16_t* src = dense ? a.o : a.hid;
  const int ld = dense ? E : F, nch = (g1 - g0) * 2;
  for (int idx = tid; idx < B * nch; idx += 256) {
    const int b = idx / nch, c = idx - b * nch;
    *(dc_u32x4*)(xs + (size_t)b * pitch + 8 * c) = *(const dc_u32x4*)(src + (int64_t)b * ld + 16 * g0 + 8 * c);
  }
  __syncthreads();
  const unsigned char* xl = (const unsigned char*)xs + (size_t)min(l32, B - 1) * pitch * 2 + hf * 16;
  dc_f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  dc_consume(fr, wp, xl, g0, k0, k1, acc);
  if (l32 < B) {
#pragma unroll
    for (int i = 0; i < 16; ++i) red[(w * 32 + (i / 4) * 8 + hf * 4 + (i & 3)) * B + l32] = acc[i];
  }
  __syncthreads();
  for (int idx = tid; idx < 32 * B; idx += 256) {
    const int r = idx / B, b = idx - r * B;
    const float v = (red[(0 * 32 + r) * B + b] + red[(1 * 32 + r) * B + b]) + (red[(2 * 32 + r) * B + b] + red[(3 * 32 + r) * B + b]);
    dc_store_f32(a.part + ((int64_t)blockIdx.y * B + b) * E + slice * 32 + r, v);
  }
  if (!dc_arrived_last(a.counters + slice * DC_CNT_STRIDE, nks, &s_flag)) return;
  for (int idx = tid; idx < 32 * B; idx += 256) {
    const int b = idx >> 5, r = idx & 31, n = slice * 32 + r;
    float v = bf2f(a.bdense[n]) + bf2f(a.b2[n]);
    for (int s0 = 0; s0 < nks; s0 += 8) {      // eight splits at a time: independent loads, summed in split order
      float pv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) pv[i] = dc_load_f32(a.part + ((int64_t)min(s0 + i, nks - 1) * B + b) * E + n);
#pragma unroll
      for (int i = 0; i < 8; ++i) v += s0 + i < nks ? pv[i] : 0.f;
    }
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
    hipError_t e = hipFuncSetAttribute((const void*)decode_in_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)decode_in_kernel<16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return (int)e;
    allowed.store(smem);
  }
  const dim3 grid((unsigned)((3 * a.E + a.F) / 64));
  if (a.E <= 2048) decode_in_kernel<4><<<grid, dim3(512), smem, (hipStream_t)stream>>>(a);
  else decode_in_kernel<16><<<grid, dim3(512), smem, (hipStream_t)stream>>>(a);
  return (int)hipGetLastError();
}

int decode_attn_block(int) { return 16 * DC_ATTN_NIT; }
int decode_counter_stride() { return DC_CNT_STRIDE; }      // keys of one block of the attention kernel

int launch_decode_attn(const DecodeAttnArgs& a, int nsplit, void* stream) {
  if (a.d != 64 && a.d != 128 && a.d != 256) return (int)hipErrorInvalidValue;
  if (nsplit < 1) return (int)hipErrorInvalidValue;
  const dim3 grid((unsigned)nsplit, (unsigned)(a.B * a.h));
  switch (a.d) {
    case 64: decode_attn_kernel<64><<<grid, dim3(256), 0, (hipStream_t)stream>>>(a); break;
    case 128: decode_attn_kernel<128><<<grid, dim3(256), 0, (hipStream_t)stream>>>(a); break;
    default: decode_attn_kernel<256><<<grid, dim3(256), 0, (hipStream_t)stream>>>(a); break;
  }
  return (int)hipGetLastError();
}

// K splits given to Wdense (the rest go to W2), the most steps any split gets, and the LDS bytes of its activation rows
static void decode_out_plan(int B, int E, int F, int nks, int* n_dense, int* per_max, size_t* smem) {
  const int KE = E / 16, KF = F / 16;
  *n_dense = std::max(1, std::min(nks - 1, (int)((int64_t)nks * KE / (KE + KF))));
  *per_max = std::max((KE + *n_dense - 1) / *n_dense, (KF + (nks - *n_dense) - 1) / (nks - *n_dense));
  *smem = (size_t)B * (*per_max * 16 + 8) * 2;
}
size_t decode_out_smem(int B, int E, int F, int nks) {
  int nd, pm; size_t smem;
  decode_out_plan(B, E, F, nks, &nd, &pm, &smem);
  return smem;
}

int launch_decode_out(const DecodeOutArgs& a0, int nks, void* stream) {
  if (nks < 2) return (int)hipErrorInvalidValue;
  DecodeOutArgs a = a0;
  size_t smem;
  decode_out_plan(a.B, a.E, a.F, nks, &a.n_dense, &a.per_max, &smem);
  if (smem > 48 * 1024) return (int)hipErrorInvalidValue;
  decode_out_kernel<<<dim3((unsigned)(a.E / 32), (unsigned)nks), dim3(256), smem, (hipStream_t)stream>>>(a);
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
