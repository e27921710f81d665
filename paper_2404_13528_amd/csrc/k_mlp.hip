// Fused MLP: Y = residual + W2 . gelu(W1 . norm(x) + b1) + b2 per token, the hidden activation never leaving the
// registers.  Not an operator pair of the paper's tables (two ILD & Variable operators are kept apart there):
// it is the deeper fusion next to the layout path, where the hidden tensor is the largest intermediate of a block.
//
// Shape of the work: a workgroup of four waves owns 32 tokens and all C output features.  The hidden dimension
// is cut into slices of 32 units and dealt round-robin to the waves; for its slice a wave forms
//   H^T[32 hidden, tokens] = W1[slice, :] . X^T        (C / 16 MFMAs, X fragments from LDS)
// applies bias + GELU in registers, and feeds the result, still in registers, as the second operand of
//   Y^T[C, tokens] += W2[:, slice] . H                  (C / 16 MFMAs)
// so a wave holds a partial Y^T over its slices (split-K across waves) and the four partials are added through
// LDS once, at the end, in a fixed order.  No weight element is used twice inside a workgroup, so the weights go
// straight from L2 into MFMA operand registers (no LDS staging, no barrier in the main loop), each fragment
// register being refilled for the wave's next slice right after the MFMA that consumed it: every load has a whole
// slice (2 * C / 16 MFMAs) to arrive.
//
// Weight layout (the paper's principle that a producer writes the layout its consumer reads best, Sec. 3.2.2, applied
// to constants: done once by mlp_pack_kernel): an MFMA operand fragment is 64 lanes x 16 bytes taken from 32 rows, 32
// bytes per row; read from the row-major matrix every such load touches 32 cache lines for a quarter of their
// bytes (measured: 76 us against 33 us for M = 6272, C = 384, hidden 1536).  Packed, a fragment is 1 KiB
// contiguous in lane order:
//   W1 fragment (slice sc, step kk) at index sc * C/16 + kk:        lane (l32, hf) = W1[32 sc + rho(l32)][16 kk + 8 hf ..+7]
//   W2 fragment (slice sc, block t, step s) at (sc * C/32 + t) * 2 + s: lane (l32, hf) = W2[32 t + l32][32 sc + 16 s + 8 hf ..+7]
// rho assigns the accumulator rows of the first product to hidden units in the order that makes the eight values a
// lane holds for one 16-wide step of the second product eight consecutive hidden units: accumulator row
// 8b + 4h + i (b < 4, h < 2, i < 4) is hidden unit 16 (b >> 1) + 8h + 4 (b & 1) + i of the slice.
#include <type_traits>
#include "device_common.h"
#include "kernels.h"

namespace sm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 mlp_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float mlp_f32x16;
typedef unsigned int mlp_u32x4 __attribute__((ext_vector_type(4)));
typedef float mlp_f32x4 __attribute__((ext_vector_type(4)));
typedef float mlp_f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 mlp_bf16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ unsigned mlp_pack2(float a, float b) {
  const mlp_f32x2 p = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(p, mlp_bf16x2));
}
__device__ __forceinline__ void mlp_unpack8(mlp_u32x4 v, float* f) {
#pragma unroll
  for (int e = 0; e < 4; ++e) { f[2 * e] = __uint_as_float(v[e] << 16); f[2 * e + 1] = __uint_as_float(v[e] & 0xffff0000u); }
}
__device__ __forceinline__ int mlp_rho(int r) { return 16 * (r >> 4) + 8 * ((r >> 2) & 1) + 4 * ((r >> 3) & 1) + (r & 3); }

// one thread per 16-byte chunk of the packed buffer: [W1 fragments | W2 fragments]
__global__ void mlp_pack_kernel(const bf16_t* W1, const bf16_t* W2, mlp_u32x4* packed, int C, int Hd) {
  const int KK = C / 16, T = C / 32;
  const int64_t n1 = (int64_t)Hd * C / 8;
  const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= 2 * n1) return;
  const int64_t q = o < n1 ? o : o - n1;
  const int lane = (int)(q & 63), l32 = lane & 31, hf = lane >> 5;
  const int64_t frag = q >> 6;
  const bf16_t* src;
  if (o < n1) {
    const int sc = (int)(frag / KK), kk = (int)(frag - (int64_t)sc * KK);
    src = W1 + (int64_t)(32 * sc + mlp_rho(l32)) * C + 16 * kk + 8 * hf;
  } else {
    const int s = (int)(frag & 1);
    const int64_t ft = frag >> 1;
    const int sc = (int)(ft / T), t = (int)(ft - (int64_t)sc * T);
    src = W2 + (int64_t)(32 * t + l32) * Hd + 32 * sc + 16 * s + 8 * hf;
  }
  packed[o] = *(const mlp_u32x4*)src;
}

// X tile of 32 token rows -> LDS, rows at an odd pitch of 16-byte slots (rows past M as zeros); 256 threads
template <int C>
__device__ __forceinline__ void mlp_load_x_tile(mlp_u32x4* x_l, const bf16_t* X, int64_t row0, int64_t M, int ident, int64_t ld,
                                                const SM_KARG RowProg* rows) {
  constexpr int XS = C / 8, XP = XS + 1;
  for (int s = threadIdx.x; s < 32 * XS; s += 256) {
    const int r = s / XS, c = s - r * XS;
    const int64_t row = row0 + r;
    mlp_u32x4 v = {0u, 0u, 0u, 0u};
    if (row < M) v = *(const mlp_u32x4*)(X + (ident ? row * ld : eval_rows_k(rows, row)) + c * 8);
    x_l[r * XP + c] = v;
  }
}

// LayerNorm of the tile's rows in place (the norm that precedes the product, folded): eight lanes per token,
// two-pass fp32 statistics, the result rounded to bf16 as a separate norm kernel would have stored it
template <int C>
__device__ __forceinline__ void mlp_norm_x_tile(mlp_u32x4* x_l, float eps, const mlp_u32x4* gam, const mlp_u32x4* bet) {
  constexpr int XS = C / 8, XP = XS + 1;
  const int r = threadIdx.x >> 3, p = threadIdx.x & 7;
  mlp_u32x4* xr = x_l + r * XP;
  float sum = 0.f;
  for (int c = p; c < XS; c += 8) {
    float f[8];
    mlp_unpack8(xr[c], f);
#pragma unroll
    for (int e = 0; e < 8; ++e) sum += f[e];
  }
  sum += __shfl_xor(sum, 1, 64); sum += __shfl_xor(sum, 2, 64); sum += __shfl_xor(sum, 4, 64);
  const float mean = sum / (float)C;
  float var = 0.f;
  for (int c = p; c < XS; c += 8) {
    float f[8];
    mlp_unpack8(xr[c], f);
#pragma unroll
    for (int e = 0; e < 8; ++e) { const float d = f[e] - mean; var += d * d; }
  }
  var += __shfl_xor(var, 1, 64); var += __shfl_xor(var, 2, 64); var += __shfl_xor(var, 4, 64);
  const float rstd = rsqrtf(var / (float)C + eps), sh = -mean * rstd;
  for (int c = p; c < XS; c += 8) {
    float f[8], gf[8], bf[8];
    mlp_unpack8(xr[c], f);
    mlp_unpack8(gam[c], gf);
    mlp_unpack8(bet[c], bf);
    mlp_u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      o[e] = mlp_pack2(fmaf(fmaf(f[2 * e], rstd, sh), gf[2 * e], bf[2 * e]), fmaf(fmaf(f[2 * e + 1], rstd, sh), gf[2 * e + 1], bf[2 * e + 1]));
    xr[c] = o;
  }
}

constexpr int MLP_RP = 36;       // floats per token row of a 32 x 32 partial tile in LDS (144 bytes: conflict-free 16-byte writes)

// PROJ: the Linear that precedes the MLP's residual stream is computed here as well (a transformer block's attention
// output projection): x1 = A . Wp^T + bp + x0 for the tile's 32 tokens, x0 read (and Y written) through y_rows, then
// Y = x1 + MLP(LayerNorm(x1)).  x1 never reaches memory: a normalised copy feeds the first product from LDS, a plain
// copy in LDS is the final residual.  The projection's weight (packed like lin_pack_kernel's) streams through the
// same registers as W1, three (C / 128) slices of 32 output features per wave, and the last slice's refill is
// already the MLP's first W1 slice.
template <int C, bool PROJ>
__global__ __launch_bounds__(256, 1) void mlp_fused_kernel(MlpArgs g) {
  constexpr int KK = C / 16;            // 16-wide steps of the first product
  constexpr int T = C / 32;             // 32-row blocks of Y^T
  constexpr int BM = 32;
  constexpr int XS = C / 8;             // 16-byte slots per token row
  constexpr int XP = XS + 1;            // odd pitch: the fragment reads of 16 tokens hit 16 different bank groups
  constexpr size_t TILE = (size_t)BM * XP * 16;
  static_assert(T % 4 == 0, "C must be a multiple of 128");
  const SM_KARG MlpArgs* gk = kernarg_ptr<MlpArgs>();
  extern __shared__ __align__(16) unsigned char smem_raw[];
  // PROJ: [A tile | x1 normalised | x1 plain | partial sums | b1 | bp]; else [X tile | partial sums | b1]
  mlp_u32x4* a_l = (mlp_u32x4*)smem_raw;
  mlp_u32x4* x_l = (mlp_u32x4*)(smem_raw + (PROJ ? TILE : 0));            // [BM][XP]
  mlp_u32x4* r_l = (mlp_u32x4*)(smem_raw + 2 * TILE);                     // PROJ only
  float* red = (float*)(smem_raw + (PROJ ? 3 : 1) * TILE);                // [4 waves][4 blocks][32][MLP_RP]
  mlp_u32x4* b1_l = (mlp_u32x4*)(smem_raw + (PROJ ? 3 : 1) * TILE + (size_t)4 * 4 * 32 * MLP_RP * 4);   // [Hd / 8]
  mlp_u32x4* bp_l = b1_l + g.Hd / 8;                                      // PROJ only: [C / 8]

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave index as a scalar: slice bases become scalar addresses
  const int64_t row0 = (int64_t)blockIdx.x * BM;
  const bf16_t* X = (const bf16_t*)g.X;
  const int Hd = g.Hd;
  const int nsub = Hd >> 5;
  const char* W1p = (const char*)g.Wp;                                    // fragments of 1 KiB, see the file header
  const char* W2p = W1p + (size_t)Hd * C * 2;

  // the wave's first slice of weights is requested before anything else
  mlp_u32x4 w1[KK], w2[T][2];
  const int sc0 = w < nsub ? w : 0;     // a wave without a slice (hidden < 128) computes nothing but loads in bounds
  {
    const unsigned o1 = PROJ ? (unsigned)(w * KK) * 1024u + lane * 16u : (unsigned)(sc0 * KK) * 1024u + lane * 16u;
    const char* first = PROJ ? (const char*)g.Wproj_p : W1p;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) w1[kk] = *(const mlp_u32x4*)(first + o1 + kk * 1024);
    const unsigned o2 = (unsigned)(sc0 * T * 2) * 1024u + lane * 16u;
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
      for (int s = 0; s < 2; ++s) w2[t][s] = *(const mlp_u32x4*)(W2p + o2 + (t * 2 + s) * 1024);
  }

  mlp_load_x_tile<C>(PROJ ? a_l : x_l, X, row0, g.M, g.x_rows.identity, g.x_rows.ld, &gk->x_rows);
  // the first bias as well: a global load inside the main loop would be waited for in issue order, behind the
  // whole weight prefetch
  for (int s = tid; s < Hd / 8; s += 256) b1_l[s] = ((const mlp_u32x4*)g.b1)[s];
  if constexpr (PROJ) for (int s = tid; s < XS; s += 256) bp_l[s] = ((const mlp_u32x4*)g.bproj)[s];
  __syncthreads();

  if constexpr (PROJ) {
    const int64_t prow = row0 + l32 < g.M ? row0 + l32 : g.M - 1;        // lanes past M read the last row's residual
    const int64_t ro0 = g.y_rows.identity ? prow * g.y_rows.ld : eval_rows_k(&gk->y_rows, prow);
    const bf16_t* R0 = (const bf16_t*)g.resid0;
#pragma unroll
    for (int j = 0; j < T / 4; ++j) {
      const int sc = w + 4 * j;                                           // 32 output features of the projection
      // loads the epilogue needs go out before the slice's weight refill (vector loads return in issue order)
      const mlp_u32x4 res0 = *(const mlp_u32x4*)(R0 + ro0 + sc * 32 + hf * 8);
      const mlp_u32x4 res1 = *(const mlp_u32x4*)(R0 + ro0 + sc * 32 + 16 + hf * 8);
      const mlp_u32x4 bias_v = bp_l[sc * 4 + hf], bias_w = bp_l[sc * 4 + 2 + hf];
      const char* nxt = j + 1 < T / 4 ? (const char*)g.Wproj_p + (size_t)((sc + 4) * KK) * 1024u : W1p + (size_t)(sc0 * KK) * 1024u;
      int ao = l32 * XP + hf;                       // opaque per slice: the A fragments are re-read from LDS instead of
      asm volatile("" : "+v"(ao));                  // being kept in (and spilled from) registers across the slices
      mlp_f32x16 h;
#pragma unroll
      for (int e = 0; e < 16; ++e) h[e] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const mlp_u32x4 af = a_l[ao + 2 * kk];
        h = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(mlp_bf16x8, w1[kk]), __builtin_bit_cast(mlp_bf16x8, af), h, 0, 0, 0);
        w1[kk] = *(const mlp_u32x4*)(nxt + kk * 1024 + lane * 16u);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      // accumulator register 4b + i of lane (token, hf) is feature 8b + 4 hf + i of the slice: one v_permlane32_swap
      // per value pair gives the lane eight consecutive features (run 2 gp + hf of the slice's four)
#pragma unroll
      for (int gp = 0; gp < 2; ++gp) {
        float v[8], bb[8], rr[8];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(h[8 * gp + q]), __float_as_uint(h[8 * gp + 4 + q]), false, false);
          v[q] = __uint_as_float(sw[0]);
          v[4 + q] = __uint_as_float(sw[1]);
        }
        mlp_unpack8(gp ? bias_w : bias_v, bb);
        mlp_unpack8(gp ? res1 : res0, rr);
        mlp_u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = mlp_pack2(v[2 * e] + bb[2 * e] + rr[2 * e], v[2 * e + 1] + bb[2 * e + 1] + rr[2 * e + 1]);
        x_l[l32 * XP + sc * 4 + 2 * gp + hf] = o;        // x1 rounded to bf16, as the separate Linear stores it
        r_l[l32 * XP + sc * 4 + 2 * gp + hf] = o;
      }
    }
    __syncthreads();
  }
  if (g.norm) {
    mlp_norm_x_tile<C>(x_l, g.norm_eps, (const mlp_u32x4*)g.norm_gamma, (const mlp_u32x4*)g.norm_beta);
    __syncthreads();
  }

  mlp_f32x16 out[T];
#pragma unroll
  for (int t = 0; t < T; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) out[t][e] = 0.f;

  for (int sc = w; sc < nsub; sc += 4) {
    const int nx = sc + 4 < nsub ? sc + 4 : sc;          // the last slice reloads itself: no branch around the prefetch
    int xo = l32 * XP + hf;                              // opaque per slice: the X fragments are re-read from LDS every
    asm volatile("" : "+v"(xo));                         // time instead of being hoisted into (and spilled from) registers
    const mlp_u32x4 bias_v = b1_l[sc * 4 + hf];
    const mlp_u32x4 bias_w = b1_l[sc * 4 + 2 + hf];
    mlp_f32x16 h;
#pragma unroll
    for (int e = 0; e < 16; ++e) h[e] = 0.f;
    {
      const unsigned o1 = (unsigned)(nx * KK) * 1024u + lane * 16u;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const mlp_u32x4 xf = x_l[xo + 2 * kk];
        h = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(mlp_bf16x8, w1[kk]), __builtin_bit_cast(mlp_bf16x8, xf), h, 0, 0, 0);
        w1[kk] = *(const mlp_u32x4*)(W1p + o1 + kk * 1024);
      }
    }
    // bias + GELU, rounded to bf16 as a stored hidden activation would be; step s of the second product takes
    // accumulator blocks 2s and 2s + 1 = hidden units 16s + 8 hf + 0..7 of the slice
    float bf_[16];
    mlp_unpack8(bias_v, bf_);
    mlp_unpack8(bias_w, bf_ + 8);
    mlp_u32x4 hfr[2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float a = gelu_poly(h[8 * s + 2 * e] + bf_[8 * s + 2 * e]);
        const float b = gelu_poly(h[8 * s + 2 * e + 1] + bf_[8 * s + 2 * e + 1]);
        hfr[s][e] = mlp_pack2(a, b);
      }
    {
      const unsigned o2 = (unsigned)(nx * T * 2) * 1024u + lane * 16u;
#pragma unroll
      for (int t = 0; t < T; ++t)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          out[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(mlp_bf16x8, w2[t][s]), __builtin_bit_cast(mlp_bf16x8, hfr[s]), out[t], 0, 0, 0);
          w2[t][s] = *(const mlp_u32x4*)(W2p + o2 + (t * 2 + s) * 1024);
        }
    }
    // issue order of the slice: every MFMA is followed by the load that refills its weight register (left alone, the
    // scheduler gathers all loads at the end of the slice, where their latency is exposed at the top of the next)
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
#pragma unroll
    for (int i = 0; i < 2 * T; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
  }

  // The four partial Y^T are added through LDS, four row blocks at a time: every wave writes its four blocks as
  // [token][feature] fp32 tiles, then wave w owns block 4 gi + w: sums the partials in wave order, adds bias and
  // residual and stores 16 consecutive features per lane.  Bias and residual are requested before the first
  // exchange so that their latency is not paid once per round.
  const bf16_t* R = (const bf16_t*)g.residual;
  bf16_t* Y = (bf16_t*)g.Y;
  const int tk = lane >> 1, hh = lane & 1;
  const int64_t row = row0 + tk;
  const bool row_ok = row < g.M;
  const int64_t ro = row_ok ? (g.y_rows.identity ? row * g.y_rows.ld : eval_rows_k(&gk->y_rows, row)) : 0;
  mlp_u32x4 rres[T / 4][2], rb2[T / 4][2];
#pragma unroll
  for (int gi = 0; gi < T / 4; ++gi) {
    const int cb = (4 * gi + w) * 32 + 16 * hh;          // first of this lane's 16 features
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      rb2[gi][q] = *(const mlp_u32x4*)((const bf16_t*)g.b2 + cb + 8 * q);
      rres[gi][q] = mlp_u32x4{0u, 0u, 0u, 0u};
      if constexpr (PROJ) rres[gi][q] = r_l[tk * XP + cb / 8 + q];
      else if (R && row_ok) rres[gi][q] = *(const mlp_u32x4*)(R + ro + cb + 8 * q);
    }
  }
#pragma unroll
  for (int gi = 0; gi < T / 4; ++gi) {
    if (gi) __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float* tile = red + (size_t)((w * 4 + j) * 32) * MLP_RP;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const mlp_f32x4 v = {out[4 * gi + j][4 * b], out[4 * gi + j][4 * b + 1], out[4 * gi + j][4 * b + 2], out[4 * gi + j][4 * b + 3]};
        *(mlp_f32x4*)(tile + l32 * MLP_RP + 8 * b + 4 * hf) = v;
      }
    }
    __syncthreads();
    float acc[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) {
      const float* tile = red + (size_t)((ww * 4 + w) * 32) * MLP_RP + tk * MLP_RP + 16 * hh;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const mlp_f32x4 v = *(const mlp_f32x4*)(tile + 4 * q);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[4 * q + e] += v[e];
      }
    }
    if (row_ok) {
      const int cb = (4 * gi + w) * 32 + 16 * hh;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        float bb[8], rr[8];
        mlp_unpack8(rb2[gi][q], bb);
        mlp_unpack8(rres[gi][q], rr);
        mlp_u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e)      // product + bias + residual in fp32, rounded to bf16 once, as the Linear's epilogue does
          o[e] = mlp_pack2(acc[8 * q + 2 * e] + bb[2 * e] + rr[2 * e], acc[8 * q + 2 * e + 1] + bb[2 * e + 1] + rr[2 * e + 1]);
        *(mlp_u32x4*)(Y + ro + cb + 8 * q) = o;
      }
    }
  }
}

static size_t mlp_smem(int C, int Hd, bool proj) {
  const size_t tile = (size_t)32 * (C / 8 + 1) * 16;
  return (proj ? 3 : 1) * tile + (size_t)4 * 4 * 32 * MLP_RP * 4 + (size_t)Hd * 2 + (proj ? (size_t)C * 2 : 0);
}

template <int C, bool PROJ>
static int mlp_launch2(const MlpArgs& g, void* stream) {
  const size_t smem = mlp_smem(C, g.Hd, PROJ);
  static size_t allowed = 0;          // raised on demand: the attribute is per kernel, the hidden size varies
  if (smem > allowed) {
    const hipError_t e = hipFuncSetAttribute((const void*)mlp_fused_kernel<C, PROJ>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return (int)e;
    allowed = smem;
  }
  const int64_t n_wg = (g.M + 31) / 32;
  mlp_fused_kernel<C, PROJ><<<dim3((unsigned)n_wg), dim3(256), smem, (hipStream_t)stream>>>(g);
  return (int)hipGetLastError();
}
template <int C>
static int mlp_launch(const MlpArgs& g, void* stream) {
  return g.Wproj_p ? mlp_launch2<C, true>(g, stream) : mlp_launch2<C, false>(g, stream);
}

// LDS capacity: the projection variant holds three token tiles
bool mlp_proj_supported(int C, int Hd, int dtype) { return mlp_fused_supported(C, Hd, dtype) && mlp_smem(C, Hd, true) <= 160 * 1024; }

bool mlp_fused_supported(int C, int Hd, int dtype) {
  return dtype == SM_BF16 && (C == 128 || C == 256 || C == 384) && Hd >= 32 && Hd % 32 == 0 && Hd <= 16384;
}

int launch_mlp_pack(const void* W1, const void* W2, int C, int Hd, void* packed, void* stream) {
  const int64_t n = 2 * ((int64_t)Hd * C / 8);
  mlp_pack_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>((const bf16_t*)W1, (const bf16_t*)W2, (mlp_u32x4*)packed, C, Hd);
  return (int)hipGetLastError();
}

int launch_mlp_fused(const MlpArgs& g, void* stream) {
  switch (g.C) {
    case 128: return mlp_launch<128>(g, stream);
    case 256: return mlp_launch<256>(g, stream);
    case 384: return mlp_launch<384>(g, stream);
  }
  return (int)hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------------------------------
// Linear for a short reduction dimension (K = C in {128, 256, 384}), Y = act(norm(X) . W^T + b) (+ residual): the first
// half of the kernel above on its own.  A workgroup owns 32 token rows, whose K elements stay in LDS for all N outputs;
// the N / 32 row slices of W are dealt round-robin to the four waves and stream from L2 straight into MFMA operand
// registers (packed by lin_pack_kernel: fragment (slice sc, step kk) at sc * K/16 + kk, lane (l32, hf) =
// W[32 sc + l32][16 kk + 8 hf ..+7]); every wave finishes its 32 x 32 outputs in registers and stores them: no
// barrier after the prologue.  Against the tiled kernel of k_gemm.hip this trades L2 -> CU traffic (W once per 32
// rows) for the absence of K-loop barriers and of a separate norm kernel.  Measured (with LayerNorm, against norm
// kernel + tiled kernel resp. the tiled kernel's own folded norm): 200704 x 384 x 128: 69 us against 89;
// 50176 x 768 x 256: 55 against 71; 6272 x 1152 x 384: 26 against 26.  The block executors do not use it.
template <int C, bool RES>
__global__ __launch_bounds__(256, 1) void lin32_kernel(Lin32Args g) {
  constexpr int KK = C / 16, XS = C / 8, XP = XS + 1;
  const SM_KARG Lin32Args* gk = kernarg_ptr<Lin32Args>();
  extern __shared__ __align__(16) unsigned char smem_raw[];
  mlp_u32x4* x_l = (mlp_u32x4*)smem_raw;                                  // [32][XP]
  mlp_u32x4* b_l = (mlp_u32x4*)(smem_raw + (size_t)32 * XP * 16);         // [N / 8]
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave index as a scalar: slice bases become scalar addresses
  const int64_t row0 = (int64_t)blockIdx.x * 32;
  const int nsub = g.N >> 5;
  const char* Wp = (const char*)g.Wp;

  mlp_u32x4 w1[KK];
  {
    const char* wb = Wp + (size_t)((w < nsub ? w : 0) * KK) * 1024u;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) w1[kk] = *(const mlp_u32x4*)(wb + kk * 1024 + lane * 16u);
  }
  mlp_load_x_tile<C>(x_l, (const bf16_t*)g.X, row0, g.M, g.x_rows.identity, g.x_rows.ld, &gk->x_rows);
  for (int s = tid; s < g.N / 8; s += 256) b_l[s] = g.bias ? ((const mlp_u32x4*)g.bias)[s] : mlp_u32x4{0u, 0u, 0u, 0u};
  __syncthreads();
  if (g.norm) {
    mlp_norm_x_tile<C>(x_l, g.norm_eps, (const mlp_u32x4*)g.norm_gamma, (const mlp_u32x4*)g.norm_beta);
    __syncthreads();
  }

  // the lane's X fragments do not depend on the slice: they stay in registers (K / 4 of them; the kernel fits two
  // workgroups per CU with them)
  mlp_u32x4 xf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) xf[kk] = x_l[l32 * XP + hf + 2 * kk];
  const int64_t row = row0 + l32;                 // the lane's token: accumulator column
  const bool row_ok = row < g.M;
  const int64_t rowc = row_ok ? row : g.M - 1;    // lanes past M read the last row's residual and store nothing
  const int64_t ro = g.y_rows.identity ? rowc * g.y_rows.ld : eval_rows_k(&gk->y_rows, rowc);
  const bf16_t* R = (const bf16_t*)g.residual;
  bf16_t* Y = (bf16_t*)g.Y;
  const bool gelu_on = g.act == SM_ACT_GELU;
  // the slice loop is one basic block up to the final masked store, so that the issue order below holds; loads
  // that the epilogue needs are issued before the slice's weight prefetch (vector loads return in issue order)
  for (int sc = w; sc < nsub; sc += 4) {
    const int nx = sc + 4 < nsub ? sc + 4 : sc;
    const mlp_u32x4 bias_v = b_l[sc * 4 + hf];          // features 8 hf ..+7 and 16 + 8 hf ..+7 of the slice: the two
    const mlp_u32x4 bias_w = b_l[sc * 4 + 2 + hf];      // runs this lane stores
    mlp_u32x4 res[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
    if constexpr (RES) {
      res[0] = *(const mlp_u32x4*)(R + ro + sc * 32 + hf * 8);
      res[1] = *(const mlp_u32x4*)(R + ro + sc * 32 + 16 + hf * 8);
    }
    mlp_f32x16 h;
#pragma unroll
    for (int e = 0; e < 16; ++e) h[e] = 0.f;
    const char* wb = Wp + (size_t)(nx * KK) * 1024u;      // scalar
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      h = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(mlp_bf16x8, w1[kk]), __builtin_bit_cast(mlp_bf16x8, xf[kk]), h, 0, 0, 0);
      w1[kk] = *(const mlp_u32x4*)(wb + kk * 1024 + lane * 16u);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
    // accumulator register 4b + i of lane (token, hf) is feature 8b + 4 hf + i: one v_permlane32_swap per value pair
    // gives each lane eight consecutive features (run 2 gp + hf of the slice's four runs of eight)
    mlp_u32x4 outv[2];
#pragma unroll
    for (int gp = 0; gp < 2; ++gp) {
      float v[8], bb[8], rr[8];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(h[8 * gp + j]), __float_as_uint(h[8 * gp + 4 + j]), false, false);
        v[j] = __uint_as_float(sw[0]);
        v[4 + j] = __uint_as_float(sw[1]);
      }
      mlp_unpack8(gp ? bias_w : bias_v, bb);
      mlp_unpack8(res[gp], rr);
      mlp_u32x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float a = v[2 * e] + bb[2 * e], b = v[2 * e + 1] + bb[2 * e + 1];
        const float ga = gelu_poly(a), gb = gelu_poly(b);
        a = gelu_on ? ga : a;
        b = gelu_on ? gb : b;
        o[e] = mlp_pack2(a + rr[2 * e], b + rr[2 * e + 1]);
      }
      outv[gp] = o;
    }
    if (row_ok) {
      // Written as assembly so that the compiler's wait-count bookkeeping sees loads only: with stores pending next to
      // loads it stops counting and waits for everything (vmcnt 0) at the top of the next slice, which exposes the
      // latency of the whole weight prefetch.  Its counts stay safe: it may wait for up to two operations more than
      // needed, never fewer (loads return in issue order among themselves).
      bf16_t* yp = Y + ro + sc * 32 + hf * 8;
      asm volatile("global_store_dwordx4 %0, %1, off\n\tglobal_store_dwordx4 %0, %2, off offset:32\n\ts_nop 2"
                   :: "v"(yp), "v"(outv[0]), "v"(outv[1]) : "memory");
    }
  }
}

__global__ void lin_pack_kernel(const bf16_t* W, mlp_u32x4* packed, int N, int K) {
  const int KK = K / 16;
  const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= (int64_t)N * K / 8) return;
  const int lane = (int)(o & 63), l32 = lane & 31, hf = lane >> 5;
  const int64_t frag = o >> 6;
  const int sc = (int)(frag / KK), kk = (int)(frag - (int64_t)sc * KK);
  packed[o] = *(const mlp_u32x4*)(W + (int64_t)(32 * sc + l32) * K + 16 * kk + 8 * hf);
}

template <int C, bool RES>
static int lin32_launch2(const Lin32Args& g, void* stream) {
  const size_t smem = (size_t)32 * (C / 8 + 1) * 16 + (size_t)g.N * 2;
  static size_t allowed = 0;
  if (smem > allowed) {
    const hipError_t e = hipFuncSetAttribute((const void*)lin32_kernel<C, RES>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return (int)e;
    allowed = smem;
  }
  lin32_kernel<C, RES><<<dim3((unsigned)((g.M + 31) / 32)), dim3(256), smem, (hipStream_t)stream>>>(g);
  return (int)hipGetLastError();
}
template <int C>
static int lin32_launch(const Lin32Args& g, void* stream) {
  return g.residual ? lin32_launch2<C, true>(g, stream) : lin32_launch2<C, false>(g, stream);
}

bool lin32_supported(int N, int K, int dtype) {
  return dtype == SM_BF16 && (K == 128 || K == 256 || K == 384) && N >= 32 && N % 32 == 0 && N <= 16384;
}

int launch_lin_pack(const void* W, int N, int K, void* packed, void* stream) {
  const int64_t n = (int64_t)N * K / 8;
  lin_pack_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>((const bf16_t*)W, (mlp_u32x4*)packed, N, K);
  return (int)hipGetLastError();
}

int launch_lin32(const Lin32Args& g, void* stream) {
  switch (g.K) {
    case 128: return lin32_launch<128>(g, stream);
    case 256: return lin32_launch<256>(g, stream);
    case 384: return lin32_launch<384>(g, stream);
  }
  return (int)hipErrorInvalidValue;
}

}  // namespace sm
