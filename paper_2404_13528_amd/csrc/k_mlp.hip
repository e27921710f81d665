// Fused MLP: Y = residual + W2 . gelu(W1 . norm(x) + b1) + b2 per token, the hidden activation never leaving the
// compute unit.  Not an operator pair of the paper's tables (two ILD & Variable operators are kept apart there):
// it is the deeper fusion next to the layout path, where the hidden tensor is the largest intermediate of a block.
//
// Shape of the work: a workgroup owns 32 tokens and has one wave per 32 output features (T = C / 32 waves).  The
// token tile (normalised in place when the norm is folded) stays in LDS.  The hidden dimension is processed in rounds
// of T slices of 32 units.  In a round, wave w first forms its slice
//   H^T[32 hidden, 32 tokens] = W1[slice, :] . X^T        (C / 16 MFMAs, X fragments from LDS)
// applies bias + GELU in registers and writes the bf16 result into the round's hidden tile in LDS; after one barrier it
// accumulates its own output block over the whole round,
//   Y^T[32 features, 32 tokens] += W2[block, round's hidden] . H        (2 T MFMAs, H fragments from LDS)
// so no partial sums are exchanged and a wave needs 16 accumulator registers per product.  The hidden tile is
// double-buffered: one barrier per round.  No weight element is used twice inside a workgroup, so the weights go
// straight from L2 into MFMA operand registers (no LDS staging): one set of C / 16 fragment registers carries the
// wave's whole weight stream, each register refilled, right after the MFMA that read it, with the fragment the next
// product needs at the same position, so every load has a full product (C / 16 MFMAs) to arrive.
//
// Weight layout (the paper's principle that a producer writes the layout its consumer reads best, Sec. 3.2.2, applied
// to constants: done once by mlp_pack_kernel): an MFMA operand fragment is 64 lanes x 16 bytes taken from 32 rows, 32
// bytes per row; read from the row-major matrix every such load touches 32 cache lines for a quarter of their
// bytes (measured on an earlier form of this kernel: 76 us against 33 us for M = 6272, C = 384, hidden 1536).
// Packed, a fragment is 1 KiB contiguous in lane order, and each wave's fragments follow each other in the order it
// uses them:
//   W1 fragment (slice sc, step kk) at index sc * C/16 + kk:            lane (l32, hf) = W1[32 sc + l32][16 kk + 8 hf ..+7]
//   W2 fragment (block t, slice sc, step s) at (t * hidden/32 + sc) * 2 + s: lane (l32, hf) = W2[32 t + l32][32 sc + 16 s + 8 hf ..+7]
#include <atomic>
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

// one thread per 16-byte chunk of the packed buffer: [W1 fragments | W2 fragments]
__global__ void mlp_pack_kernel(const bf16_t* W1, const bf16_t* W2, mlp_u32x4* packed, int C, int Hd) {
  const int KK = C / 16, nsub = Hd / 32;
  const int64_t n1 = (int64_t)Hd * C / 8;
  const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= 2 * n1) return;
  const int64_t q = o < n1 ? o : o - n1;
  const int lane = (int)(q & 63), l32 = lane & 31, hf = lane >> 5;
  const int64_t frag = q >> 6;
  const bf16_t* src;
  if (o < n1) {
    const int sc = (int)(frag / KK), kk = (int)(frag - (int64_t)sc * KK);
    src = W1 + (int64_t)(32 * sc + l32) * C + 16 * kk + 8 * hf;
  } else {
    const int s = (int)(frag & 1);
    const int64_t ft = frag >> 1;
    const int t = (int)(ft / nsub), sc = (int)(ft - (int64_t)t * nsub);
    src = W2 + (int64_t)(32 * t + l32) * Hd + 32 * sc + 16 * s + 8 * hf;
  }
  packed[o] = *(const mlp_u32x4*)src;
}

// X tile of 32 token rows -> LDS, rows at an odd pitch of 16-byte slots (rows past M as zeros); 256 threads
template <int C, int NTHR = 256>
__device__ __forceinline__ void mlp_load_x_tile(mlp_u32x4* x_l, const bf16_t* X, int64_t row0, int64_t M, int ident, int64_t ld,
                                                const SM_KARG RowProg* rows) {
  constexpr int XS = C / 8, XP = XS + 1, NIT = (32 * XS + NTHR - 1) / NTHR;
  // three passes, so that the offset lookups (a table load each, where the rows go through one) are in flight together,
  // and then the data loads: one latency each instead of one per chunk
  const int32_t* tab = ident ? nullptr : rows->table;
  int64_t off[NIT];
  int toff[NIT];
#pragma unroll
  for (int i = 0; i < NIT; ++i) {
    const int s = threadIdx.x + i * NTHR, r = s / XS;
    const int64_t row = min(row0 + min(r, 31), M - 1);
    if (ident) off[i] = row * ld;
    else if (tab) toff[i] = tab[row];
    else off[i] = eval_rows_k(rows, row);
  }
  mlp_u32x4 v[NIT];
#pragma unroll
  for (int i = 0; i < NIT; ++i) {
    const int s = threadIdx.x + i * NTHR, r = s / XS, c = s - r * XS;
    if (!ident && tab) off[i] = (int64_t)toff[i];
    v[i] = *(const mlp_u32x4*)(X + off[i] + (s < 32 * XS ? c : 0) * 8);
  }
#pragma unroll
  for (int i = 0; i < NIT; ++i) {
    const int s = threadIdx.x + i * NTHR, r = s / XS, c = s - r * XS;
    if (s < 32 * XS) x_l[r * XP + c] = row0 + r < M ? v[i] : mlp_u32x4{0u, 0u, 0u, 0u};
  }
}

// LayerNorm of the tile's rows in place (the norm that precedes the product, folded): eight lanes per token,
// two-pass fp32 statistics, the result rounded to bf16 as a separate norm kernel would have stored it
template <int C, int NTOK = 32>
__device__ __forceinline__ void mlp_norm_x_tile(mlp_u32x4* x_l, float eps, const mlp_u32x4* gam, const mlp_u32x4* bet) {
  constexpr int XS = C / 8, XP = XS + 1;
  const int p = threadIdx.x & 7;                // eight threads per token; no barrier inside
  for (int r = threadIdx.x >> 3; r < NTOK; r += blockDim.x >> 3) {
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
}

// bias, optional GELU, optional residual of one 32 x 32 accumulator: register 4b + i of lane (token, hf) is row
// 8b + 4 hf + i of the block; one v_permlane32_swap per value pair gives the lane eight consecutive rows (run
// 2 gp + hf of the block's four), packed to bf16 in outv[gp]
__device__ __forceinline__ mlp_u32x4 mlp_finish_half(const mlp_f32x16& h, int gp, const mlp_u32x4& bias, const mlp_u32x4& res, bool gelu_on) {
  float v[8], bb[8], rr[8];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(h[8 * gp + q]), __float_as_uint(h[8 * gp + 4 + q]), false, false);
    v[q] = __uint_as_float(sw[0]);
    v[4 + q] = __uint_as_float(sw[1]);
  }
  mlp_unpack8(bias, bb);
  mlp_unpack8(res, rr);
  mlp_u32x4 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    float a = v[2 * e] + bb[2 * e], b = v[2 * e + 1] + bb[2 * e + 1];
    const float ga = gelu_poly(a), gb = gelu_poly(b);
    a = gelu_on ? ga : a;
    b = gelu_on ? gb : b;
    o[e] = mlp_pack2(a + rr[2 * e], b + rr[2 * e + 1]);
  }
  return o;
}
__device__ __forceinline__ void mlp_finish(const mlp_f32x16& h, const mlp_u32x4& bias_v, const mlp_u32x4& bias_w, const mlp_u32x4* res,
                                           bool gelu_on, mlp_u32x4* outv) {
#pragma unroll
  for (int gp = 0; gp < 2; ++gp) outv[gp] = mlp_finish_half(h, gp, gp ? bias_w : bias_v, res[gp], gelu_on);
}

// PROJ: the Linear that precedes the MLP's residual stream is computed here as well (a transformer block's attention
// output projection): x1 = A . Wp^T + bp + x0 for the tile's 32 tokens, x0 read (and Y written) through y_rows, then
// Y = x1 + MLP(LayerNorm(x1)).  x1 never reaches memory: a normalised copy feeds the first product from LDS, a plain
// copy in LDS is the final residual.
// LNOUT = 1: a second output, LayerNorm(Y) with its own gamma / beta, stored through its own row map: the norm that opens
// the next block, computed while the rows are still in registers (statistics over the C / 32 waves through LDS).
// LNOUT = 2 (with PROJ): that norm stays in LDS and the Linear that follows it (the next block's QKV, N = 3 C, packed
// like lin_pack_kernel's) runs here too, three slices of 32 outputs per wave, stored through the same row map.
template <int C, bool PROJ, int LNOUT>
__global__ __launch_bounds__(64 * (C / 32), 1) void mlp_fused_kernel(MlpArgs g) {
  constexpr int KK = C / 16;            // 16-wide steps of the first product
  constexpr int T = C / 32;             // 32-row blocks of Y^T = waves of the workgroup
  constexpr int NTHR = 64 * T;
  constexpr int XS = C / 8;             // 16-byte slots per token row
  constexpr int XP = XS + 1;            // odd pitch: the fragment reads of 16 tokens hit 16 different bank groups
  constexpr int HP = 4 * T + 1;         // the same for a round's hidden tile (T slices of 32 = 4 slots each)
  constexpr size_t TILE = (size_t)32 * XP * 16, HTILE = (size_t)32 * HP * 16;
  const SM_KARG MlpArgs* gk = kernarg_ptr<MlpArgs>();
  extern __shared__ __align__(16) unsigned char smem_raw[];
  // PROJ: [A tile | x1 normalised | x1 plain | H x 2 | b1 | bp]; else [X tile | H x 2 | b1]
  mlp_u32x4* a_l = (mlp_u32x4*)smem_raw;
  mlp_u32x4* x_l = (mlp_u32x4*)(smem_raw + (PROJ ? TILE : 0));            // [32][XP]
  mlp_u32x4* r_l = (mlp_u32x4*)(smem_raw + 2 * TILE);                     // PROJ only
  mlp_u32x4* h_l = (mlp_u32x4*)(smem_raw + (PROJ ? 3 : 1) * TILE);        // [2][32][HP]
  mlp_u32x4* b1_l = (mlp_u32x4*)(smem_raw + (PROJ ? 3 : 1) * TILE + 2 * HTILE);   // [Hd / 8]
  mlp_u32x4* bp_l = b1_l + g.Hd / 8;                                      // PROJ only: [C / 8]
  float* st_l = (float*)(b1_l + g.Hd / 8 + (PROJ ? XS : 0));              // LNOUT only: [2][T][32] row statistics

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave index as a scalar: fragment bases become scalar addresses
  const int64_t row0 = (int64_t)blockIdx.x * 32;
  const int Hd = g.Hd;
  const int nsub = Hd >> 5;
  const int rounds = (nsub + T - 1) / T;
  // Weight fragments (1 KiB each, see the file header) are fetched with buffer loads: the descriptor and the fragment's
  // offset are scalar, the only vector operand is the lane's 16 bytes within the fragment, so no address arithmetic
  // touches the vector registers (and a fragment index past the end would read zeros instead of faulting).
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.Wp), 0, 4 * Hd * C, 0x00020000);
  const int W2o = 2 * Hd * C + w * nsub * 2048;                           // byte offset of this wave's W2 row block: (slice, step) in order
  const int lo = lane * 16;
  auto wload = [&](const __amdgpu_buffer_rsrc_t& r, int soff) __attribute__((always_inline)) { return __builtin_amdgcn_raw_buffer_load_b128(r, lo, soff, 0); };

  // One set of C / 16 fragment registers carries the whole weight stream of the wave: a product of C / 16 MFMAs
  // consumes them in order, and each is refilled, right after the MFMA that read it, with the fragment the NEXT
  // product needs at the same position (first product -> this round's W2 fragments -> next round's W1 slice -> ...):
  // every load has a full product to arrive and the compiler's wait is one constant count.
  mlp_u32x4 wf[KK];
  const int sc0 = w < nsub ? w : nsub - 1;      // (a wave past the last slice works on a copy of it and contributes zeros)
  __amdgpu_buffer_rsrc_t rp = rw, rq = rw;
  if constexpr (PROJ) rp = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.Wproj_p), 0, 2 * C * C, 0x00020000);
  if constexpr (LNOUT == 2) rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.Wq_p), 0, 6 * C * C, 0x00020000);
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) wf[kk] = PROJ ? wload(rp, (w * KK + kk) * 1024) : wload(rw, (sc0 * KK + kk) * 1024);

  // the lane's output-row offsets (table lookups, where the rows are mapped) are requested before the tile's loads,
  // not where they are first used
  const int64_t prow = row0 + l32 < g.M ? row0 + l32 : g.M - 1;          // lanes past M read the last row and store nothing
  const bool row_ok = row0 + l32 < g.M;
  const int64_t ro = g.y_rows.identity ? prow * g.y_rows.ld : eval_rows_k(&gk->y_rows, prow);
  int64_t ro2 = 0;
  if constexpr (LNOUT != 0) ro2 = g.y2_rows.identity ? prow * g.y2_rows.ld : eval_rows_k(&gk->y2_rows, prow);
  mlp_load_x_tile<C, NTHR>(PROJ ? a_l : x_l, (const bf16_t*)g.X, row0, g.M, g.x_rows.identity, g.x_rows.ld, &gk->x_rows);
  for (int s = tid; s < Hd / 8; s += NTHR) b1_l[s] = ((const mlp_u32x4*)g.b1)[s];
  if constexpr (PROJ) for (int s = tid; s < XS; s += NTHR) bp_l[s] = ((const mlp_u32x4*)g.bproj)[s];
  __syncthreads();

  const int fo = w * 32 + hf * 8;                                         // first of the lane's features in the wave's block

  mlp_u32x4 resid[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};              // residual of the final sum (lane's two runs of eight)
  if constexpr (PROJ) {
    // wave w forms features 32 w ..+31 of x1
    const bf16_t* R0 = (const bf16_t*)g.resid0;
    const mlp_u32x4 res[2] = {*(const mlp_u32x4*)(R0 + ro + fo), *(const mlp_u32x4*)(R0 + ro + fo + 16)};
    const mlp_u32x4 bias_v = bp_l[w * 4 + hf], bias_w = bp_l[w * 4 + 2 + hf];
    int ao = l32 * XP + hf;
    asm volatile("" : "+v"(ao));
    mlp_f32x16 h;
#pragma unroll
    for (int e = 0; e < 16; ++e) h[e] = 0.f;
    mlp_u32x4 fb[3] = {a_l[ao], a_l[ao + 2], a_l[ao + 4]};       // LDS fragments three steps ahead of their MFMA
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      h = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(mlp_bf16x8, wf[kk]), __builtin_bit_cast(mlp_bf16x8, fb[kk % 3]), h, 0, 0, 0);
      wf[kk] = wload(rw, (sc0 * KK + kk) * 1024);
      if (kk + 3 < KK) fb[kk % 3] = a_l[ao + 2 * (kk + 3)];
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);        // LDS fragment reads run three steps ahead of their MFMA
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    mlp_finish(h, bias_v, bias_w, res, false, resid);          // x1 rounded to bf16, as the separate Linear stores it
#pragma unroll
    for (int gp = 0; gp < 2; ++gp) {
      x_l[l32 * XP + w * 4 + 2 * gp + hf] = resid[gp];
      r_l[l32 * XP + w * 4 + 2 * gp + hf] = resid[gp];
    }
    __syncthreads();
  }
  if (g.norm) {
    mlp_norm_x_tile<C>(x_l, g.norm_eps, (const mlp_u32x4*)g.norm_gamma, (const mlp_u32x4*)g.norm_beta);
    __syncthreads();
  }

  mlp_f32x16 out;
#pragma unroll
  for (int e = 0; e < 16; ++e) out[e] = 0.f;
  const mlp_u32x4 zero4[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};

  for (int r = 0; r < rounds; ++r) {
    // ---- first product: this wave's slice of the round -> H (bias, GELU, bf16) into LDS
    const int sc = r * T + w;
    const bool sc_ok = sc < nsub;
    const int scc = sc_ok ? sc : nsub - 1;
    const int nsc = sc + T < nsub ? sc + T : scc;
    int xo = l32 * XP + hf;                              // opaque per round: the X fragments are re-read from LDS instead
    asm volatile("" : "+v"(xo));                         // of being hoisted into (and spilled from) registers
    const int s0 = r * T;                                // first slice of the round
    const int rem = nsub - s0;                           // slices of W2 from this round's first to the end (>= 1)
    const int cur2 = W2o + s0 * 2048;                    // scalar: this round's W2 fragments of this wave, (slice, step) in order
    mlp_f32x16 h;
#pragma unroll
    for (int e = 0; e < 16; ++e) h[e] = 0.f;
    mlp_u32x4 fb[3] = {x_l[xo], x_l[xo + 2], x_l[xo + 4]};        // LDS fragments three steps ahead of their MFMA
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      h = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(mlp_bf16x8, wf[kk]), __builtin_bit_cast(mlp_bf16x8, fb[kk % 3]), h, 0, 0, 0);
      if (kk + 3 < KK) fb[kk % 3] = x_l[xo + 2 * (kk + 3)];
      // refill with the second product's fragment kk of this round; past the end of W2 the last valid pair again (its H is zero)
      wf[kk] = wload(rw, cur2 + (kk < 2 * rem ? kk : (kk & 1) + 2 * (rem - 1)) * 1024);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);        // LDS fragment reads run three steps ahead of their MFMA
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    mlp_u32x4 hv[2];
    const mlp_u32x4 bias_v = b1_l[scc * 4 + hf], bias_w = b1_l[scc * 4 + 2 + hf];
    mlp_finish(h, bias_v, bias_w, zero4, true, hv);
    mlp_u32x4* hb = h_l + (r & 1) * (32 * HP);
#pragma unroll
    for (int gp = 0; gp < 2; ++gp) hb[l32 * HP + w * 4 + 2 * gp + hf] = sc_ok ? hv[gp] : zero4[0];     // past the last slice: zeros
    __syncthreads();
    // ---- second product: this wave's 32 output features over the round's T slices.  One barrier per round: the
    // other H buffer is written next, and nobody writes this one again before the barrier after that
    int ho = l32 * HP + hf;
    asm volatile("" : "+v"(ho));
    mlp_u32x4 gb[3] = {hb[ho], hb[ho + 2], hb[ho + 4]};
#pragma unroll
    for (int i = 0; i < 2 * T; ++i) {                                       // i = 2 * (slice of the round) + step
      out = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(mlp_bf16x8, wf[i]), __builtin_bit_cast(mlp_bf16x8, gb[i % 3]), out, 0, 0, 0);
      if (i + 3 < 2 * T) gb[i % 3] = hb[ho + 2 * (i + 3)];
      wf[i] = wload(rw, (nsc * KK + i) * 1024);                             // the wave's slice of the next round (after the last: a copy, unused)
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
#pragma unroll
    for (int i = 0; i < 2 * T; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
  }

  if constexpr (LNOUT == 2) {       // first fragments of the Linear that follows, under the epilogue below
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) wf[kk] = wload(rq, (w * KK + kk) * 1024);
  }
  // every wave holds its 32 features of Y^T complete: bias, residual, two 16-byte stores per lane
  if constexpr (PROJ) { resid[0] = r_l[l32 * XP + w * 4 + hf]; resid[1] = r_l[l32 * XP + w * 4 + 2 + hf]; }
  else if (g.residual) {          // (asked for here, not before the rounds: eight more live registers there mean spills)
    const bf16_t* R = (const bf16_t*)g.residual;
    resid[0] = *(const mlp_u32x4*)(R + ro + fo);
    resid[1] = *(const mlp_u32x4*)(R + ro + fo + 16);
  }
  const mlp_u32x4 b2v = *(const mlp_u32x4*)((const bf16_t*)g.b2 + fo), b2w = *(const mlp_u32x4*)((const bf16_t*)g.b2 + fo + 16);
  mlp_u32x4 yv[2];
  mlp_finish(out, b2v, b2w, resid, false, yv);
  if (row_ok) {
    bf16_t* Y = (bf16_t*)g.Y;
    *(mlp_u32x4*)(Y + ro + fo) = yv[0];
    *(mlp_u32x4*)(Y + ro + fo + 16) = yv[1];
  }
  if constexpr (LNOUT != 0) {
    // two-pass fp32 statistics of the bf16 row, as the norm kernel would compute them from the stored Y: a lane holds
    // 16 of its token's features, its partner lane (other hf) 16 more, the other waves the rest
    const mlp_u32x4 gv[2] = {*(const mlp_u32x4*)((const bf16_t*)g.ln2_gamma + fo), *(const mlp_u32x4*)((const bf16_t*)g.ln2_gamma + fo + 16)};
    const mlp_u32x4 bv[2] = {*(const mlp_u32x4*)((const bf16_t*)g.ln2_beta + fo), *(const mlp_u32x4*)((const bf16_t*)g.ln2_beta + fo + 16)};
    float f[16];
    mlp_unpack8(yv[0], f);
    mlp_unpack8(yv[1], f + 8);
    float sum = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) sum += f[e];
    sum += __shfl_xor(sum, 32, 64);
    if (hf == 0) st_l[w * 32 + l32] = sum;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int ww = 0; ww < T; ++ww) tot += st_l[ww * 32 + l32];
    const float mean = tot / (float)C;
    float var = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) { const float d = f[e] - mean; var += d * d; }
    var += __shfl_xor(var, 32, 64);
    if (hf == 0) st_l[(T + w) * 32 + l32] = var;
    __syncthreads();
    tot = 0.f;
#pragma unroll
    for (int ww = 0; ww < T; ++ww) tot += st_l[(T + ww) * 32 + l32];
    const float rstd = rsqrtf(tot / (float)C + g.ln2_eps), sh = -mean * rstd;
    mlp_u32x4 nv[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      float gf[8], bf[8];
      mlp_unpack8(gv[q], gf);
      mlp_unpack8(bv[q], bf);
#pragma unroll
      for (int e = 0; e < 4; ++e)
        nv[q][e] = mlp_pack2(fmaf(fmaf(f[8 * q + 2 * e], rstd, sh), gf[2 * e], bf[2 * e]), fmaf(fmaf(f[8 * q + 2 * e + 1], rstd, sh), gf[2 * e + 1], bf[2 * e + 1]));
    }
    if constexpr (LNOUT == 1) {
      if (row_ok) {
        bf16_t* Y2 = (bf16_t*)g.Y2;
        *(mlp_u32x4*)(Y2 + ro2 + fo) = nv[0];
        *(mlp_u32x4*)(Y2 + ro2 + fo + 16) = nv[1];
      }
    } else {
      static_assert(LNOUT != 2 || PROJ, "the fused following Linear needs the projection variant's spare LDS tile");
      // the normalised tile (bf16, as a norm kernel would have stored it) into the A tile's LDS, the following
      // Linear's bias over the first bias (both dead by now), then wave w forms outputs 32 (w + T j) ..+31, j < 3
      mlp_u32x4* n_l = a_l;
      n_l[l32 * XP + w * 4 + hf] = nv[0];
      n_l[l32 * XP + w * 4 + 2 + hf] = nv[1];
      for (int s = tid; s < 3 * XS; s += NTHR) b1_l[s] = ((const mlp_u32x4*)g.bq)[s];
      __syncthreads();
      bf16_t* Q = (bf16_t*)g.Y2;
      const int64_t qo = ro2 * 3;                       // same row map, rows three times as long
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        const int sc = w + T * j;
        const mlp_u32x4 bias_v = b1_l[sc * 4 + hf], bias_w = b1_l[sc * 4 + 2 + hf];
        int no = l32 * XP + hf;
        asm volatile("" : "+v"(no));
        mlp_f32x16 h;
#pragma unroll
        for (int e = 0; e < 16; ++e) h[e] = 0.f;
        mlp_u32x4 fb[3] = {n_l[no], n_l[no + 2], n_l[no + 4]};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          h = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(mlp_bf16x8, wf[kk]), __builtin_bit_cast(mlp_bf16x8, fb[kk % 3]), h, 0, 0, 0);
          if (kk + 3 < KK) fb[kk % 3] = n_l[no + 2 * (kk + 3)];
          if (j < 2) wf[kk] = wload(rq, ((sc + T) * KK + kk) * 1024);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        mlp_u32x4 qv[2];
        mlp_finish(h, bias_v, bias_w, zero4, false, qv);
        if (row_ok) {
          // (assembly: with stores pending next to loads the compiler's wait counting falls back to waiting for all
          // of them before the next slice's first fragment; its counts stay safe, see lin32_kernel)
          bf16_t* qp = Q + qo + sc * 32 + hf * 8;
          asm volatile("global_store_dwordx4 %0, %1, off\n\tglobal_store_dwordx4 %0, %2, off offset:32\n\ts_nop 2" :: "v"(qp), "v"(qv[0]), "v"(qv[1]) : "memory");
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------------------------
// The fused MLP for wide rows (C = 512): Y = residual + W2 . gelu(W1 . LayerNorm(x) + b1) + b2 with a tile of 64 tokens
// per workgroup and eight waves, each owning 64 output features.  With 32 tokens every weight fragment feeds one MFMA
// and the stream of fragments from L2 sets the pace; here a fragment of W1 feeds two MFMAs (the two token blocks) and
// in the second product two weight fragments and two hidden fragments feed four, so per MFMA half a KiB comes from L2
// and half a KiB from LDS.  Rounds of 256 hidden units: wave w forms slice 8 r + w of the round (32 hidden units x 64
// tokens: bias, GELU, bf16 into the round's hidden tile in LDS, double-buffered, one barrier per round), then adds
// the round to its 64 x 64 block of Y^T.  Same packed weight layout as the kernel above (mlp_pack_kernel).  The weight
// stream of a wave (blocks of 32 fragments: a W1 slice, or a round's W2 fragments in (step, feature block) order) runs
// through a ring of 16 fragment registers: each is refilled, right after the MFMAs that read it, with the fragment 16
// places on.
template <int C>
__global__ __launch_bounds__(C, (C >= 384 ? 1 : 2)) void mlp64_kernel(MlpArgs g) {
  constexpr int KK = C / 16, XS = C / 8, XP = XS + 1, NW = C / 64, NTHR = 64 * NW, RING = KK % 16 == 0 ? 16 : 8;
  constexpr int UG = NW / 2;                            // steps of the second product between two quarters of the bias + GELU work
  constexpr int HP = 4 * NW + 1;                        // slots of a token's row of the round's hidden tile (+1: odd pitch)
  constexpr size_t TILE = (size_t)64 * XP * 16, HTILE = (size_t)64 * HP * 16;
  static_assert(C % 64 == 0 && KK % RING == 0 && 4 * NW == KK && NW % 2 == 0, "the ring position of a fragment must be a compile-time constant");
  const SM_KARG MlpArgs* gk = kernarg_ptr<MlpArgs>();
  extern __shared__ __align__(16) unsigned char smem_raw[];
  mlp_u32x4* x_l = (mlp_u32x4*)smem_raw;                               // [64][XP] token tile, normalised in place
  mlp_u32x4* h_l = (mlp_u32x4*)(smem_raw + TILE);                      // [2][64][HP]
  mlp_u32x4* b1_l = (mlp_u32x4*)(smem_raw + TILE + 2 * HTILE);         // [Hd / 8]
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t row0 = (int64_t)blockIdx.x * 64;
  const int Hd = g.Hd, nsub = Hd >> 5, rounds = nsub / NW;
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.Wp), 0, 4 * Hd * C, 0x00020000);
  const int lo = lane * 16;
  auto wload = [&](int soff) __attribute__((always_inline)) { return __builtin_amdgcn_raw_buffer_load_b128(rw, lo, soff, 0); };
  // The wave's weight stream in blocks of 32 fragments: W1 slice of round 0; then, for every further round r, the W1
  // slice of round r followed by the W2 fragments of round r - 1 (step, feature block); last the W2 fragments of the last
  // round.  Byte offset of fragment s of block b (s may run into the next block; past the last block that one again).
  const int last_blk = 2 * rounds - 1;
  auto foff = [&](int b, int s) __attribute__((always_inline)) -> int {
    if (s >= KK) { b += 1; s -= KK; }
    b = b < last_blk ? b : last_blk;
    const bool w2 = b == last_blk || (b != 0 && !(b & 1));
    const int rr = b == last_blk ? rounds - 1 : (b & 1 ? (b + 1) >> 1 : (b ? (b >> 1) - 1 : 0));
    return w2 ? 2 * Hd * C + (((2 * w + (s & 1)) * nsub + NW * rr) * 2 + (s >> 1)) * 1024 : ((NW * rr + w) * KK + s) * 1024;
  };
  mlp_u32x4 wf[RING];
#pragma unroll
  for (int s = 0; s < RING; ++s) wf[s] = wload(foff(0, s));

  // the lane's two token rows (one per token block): offsets for the residual and the store
  int64_t ro[2]; bool row_ok[2];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb) {
    const int64_t row = row0 + 32 * tb + l32;
    row_ok[tb] = row < g.M;
    const int64_t prow = row_ok[tb] ? row : g.M - 1;
    ro[tb] = g.y_rows.identity ? prow * g.y_rows.ld : eval_rows_k(&gk->y_rows, prow);
  }
  mlp_load_x_tile<C, NTHR>(x_l, (const bf16_t*)g.X, row0, g.M, g.x_rows.identity, g.x_rows.ld, &gk->x_rows);
  if (row0 + 32 < g.M) mlp_load_x_tile<C, NTHR>(x_l + 32 * XP, (const bf16_t*)g.X, row0 + 32, g.M, g.x_rows.identity, g.x_rows.ld, &gk->x_rows);
  else for (int s = tid; s < 32 * XP; s += NTHR) x_l[32 * XP + s] = mlp_u32x4{0u, 0u, 0u, 0u};
  for (int s = tid; s < Hd / 8; s += NTHR) b1_l[s] = ((const mlp_u32x4*)g.b1)[s];
  __syncthreads();
  if (g.norm) {
    mlp_norm_x_tile<C, 64>(x_l, g.norm_eps, (const mlp_u32x4*)g.norm_gamma, (const mlp_u32x4*)g.norm_beta);
    __syncthreads();
  }

  mlp_f32x16 out[2][2];                                 // [feature block][token block]
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) out[i >> 1][i & 1][e] = 0.f;
  const mlp_u32x4 zero4[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};

  // first product of round r: slice NW r + w of the hidden units, both token blocks (block `blk` of the stream)
  auto first = [&](int blk, mlp_f32x16 (&h)[2]) __attribute__((always_inline)) {
    int xo = l32 * XP + hf;
    asm volatile("" : "+v"(xo));                        // opaque per round: the X fragments are re-read, not hoisted
#pragma unroll
    for (int e = 0; e < 16; ++e) { h[0][e] = 0.f; h[1][e] = 0.f; }
    mlp_u32x4 fa[2][2] = {{x_l[xo], x_l[xo + 32 * XP]}, {x_l[xo + 2], x_l[xo + 2 + 32 * XP]}};     // two steps ahead
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const mlp_bf16x8 wv = __builtin_bit_cast(mlp_bf16x8, wf[kk % RING]);
      h[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, __builtin_bit_cast(mlp_bf16x8, fa[kk & 1][0]), h[0], 0, 0, 0);
      h[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, __builtin_bit_cast(mlp_bf16x8, fa[kk & 1][1]), h[1], 0, 0, 0);
      wf[kk % RING] = wload(foff(blk, kk + RING));
      if (kk + 2 < KK) { fa[kk & 1][0] = x_l[xo + 2 * (kk + 2)]; fa[kk & 1][1] = x_l[xo + 2 * (kk + 2) + 32 * XP]; }
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
  };
  // bias + GELU of a quarter (token block u / 2, half u % 2 of its 32 hidden units) of the slice just formed, bf16, into `hb`
  auto finish_unit = [&](int r, int u, const mlp_f32x16 (&h)[2], mlp_u32x4* hb) __attribute__((always_inline)) {
    const int sc = NW * r + w, tb = u >> 1, gp = u & 1;
    hb[(32 * tb + l32) * HP + w * 4 + 2 * gp + hf] = mlp_finish_half(h[tb], gp, b1_l[sc * 4 + 2 * gp + hf], zero4[0], true);
  };
  // second product of a round: the wave's 64 features over the 256 hidden units of tile `hp` (16 steps), both token
  // blocks.  between(q), q < 4, runs after every UG steps.
  auto second = [&](int blk, const mlp_u32x4* hp, auto between) __attribute__((always_inline)) {
    int ho = l32 * HP + hf;
    asm volatile("" : "+v"(ho));
    mlp_u32x4 ga[2][2] = {{hp[ho], hp[ho + 32 * HP]}, {hp[ho + 2], hp[ho + 2 + 32 * HP]}};
#pragma unroll
    for (int i = 0; i < 2 * NW; ++i) {
#pragma unroll
      for (int bt = 0; bt < 2; ++bt) {
        const int s = 2 * i + bt;
        const mlp_bf16x8 wv = __builtin_bit_cast(mlp_bf16x8, wf[s % RING]);
        out[bt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, __builtin_bit_cast(mlp_bf16x8, ga[i & 1][0]), out[bt][0], 0, 0, 0);
        out[bt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, __builtin_bit_cast(mlp_bf16x8, ga[i & 1][1]), out[bt][1], 0, 0, 0);
        wf[s % RING] = wload(foff(blk, s + RING));
      }
      if (i + 2 < 2 * NW) { ga[i & 1][0] = hp[ho + 2 * (i + 2)]; ga[i & 1][1] = hp[ho + 2 * (i + 2) + 32 * HP]; }
      if (i % UG == UG - 1) {
        __builtin_amdgcn_sched_barrier(0);
        between(i / UG);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  // Rounds, software-pipelined: the second product of round r - 1 (matrix cores) alternates, a quarter at a time, with
  // the bias + GELU of round r's slice (vector ALU).  A barrier per round puts all waves of the workgroup in the same
  // phase; alternating in short stretches lets the two waves of a SIMD cover each other's vector work with MFMAs.
  {
    mlp_f32x16 h[2];
    first(0, h);
#pragma unroll
    for (int u = 0; u < 4; ++u) finish_unit(0, u, h, h_l);
    __syncthreads();
    for (int r = 1; r < rounds; ++r) {
      first(2 * r - 1, h);
      mlp_u32x4* hb = h_l + (r & 1) * (64 * HP);
      second(2 * r, h_l + ((r - 1) & 1) * (64 * HP), [&](int q) __attribute__((always_inline)) { finish_unit(r, q, h, hb); });
      __syncthreads();
    }
    second(last_blk, h_l + ((rounds - 1) & 1) * (64 * HP), [&](int) __attribute__((always_inline)) {});
  }

  // every wave holds its 64 features of Y^T for the 64 tokens: bias, residual, two 16-byte stores per block and lane
  bf16_t* Y = (bf16_t*)g.Y;
  const bf16_t* R = (const bf16_t*)g.residual;
#pragma unroll
  for (int bt = 0; bt < 2; ++bt) {
    const int fo = (2 * w + bt) * 32 + hf * 8;
    const mlp_u32x4 b2v = *(const mlp_u32x4*)((const bf16_t*)g.b2 + fo), b2w = *(const mlp_u32x4*)((const bf16_t*)g.b2 + fo + 16);
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      mlp_u32x4 resid[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
      if (R) { resid[0] = *(const mlp_u32x4*)(R + ro[tb] + fo); resid[1] = *(const mlp_u32x4*)(R + ro[tb] + fo + 16); }
      mlp_u32x4 yv[2];
      mlp_finish(out[bt][tb], b2v, b2w, resid, false, yv);
      if (row_ok[tb]) {
        *(mlp_u32x4*)(Y + ro[tb] + fo) = yv[0];
        *(mlp_u32x4*)(Y + ro[tb] + fo + 16) = yv[1];
      }
    }
  }
}

// mlp64_kernel with the attention output projection in front and, optionally, the next block's LayerNorm-1 (LNOUT = 1)
// or LayerNorm-1 + QKV Linear (LNOUT = 2) behind it: the C = 512 form of mlp_fused_kernel<C, true, LNOUT>, 64-token
// tiles.  x1 = A . Wproj^T + bproj + x0 (x0 read and Y written through y_rows); x1 (bf16) goes to LDS, where it is
// normalised for the first product, and to Y in memory, from where every lane reads back what it stored itself as the
// residual of the final sum (three 64-token tiles do not fit the LDS).  LDS: [x1 normalised | A tile, then the two
// hidden tiles, then the normalised Y for the QKV Linear | b1, then bq | bproj | row statistics].
// One weight stream per wave through the ring of 16 fragment registers, in blocks of 32 fragments: two blocks of Wproj
// ((step, feature block) order, the wave's two slices of lin_pack_kernel's layout), the blocks of mlp64_kernel, then
// the wave's six QKV slices.
template <int C, int LNOUT>
__global__ __launch_bounds__(C, (C >= 384 ? 1 : 2)) void mlp64p_kernel(MlpArgs g) {
  constexpr int KK = C / 16, XS = C / 8, XP = XS + 1, NW = C / 64, NTHR = 64 * NW, RING = KK % 16 == 0 ? 16 : 8, HP = 4 * NW + 1, NQ = 3 * C / 32 / NW;
  constexpr int UG = NW / 2;                            // steps of the second product between two quarters of the bias + GELU work
  constexpr size_t TILE = (size_t)64 * XP * 16, HTILE = (size_t)64 * HP * 16;
  static_assert(C % 64 == 0 && KK % RING == 0 && 4 * NW == KK && NW % 2 == 0 && 2 * HTILE >= TILE, "block and alias assumptions");
  const SM_KARG MlpArgs* gk = kernarg_ptr<MlpArgs>();
  extern __shared__ __align__(16) unsigned char smem_raw[];
  mlp_u32x4* x_l = (mlp_u32x4*)smem_raw;                               // [64][XP] x1, normalised in place
  mlp_u32x4* a_l = (mlp_u32x4*)(smem_raw + TILE);                      // [64][XP] attention output; dead after the projection
  mlp_u32x4* h_l = a_l;                                                // [2][64][HP] hidden tiles
  mlp_u32x4* n_l = a_l;                                                // [64][XP] normalised Y (LNOUT = 2), after the last round
  mlp_u32x4* b1_l = (mlp_u32x4*)(smem_raw + TILE + 2 * HTILE);         // [Hd / 8], later bq [3 C / 8]
  mlp_u32x4* bp_l = b1_l + g.Hd / 8;                                   // [C / 8]
  float* st_l = (float*)(bp_l + XS);                                   // [2][NW][64] row statistics
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t row0 = (int64_t)blockIdx.x * 64;
  const int Hd = g.Hd, nsub = Hd >> 5, rounds = nsub / NW;
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.Wp), 0, 4 * Hd * C, 0x00020000);
  const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.Wproj_p), 0, 2 * C * C, 0x00020000);
  const __amdgpu_buffer_rsrc_t rq = LNOUT == 2 ? __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.Wq_p), 0, 6 * C * C, 0x00020000) : rw;
  const int lo = lane * 16;
  // The wave's stream: 64 fragments of Wproj ((step, feature block) order), the MLP's blocks of 32 (see mlp64_kernel),
  // then NQ blocks of the QKV weight.  Which weight a refill reads is known where it is written, so each kind has its
  // own loader (descriptor and offset scalar) and the MFMA loops stay straight-line code.
  const int lastm = 2 * rounds - 1;
  auto frag_p = [&](int t) __attribute__((always_inline)) {          // t < 64: step t / 2, feature block t % 2
    return __builtin_amdgcn_raw_buffer_load_b128(rp, lo, ((2 * w + (t & 1)) * KK + (t >> 1)) * 1024, 0);
  };
  auto frag_m = [&](int m, int s) __attribute__((always_inline)) {   // fragment s of MLP block m (s >= KK: of block m + 1)
    if (s >= KK) { m += 1; s -= KK; }
    m = m < lastm ? m : lastm;
    const bool w2 = m == lastm || (m != 0 && !(m & 1));
    const int rr = m == lastm ? rounds - 1 : (m & 1 ? (m + 1) >> 1 : (m ? (m >> 1) - 1 : 0));
    return __builtin_amdgcn_raw_buffer_load_b128(rw, lo, w2 ? 2 * Hd * C + (((2 * w + (s & 1)) * nsub + NW * rr) * 2 + (s >> 1)) * 1024
                                                            : ((NW * rr + w) * KK + s) * 1024, 0);
  };
  auto frag_q = [&](int j, int s) __attribute__((always_inline)) {   // fragment s of the wave's j-th QKV slice
    if (s >= KK) { j += 1; s -= KK; }
    j = j < NQ ? j : NQ - 1;
    return __builtin_amdgcn_raw_buffer_load_b128(rq, lo, ((w + NW * j) * KK + s) * 1024, 0);
  };
  mlp_u32x4 wf[RING];
#pragma unroll
  for (int s = 0; s < RING; ++s) wf[s] = frag_p(s);

  int64_t ro[2], ro2[2] = {0, 0}; bool row_ok[2];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb) {
    const int64_t row = row0 + 32 * tb + l32;
    row_ok[tb] = row < g.M;
    const int64_t prow = row_ok[tb] ? row : g.M - 1;
    ro[tb] = g.y_rows.identity ? prow * g.y_rows.ld : eval_rows_k(&gk->y_rows, prow);
    if constexpr (LNOUT != 0) ro2[tb] = g.y2_rows.identity ? prow * g.y2_rows.ld : eval_rows_k(&gk->y2_rows, prow);
  }
  mlp_load_x_tile<C, NTHR>(a_l, (const bf16_t*)g.X, row0, g.M, g.x_rows.identity, g.x_rows.ld, &gk->x_rows);
  if (row0 + 32 < g.M) mlp_load_x_tile<C, NTHR>(a_l + 32 * XP, (const bf16_t*)g.X, row0 + 32, g.M, g.x_rows.identity, g.x_rows.ld, &gk->x_rows);
  else for (int s = tid; s < 32 * XP; s += NTHR) a_l[32 * XP + s] = mlp_u32x4{0u, 0u, 0u, 0u};
  for (int s = tid; s < Hd / 8; s += NTHR) b1_l[s] = ((const mlp_u32x4*)g.b1)[s];
  for (int s = tid; s < XS; s += NTHR) bp_l[s] = ((const mlp_u32x4*)g.bproj)[s];
  __syncthreads();

  mlp_f32x16 out[2][2];                                 // [feature block][token block]: the projection, then Y^T
  const mlp_u32x4 zero4[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
  auto clear_out = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) out[i >> 1][i & 1][e] = 0.f;
  };
  // out[bt][tb] += W(step i, feature block bt) x tile(token block tb, step i) for `steps` steps: the wave's 64 features
  // against a 64-token tile in LDS (row pitch `pitch` slots); refill(t) loads the fragment at position t of the call's
  // stream (t >= 2 * steps: what follows it).  between(q) after steps 4 q .. 4 q + 3.
  auto pair_product = [&](const mlp_u32x4* tile, int pitch, int steps, auto refill, auto between) __attribute__((always_inline)) {
    int to = l32 * pitch + hf;
    asm volatile("" : "+v"(to));
    const int hi = 32 * pitch;
    mlp_u32x4 ga[2][2] = {{tile[to], tile[to + hi]}, {tile[to + 2], tile[to + 2 + hi]}};
#pragma unroll
    for (int i = 0; i < KK; ++i) {
      if (i < steps) {
#pragma unroll
        for (int bt = 0; bt < 2; ++bt) {
          const int t = 2 * i + bt;
          const mlp_bf16x8 wv = __builtin_bit_cast(mlp_bf16x8, wf[t % RING]);
          out[bt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, __builtin_bit_cast(mlp_bf16x8, ga[i & 1][0]), out[bt][0], 0, 0, 0);
          out[bt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, __builtin_bit_cast(mlp_bf16x8, ga[i & 1][1]), out[bt][1], 0, 0, 0);
          wf[t % RING] = refill(t + RING);
        }
        if (i + 2 < steps) { ga[i & 1][0] = tile[to + 2 * (i + 2)]; ga[i & 1][1] = tile[to + 2 * (i + 2) + hi]; }
        if (i % UG == UG - 1 && i / UG < 4) {
          __builtin_amdgcn_sched_barrier(0);
          between(i / UG);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  };
  // h[tb] = W(slice of block blk) x tile(token block tb): 32 hidden / output features of a slice for the 64 tokens
  // between(q), q < 4, after every KK / 4 steps
  auto slice_product = [&](const mlp_u32x4* tile, mlp_f32x16 (&h)[2], auto refill, auto between) __attribute__((always_inline)) {
    int xo = l32 * XP + hf;
    asm volatile("" : "+v"(xo));
#pragma unroll
    for (int e = 0; e < 16; ++e) { h[0][e] = 0.f; h[1][e] = 0.f; }
    mlp_u32x4 fa[2][2] = {{tile[xo], tile[xo + 32 * XP]}, {tile[xo + 2], tile[xo + 2 + 32 * XP]}};
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const mlp_bf16x8 wv = __builtin_bit_cast(mlp_bf16x8, wf[kk % RING]);
      h[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, __builtin_bit_cast(mlp_bf16x8, fa[kk & 1][0]), h[0], 0, 0, 0);
      h[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, __builtin_bit_cast(mlp_bf16x8, fa[kk & 1][1]), h[1], 0, 0, 0);
      wf[kk % RING] = refill(kk + RING);
      if (kk + 2 < KK) { fa[kk & 1][0] = tile[xo + 2 * (kk + 2)]; fa[kk & 1][1] = tile[xo + 2 * (kk + 2) + 32 * XP]; }
      if (kk % (KK / 4) == KK / 4 - 1) {
        __builtin_amdgcn_sched_barrier(0);
        between(kk / (KK / 4));
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  auto nothing = [&](int) __attribute__((always_inline)) {};
  bf16_t* Y = (bf16_t*)g.Y;

  // ---- projection: x1 = A . Wproj^T + bproj + x0 for the wave's 64 features
  clear_out();
  pair_product(a_l, XP, KK, [&](int t) __attribute__((always_inline)) { return t < 2 * KK ? frag_p(t) : frag_m(0, t - 2 * KK); }, nothing);
  {
    const bf16_t* R0 = (const bf16_t*)g.resid0;
#pragma unroll
    for (int bt = 0; bt < 2; ++bt) {
      const int fb = 2 * w + bt, fo = fb * 32 + hf * 8;
      const mlp_u32x4 bias_v = bp_l[fb * 4 + hf], bias_w = bp_l[fb * 4 + 2 + hf];
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) {
        const mlp_u32x4 res[2] = {*(const mlp_u32x4*)(R0 + ro[tb] + fo), *(const mlp_u32x4*)(R0 + ro[tb] + fo + 16)};
        mlp_u32x4 xv[2];
        mlp_finish(out[bt][tb], bias_v, bias_w, res, false, xv);          // x1 rounded to bf16, as the separate Linear stores it
#pragma unroll
        for (int gp = 0; gp < 2; ++gp) x_l[(32 * tb + l32) * XP + fb * 4 + 2 * gp + hf] = xv[gp];
        if (row_ok[tb]) {                                                  // the residual of the final sum, read back below
          *(mlp_u32x4*)(Y + ro[tb] + fo) = xv[0];
          *(mlp_u32x4*)(Y + ro[tb] + fo + 16) = xv[1];
        }
      }
    }
  }
  __syncthreads();
  mlp_norm_x_tile<C, 64>(x_l, g.norm_eps, (const mlp_u32x4*)g.norm_gamma, (const mlp_u32x4*)g.norm_beta);
  __syncthreads();

  // ---- the MLP's rounds, as in mlp64_kernel (stream blocks 2 ..)
  clear_out();
  auto finish_unit = [&](int r, int u, const mlp_f32x16 (&h)[2], mlp_u32x4* hb) __attribute__((always_inline)) {
    const int sc = NW * r + w, tb = u >> 1, gp = u & 1;
    hb[(32 * tb + l32) * HP + w * 4 + 2 * gp + hf] = mlp_finish_half(h[tb], gp, b1_l[sc * 4 + 2 * gp + hf], zero4[0], true);
  };
  {
    mlp_f32x16 h[2];
    slice_product(x_l, h, [&](int s) __attribute__((always_inline)) { return frag_m(0, s); }, nothing);
#pragma unroll
    for (int u = 0; u < 4; ++u) finish_unit(0, u, h, h_l);
    __syncthreads();
    for (int r = 1; r < rounds; ++r) {
      slice_product(x_l, h, [&](int s) __attribute__((always_inline)) { return frag_m(2 * r - 1, s); }, nothing);
      mlp_u32x4* hb = h_l + (r & 1) * (64 * HP);
      pair_product(h_l + ((r - 1) & 1) * (64 * HP), HP, 2 * NW, [&](int s) __attribute__((always_inline)) { return frag_m(2 * r, s); },
                   [&](int q) __attribute__((always_inline)) { finish_unit(r, q, h, hb); });
      __syncthreads();
    }
    // the last block of the MLP: what follows it in the stream is the first QKV slice (or nothing)
    pair_product(h_l + ((rounds - 1) & 1) * (64 * HP), HP, 2 * NW,
                 [&](int s) __attribute__((always_inline)) { return (LNOUT == 2 && s >= KK) ? frag_q(0, s - KK) : frag_m(lastm, s < KK ? s : KK - 1); }, nothing);
  }

  // ---- Y = x1 + MLP: bias, the residual this lane stored above, two 16-byte stores per block and lane
  mlp_u32x4 yv[2][2][2];
#pragma unroll
  for (int bt = 0; bt < 2; ++bt) {
    const int fo = (2 * w + bt) * 32 + hf * 8;
    const mlp_u32x4 b2v = *(const mlp_u32x4*)((const bf16_t*)g.b2 + fo), b2w = *(const mlp_u32x4*)((const bf16_t*)g.b2 + fo + 16);
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      const mlp_u32x4 resid[2] = {*(const mlp_u32x4*)(Y + ro[tb] + fo), *(const mlp_u32x4*)(Y + ro[tb] + fo + 16)};
      mlp_finish(out[bt][tb], b2v, b2w, resid, false, yv[bt][tb]);
      if (row_ok[tb]) {
        *(mlp_u32x4*)(Y + ro[tb] + fo) = yv[bt][tb][0];
        *(mlp_u32x4*)(Y + ro[tb] + fo + 16) = yv[bt][tb][1];
      }
    }
  }
  if constexpr (LNOUT != 0) {
    // LayerNorm of the bf16 rows of Y (two-pass fp32 statistics, as the norm kernel computes them from the stored
    // tensor): a lane holds 32 of its token's features per token block, its partner lane 32 more, the other waves the rest
    float mean[2], rstd[2];
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) {
        float acc = 0.f;
#pragma unroll
        for (int bt = 0; bt < 2; ++bt)
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            float f[8];
            mlp_unpack8(yv[bt][tb][q], f);
#pragma unroll
            for (int e = 0; e < 8; ++e) { const float d = pass ? f[e] - mean[tb] : f[e]; acc += pass ? d * d : d; }
          }
        acc += __shfl_xor(acc, 32, 64);
        if (hf == 0) st_l[(pass * NW + w) * 64 + 32 * tb + l32] = acc;
      }
      __syncthreads();
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) {
        float tot = 0.f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) tot += st_l[(pass * NW + ww) * 64 + 32 * tb + l32];
        if (pass == 0) mean[tb] = tot / (float)C; else rstd[tb] = rsqrtf(tot / (float)C + g.ln2_eps);
      }
    }
#pragma unroll
    for (int bt = 0; bt < 2; ++bt) {
      const int fb = 2 * w + bt, fo = fb * 32 + hf * 8;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        float gf[8], bf[8];
        mlp_unpack8(*(const mlp_u32x4*)((const bf16_t*)g.ln2_gamma + fo + 16 * q), gf);
        mlp_unpack8(*(const mlp_u32x4*)((const bf16_t*)g.ln2_beta + fo + 16 * q), bf);
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
          float f[8];
          mlp_unpack8(yv[bt][tb][q], f);
          const float sh = -mean[tb] * rstd[tb];
          mlp_u32x4 nv;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            nv[e] = mlp_pack2(fmaf(fmaf(f[2 * e], rstd[tb], sh), gf[2 * e], bf[2 * e]), fmaf(fmaf(f[2 * e + 1], rstd[tb], sh), gf[2 * e + 1], bf[2 * e + 1]));
          if constexpr (LNOUT == 1) {
            if (row_ok[tb]) *(mlp_u32x4*)((bf16_t*)g.Y2 + ro2[tb] + fo + 16 * q) = nv;
          } else {
            n_l[(32 * tb + l32) * XP + fb * 4 + 2 * q + hf] = nv;        // (the hidden tiles are dead: two barriers ago)
          }
        }
      }
    }
    if constexpr (LNOUT == 2) {
      // the next block's QKV Linear on the normalised tile: wave w forms outputs 32 (w + NW j) ..+31, j < NQ
      for (int s = tid; s < 3 * XS; s += NTHR) b1_l[s] = ((const mlp_u32x4*)g.bq)[s];
      __syncthreads();
      bf16_t* Q = (bf16_t*)g.Y2;
      // bias and store of slice j (a quarter at a time: token block u / 2, half u % 2 of its 32 outputs) are issued
      // between the quarters of slice j + 1's product
      auto emit = [&](int j, int u, const mlp_f32x16 (&h)[2]) __attribute__((always_inline)) {
        const int sc = w + NW * j, tb = u >> 1, gp = u & 1;
        const mlp_u32x4 qv = mlp_finish_half(h[tb], gp, b1_l[sc * 4 + 2 * gp + hf], zero4[0], false);
        if (row_ok[tb]) {
          bf16_t* qp = Q + 3 * ro2[tb] + sc * 32 + hf * 8 + 16 * gp;      // same row map, rows three times as long
          asm volatile("global_store_dwordx4 %0, %1, off\n\ts_nop 1" :: "v"(qp), "v"(qv) : "memory");
        }
      };
      static_assert(NQ % 2 == 0, "slices are taken two at a time");
      mlp_f32x16 ha[2], hb2[2];
      slice_product(n_l, ha, [&](int s) __attribute__((always_inline)) { return frag_q(0, s); }, nothing);
#pragma unroll 1
      for (int j = 0; j < NQ; j += 2) {
        slice_product(n_l, hb2, [&](int s) __attribute__((always_inline)) { return frag_q(j + 1, s); },
                      [&](int u) __attribute__((always_inline)) { emit(j, u, ha); });
        if (j + 2 < NQ) {
          slice_product(n_l, ha, [&](int s) __attribute__((always_inline)) { return frag_q(j + 2, s); },
                        [&](int u) __attribute__((always_inline)) { emit(j + 1, u, hb2); });
        } else {
#pragma unroll
          for (int u = 0; u < 4; ++u) emit(j + 1, u, hb2);
        }
      }
    }
  }
}

static size_t mlp64p_smem(int C, int Hd) {
  const int NW = C / 64;
  return (size_t)64 * (C / 8 + 1) * 16 + 2 * (size_t)64 * (4 * NW + 1) * 16 + (size_t)Hd * 2 + (size_t)C * 2 + (size_t)2 * NW * 64 * 4;
}

template <int C, int LNOUT>
static int mlp64p_launch(const MlpArgs& g, void* stream) {
  const size_t smem = mlp64p_smem(C, g.Hd);
  static std::atomic<size_t> allowed{0};
  if (smem > allowed.load()) {
    const hipError_t e = hipFuncSetAttribute((const void*)mlp64p_kernel<C, LNOUT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return (int)e;
    allowed.store(smem);
  }
  mlp64p_kernel<C, LNOUT><<<dim3((unsigned)((g.M + 63) / 64)), dim3(C), smem, (hipStream_t)stream>>>(g);
  return (int)hipGetLastError();
}

static size_t mlp64_smem(int C, int Hd) { return (size_t)64 * (C / 8 + 1) * 16 + 2 * (size_t)64 * (4 * (C / 64) + 1) * 16 + (size_t)Hd * 2; }
// shapes the 64-token kernels take: whole rounds of C / 2 hidden units
static bool mlp64_shape(int C, int Hd) { return (C == 256 || C == 384 || C == 512) && Hd >= C / 2 && Hd % (C / 2) == 0 && Hd <= 16384; }
// ... and where they are used: always at C = 512 (the 32-token kernels stop at 384); at 256 and 384 on grids of at least
// one workgroup of 64 tokens per CU (on smaller ones the 32-token tile fills more CUs); not at 128, where the 32-token
// kernel is faster (measured at 32768 tokens, MLP alone: C = 128 21 us against 32; 256: 66 against 51; 384: 147 against 122)
static bool mlp64_use(const MlpArgs& g) {
  if (!mlp64_shape(g.C, g.Hd)) return false;
  if (g.C == 512) return true;
  if (g.C == 128 || g.M < 64 * 256) return false;
  if (g.Wproj_p) return g.norm && g.Hd >= 3 * g.C && mlp64p_smem(g.C, g.Hd) <= 160 * 1024;
  return !g.Y2 && !g.Wq_p && mlp64_smem(g.C, g.Hd) <= 160 * 1024;
}

template <int C>
static int mlp64_launch(const MlpArgs& g, void* stream) {
  if (g.Wproj_p) {      // projection in front (the folded LayerNorm is part of that form), optionally the next block's norm / QKV
    if (!g.norm || g.Hd < 3 * C) return (int)hipErrorInvalidValue;
    if (g.Y2 && g.Wq_p) return mlp64p_launch<C, 2>(g, stream);
    return g.Y2 ? mlp64p_launch<C, 1>(g, stream) : mlp64p_launch<C, 0>(g, stream);
  }
  if (g.Y2 || g.Wq_p) return (int)hipErrorInvalidValue;
  const size_t smem = mlp64_smem(C, g.Hd);
  static std::atomic<size_t> allowed{0};
  if (smem > allowed.load()) {
    const hipError_t e = hipFuncSetAttribute((const void*)mlp64_kernel<C>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return (int)e;
    allowed.store(smem);
  }
  mlp64_kernel<C><<<dim3((unsigned)((g.M + 63) / 64)), dim3(C), smem, (hipStream_t)stream>>>(g);
  return (int)hipGetLastError();
}

static size_t mlp_smem(int C, int Hd, bool proj, bool lnout) {
  const size_t tile = (size_t)32 * (C / 8 + 1) * 16, htile = (size_t)32 * (C / 8 + 1) * 16;
  return (proj ? 3 : 1) * tile + 2 * htile + (size_t)Hd * 2 + (proj ? (size_t)C * 2 : 0) + (lnout ? (size_t)2 * (C / 32) * 32 * 4 : 0);
}

template <int C, bool PROJ, int LNOUT>
static int mlp_launch3(const MlpArgs& g, void* stream) {
  const size_t smem = mlp_smem(C, g.Hd, PROJ, LNOUT != 0);
  static std::atomic<size_t> allowed{0};   // raised on demand: the attribute is per kernel, the hidden size varies
  if (smem > allowed.load()) {
    const hipError_t e = hipFuncSetAttribute((const void*)mlp_fused_kernel<C, PROJ, LNOUT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return (int)e;
    allowed.store(smem);
  }
  const int64_t n_wg = (g.M + 31) / 32;
  mlp_fused_kernel<C, PROJ, LNOUT><<<dim3((unsigned)n_wg), dim3(64 * (C / 32)), smem, (hipStream_t)stream>>>(g);
  return (int)hipGetLastError();
}
template <int C>
static int mlp_launch(const MlpArgs& g, void* stream) {
  if (g.Wproj_p) {
    if (g.Y2 && g.Wq_p) return g.Hd >= 3 * C ? mlp_launch3<C, true, 2>(g, stream) : (int)hipErrorInvalidValue;   // (the following bias reuses the first bias's LDS)
    return g.Y2 ? mlp_launch3<C, true, 1>(g, stream) : mlp_launch3<C, true, 0>(g, stream);
  }
  if (g.Wq_p) return (int)hipErrorInvalidValue;
  return g.Y2 ? mlp_launch3<C, false, 1>(g, stream) : mlp_launch3<C, false, 0>(g, stream);
}

// LDS capacity: the projection variant holds three token tiles
bool mlp_proj_supported(int C, int Hd, int dtype) {
  if (!mlp_fused_supported(C, Hd, dtype)) return false;
  if (C == 512) return mlp64_shape(C, Hd) && Hd >= 3 * C && mlp64p_smem(C, Hd) <= 160 * 1024;
  return mlp_smem(C, Hd, true, true) <= 160 * 1024;
}

bool mlp_fused_supported(int C, int Hd, int dtype) {
  if (dtype != SM_BF16) return false;
  if (C == 512) return mlp64_shape(C, Hd) && mlp64_smem(C, Hd) <= 160 * 1024;      // wide rows: the 64-token kernels only
  return (C == 128 || C == 256 || C == 384) && Hd >= 32 && Hd % 32 == 0 && Hd <= 16384;
}

int launch_mlp_pack(const void* W1, const void* W2, int C, int Hd, void* packed, void* stream) {
  const int64_t n = 2 * ((int64_t)Hd * C / 8);
  mlp_pack_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>((const bf16_t*)W1, (const bf16_t*)W2, (mlp_u32x4*)packed, C, Hd);
  return (int)hipGetLastError();
}

int launch_mlp_fused(const MlpArgs& g, void* stream) {
  if (mlp64_use(g)) {
    switch (g.C) {
      case 256: return mlp64_launch<256>(g, stream);
      case 384: return mlp64_launch<384>(g, stream);
      case 512: return mlp64_launch<512>(g, stream);
    }
  }
  switch (g.C) {
    case 128: return mlp_launch<128>(g, stream);
    case 256: return mlp_launch<256>(g, stream);
    case 384: return mlp_launch<384>(g, stream);
  }
  return (int)hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------------------------------
// Linear for a short reduction dimension (K = C in {128, 256, 384}), Y = act(norm(X) . W^T + b) (+ residual): the first
// product of the kernel above on its own, with four waves.  A workgroup owns 32 token rows, whose K elements stay in LDS for all N outputs;
// the N / 32 row slices of W are dealt round-robin to the four waves and stream from L2 straight into MFMA operand
// registers (packed by lin_pack_kernel: fragment (slice sc, step kk) at sc * K/16 + kk, lane (l32, hf) =
// W[32 sc + l32][16 kk + 8 hf ..+7]); every wave finishes its 32 x 32 outputs in registers and stores them: no
// barrier after the prologue.  Against the tiled kernel of k_gemm.hip this trades L2 -> CU traffic (W once per 32
// rows) for the absence of K-loop barriers and of a separate norm kernel.  Measured (with LayerNorm, against norm
// kernel + tiled kernel resp. the tiled kernel's own folded norm): 200704 x 384 x 128: 69 us against 89;
// 50176 x 768 x 256: 55 against 71; 6272 x 1152 x 384: 23.7 against 26.
// NW waves per workgroup: 4 (two workgroups per CU, X fragments in registers: large grids) or C / 32 (one workgroup
// per CU with three waves per SIMD at C = 384, X fragments re-read from LDS: grids of about one workgroup per CU)
template <int C, bool RES, int NW>
__global__ __launch_bounds__(64 * NW, 1) void lin32_kernel(Lin32Args g) {
  constexpr int KK = C / 16, XS = C / 8, XP = XS + 1, NTHR = 64 * NW;
  constexpr bool XREG = NW <= 4;
  const SM_KARG Lin32Args* gk = kernarg_ptr<Lin32Args>();
  extern __shared__ __align__(16) unsigned char smem_raw[];
  mlp_u32x4* x_l = (mlp_u32x4*)smem_raw;                                  // [32][XP]
  mlp_u32x4* b_l = (mlp_u32x4*)(smem_raw + (size_t)32 * XP * 16);         // [N / 8]
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave index as a scalar: slice bases become scalar addresses
  const int64_t row0 = (int64_t)blockIdx.x * 32;
  const int nsub = g.N >> 5;
  const char* Wp = (const char*)g.Wp;

  // weight fragments by buffer loads: descriptor and fragment offset scalar, the lane's 16 bytes the only vector operand
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.Wp), 0, 2 * g.N * C, 0x00020000);
  const int lo = lane * 16;
  (void)Wp;
  mlp_u32x4 w1[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) w1[kk] = __builtin_amdgcn_raw_buffer_load_b128(rw, lo, ((w < nsub ? w : 0) * KK + kk) * 1024, 0);
  mlp_load_x_tile<C, NTHR>(x_l, (const bf16_t*)g.X, row0, g.M, g.x_rows.identity, g.x_rows.ld, &gk->x_rows);
  for (int s = tid; s < g.N / 8; s += NTHR) b_l[s] = g.bias ? ((const mlp_u32x4*)g.bias)[s] : mlp_u32x4{0u, 0u, 0u, 0u};
  __syncthreads();
  if (g.norm) {
    mlp_norm_x_tile<C>(x_l, g.norm_eps, (const mlp_u32x4*)g.norm_gamma, (const mlp_u32x4*)g.norm_beta);
    __syncthreads();
  }

  // the lane's X fragments do not depend on the slice: with four waves they stay in registers (K / 4 of them)
  mlp_u32x4 xf[XREG ? KK : 1];
  if constexpr (XREG) {
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) xf[kk] = x_l[l32 * XP + hf + 2 * kk];
  }
  const int64_t row = row0 + l32;                 // the lane's token: accumulator column
  const bool row_ok = row < g.M;
  const int64_t rowc = row_ok ? row : g.M - 1;    // lanes past M read the last row's residual and store nothing
  const int64_t ro = g.y_rows.identity ? rowc * g.y_rows.ld : eval_rows_k(&gk->y_rows, rowc);
  const bf16_t* R = (const bf16_t*)g.residual;
  bf16_t* Y = (bf16_t*)g.Y;
  const bool gelu_on = g.act == SM_ACT_GELU;
  // the slice loop is one basic block up to the final masked store, so that the issue order below holds; loads
  // that the epilogue needs are issued before the slice's weight prefetch (vector loads return in issue order)
  for (int sc = w; sc < nsub; sc += NW) {
    const int nx = sc + NW < nsub ? sc + NW : sc;
    int xo = l32 * XP + hf;
    if constexpr (!XREG) asm volatile("" : "+v"(xo));   // opaque per slice: fragments re-read from LDS, not kept in registers
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
    mlp_u32x4 fb[3] = {x_l[xo], x_l[xo + 2], x_l[xo + 4]};      // (!XREG) LDS fragments three steps ahead of their MFMA
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const mlp_u32x4 xv = XREG ? xf[XREG ? kk : 0] : fb[kk % 3];
      h = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(mlp_bf16x8, w1[kk]), __builtin_bit_cast(mlp_bf16x8, xv), h, 0, 0, 0);
      w1[kk] = __builtin_amdgcn_raw_buffer_load_b128(rw, lo, (nx * KK + kk) * 1024, 0);
      if (!XREG && kk + 3 < KK) fb[kk % 3] = x_l[xo + 2 * (kk + 3)];
    }
    __builtin_amdgcn_sched_group_barrier(0x100, XREG ? 2 : 5, 0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      if constexpr (!XREG) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    mlp_u32x4 outv[2];
    // (a literal flag in each branch: with a run-time flag the polynomial is evaluated for every value and thrown away)
    if (gelu_on) mlp_finish(h, bias_v, bias_w, res, true, outv); else mlp_finish(h, bias_v, bias_w, res, false, outv);
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

// The same Linear for wide rows (K = 512): 64 tokens per workgroup, eight waves, every weight fragment feeding two
// MFMAs (the two token blocks); the N / 32 slices of W are dealt round-robin to the waves and a wave's fragments run
// through a ring of 16 registers, as in mlp64_kernel.  LayerNorm folded as above.
template <int C, bool RES>
__global__ __launch_bounds__(512, 1) void lin64_kernel(Lin32Args g) {
  constexpr int KK = C / 16, XS = C / 8, XP = XS + 1, NW = 8, RING = 16;
  const SM_KARG Lin32Args* gk = kernarg_ptr<Lin32Args>();
  extern __shared__ __align__(16) unsigned char smem_raw[];
  mlp_u32x4* x_l = (mlp_u32x4*)smem_raw;                                  // [64][XP]
  mlp_u32x4* b_l = (mlp_u32x4*)(smem_raw + (size_t)64 * XP * 16);         // [N / 8]
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t row0 = (int64_t)blockIdx.x * 64;
  const int nsub = g.N >> 5;
  const int njobs = (nsub - w + NW - 1) / NW;                             // slices of this wave: w, w + NW, ...
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.Wp), 0, 2 * g.N * C, 0x00020000);
  const int lo = lane * 16;
  auto wload = [&](int soff) __attribute__((always_inline)) { return __builtin_amdgcn_raw_buffer_load_b128(rw, lo, soff, 0); };
  // fragment s of the wave's j-th slice (s may run into the next slice; past the last slice that one again)
  auto foff = [&](int j, int s) __attribute__((always_inline)) -> int {
    if (s >= KK) { j += 1; s -= KK; }
    j = j < njobs ? j : njobs - 1;
    return ((w + NW * (j > 0 ? j : 0)) * KK + s) * 1024;
  };
  mlp_u32x4 wf[RING];
#pragma unroll
  for (int s = 0; s < RING; ++s) wf[s] = wload(foff(0, s));
  int64_t ro[2]; bool row_ok[2];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb) {
    const int64_t row = row0 + 32 * tb + l32;
    row_ok[tb] = row < g.M;
    const int64_t prow = row_ok[tb] ? row : g.M - 1;
    ro[tb] = g.y_rows.identity ? prow * g.y_rows.ld : eval_rows_k(&gk->y_rows, prow);
  }
  mlp_load_x_tile<C, 512>(x_l, (const bf16_t*)g.X, row0, g.M, g.x_rows.identity, g.x_rows.ld, &gk->x_rows);
  if (row0 + 32 < g.M) mlp_load_x_tile<C, 512>(x_l + 32 * XP, (const bf16_t*)g.X, row0 + 32, g.M, g.x_rows.identity, g.x_rows.ld, &gk->x_rows);
  else for (int s = tid; s < 32 * XP; s += 512) x_l[32 * XP + s] = mlp_u32x4{0u, 0u, 0u, 0u};
  for (int s = tid; s < g.N / 8; s += 512) b_l[s] = g.bias ? ((const mlp_u32x4*)g.bias)[s] : mlp_u32x4{0u, 0u, 0u, 0u};
  __syncthreads();
  if (g.norm) {
    mlp_norm_x_tile<C, 64>(x_l, g.norm_eps, (const mlp_u32x4*)g.norm_gamma, (const mlp_u32x4*)g.norm_beta);
    __syncthreads();
  }
  const bf16_t* R = (const bf16_t*)g.residual;
  bf16_t* Y = (bf16_t*)g.Y;
  const bool gelu_on = g.act == SM_ACT_GELU;
  for (int j = 0; j < njobs; ++j) {
    const int sc = w + NW * j;
    int xo = l32 * XP + hf;
    asm volatile("" : "+v"(xo));                        // opaque per slice: the X fragments are re-read, not hoisted
    const mlp_u32x4 bias_v = b_l[sc * 4 + hf], bias_w = b_l[sc * 4 + 2 + hf];
    mlp_u32x4 res[2][2] = {{{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}}, {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}}};
    if constexpr (RES) {
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) {
        res[tb][0] = *(const mlp_u32x4*)(R + ro[tb] + sc * 32 + hf * 8);
        res[tb][1] = *(const mlp_u32x4*)(R + ro[tb] + sc * 32 + 16 + hf * 8);
      }
    }
    mlp_f32x16 h[2];
#pragma unroll
    for (int e = 0; e < 16; ++e) { h[0][e] = 0.f; h[1][e] = 0.f; }
    mlp_u32x4 fa[2][2] = {{x_l[xo], x_l[xo + 32 * XP]}, {x_l[xo + 2], x_l[xo + 2 + 32 * XP]}};     // two steps ahead
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const mlp_bf16x8 wv = __builtin_bit_cast(mlp_bf16x8, wf[kk % RING]);
      h[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, __builtin_bit_cast(mlp_bf16x8, fa[kk & 1][0]), h[0], 0, 0, 0);
      h[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, __builtin_bit_cast(mlp_bf16x8, fa[kk & 1][1]), h[1], 0, 0, 0);
      wf[kk % RING] = wload(foff(j, kk + RING));
      if (kk + 2 < KK) { fa[kk & 1][0] = x_l[xo + 2 * (kk + 2)]; fa[kk & 1][1] = x_l[xo + 2 * (kk + 2) + 32 * XP]; }
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      mlp_u32x4 outv[2];
      if (gelu_on) mlp_finish(h[tb], bias_v, bias_w, res[tb], true, outv); else mlp_finish(h[tb], bias_v, bias_w, res[tb], false, outv);
      if (row_ok[tb]) {
        // (assembly, as in lin32_kernel: with stores pending next to loads the compiler's wait counting falls back to
        // waiting for everything before the next slice's first fragment)
        bf16_t* yp = Y + ro[tb] + sc * 32 + hf * 8;
        asm volatile("global_store_dwordx4 %0, %1, off\n\tglobal_store_dwordx4 %0, %2, off offset:32\n\ts_nop 2"
                     :: "v"(yp), "v"(outv[0]), "v"(outv[1]) : "memory");
      }
    }
  }
}

template <int C>
static int lin64_launch(const Lin32Args& g, void* stream) {
  const size_t smem = (size_t)64 * (C / 8 + 1) * 16 + (size_t)g.N * 2;
  static std::atomic<size_t> allowed{0};
  if (smem > allowed.load()) {
    hipError_t e = hipFuncSetAttribute((const void*)lin64_kernel<C, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)lin64_kernel<C, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return (int)e;
    allowed.store(smem);
  }
  const dim3 grid((unsigned)((g.M + 63) / 64));
  if (g.residual) lin64_kernel<C, true><<<grid, dim3(512), smem, (hipStream_t)stream>>>(g);
  else lin64_kernel<C, false><<<grid, dim3(512), smem, (hipStream_t)stream>>>(g);
  return (int)hipGetLastError();
}

template <int C, bool RES, int NW>
static int lin32_launch3(const Lin32Args& g, void* stream) {
  const size_t smem = (size_t)32 * (C / 8 + 1) * 16 + (size_t)g.N * 2;
  static std::atomic<size_t> allowed{0};
  if (smem > allowed.load()) {
    const hipError_t e = hipFuncSetAttribute((const void*)lin32_kernel<C, RES, NW>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return (int)e;
    allowed.store(smem);
  }
  lin32_kernel<C, RES, NW><<<dim3((unsigned)((g.M + 31) / 32)), dim3(64 * NW), smem, (hipStream_t)stream>>>(g);
  return (int)hipGetLastError();
}
template <int C, bool RES>
static int lin32_launch2(const Lin32Args& g, void* stream) {
  // few workgroups (about one per CU) and enough slices to go round: C / 32 waves each
  if constexpr (C / 32 > 4) { if ((g.M + 31) / 32 <= 512 && g.N / 32 >= C / 32) return lin32_launch3<C, RES, C / 32>(g, stream); }
  return lin32_launch3<C, RES, 4>(g, stream);
}
template <int C>
static int lin32_launch(const Lin32Args& g, void* stream) {
  return g.residual ? lin32_launch2<C, true>(g, stream) : lin32_launch2<C, false>(g, stream);
}

bool lin32_supported(int N, int K, int dtype) {
  return dtype == SM_BF16 && (K == 128 || K == 256 || K == 384 || K == 512) && N >= 32 && N % 32 == 0 && N <= 16384;
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
    case 512: return lin64_launch<512>(g, stream);      // wide rows: 64-token tiles
  }
  return (int)hipErrorInvalidValue;
}

}  // namespace sm
