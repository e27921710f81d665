// Fused attention O = softmax(scale Q K^T + bias + mask) V reading Q, K, V in
// place through 4-D strides, so that head split / merge permutes and the
// q/k/v slices are address arithmetic (paper Sec. 3.2.1).  The paper treats
// QK^T, Softmax and AV as separate operators and names tiled attention as
// complementary (Sec. 6); here they are one ILD & Variable kernel.
//
// bf16 paths (matrix cores).  Scores are computed transposed, S^T = K Q^T, so
// that a lane holds one query (column) and 16 keys (rows): row max / sum are
// in-lane reductions plus one cross-half shuffle, the probabilities are already
// in the register layout the next MFMA wants as its B operand (O^T = V^T P^T),
// and the running rescale of O^T is lane-local.  Three kernels share that
// layout: attn_flash_kernel (global attention: K / V tiles through LDS, shared
// by the four waves of a workgroup), attn_window32_kernel (Swin windows of at
// most 64 tokens, head size 32) and attn_bf16_kernel (the general fallback: one
// wave per 32 queries, operands straight from global memory).  Window attention
// adds the relative-position bias gathered from its table and the
// shifted-window mask computed from the window's position: no bias or mask
// tensor is ever materialised.  attn_flash_kernel's stripe mode reads the stripes of
// CSwin's cross-shaped windows in place (two more strides per operand) and can add
// to its output; attn_stripe_pair_kernel puts the two halves of such an attention
// into one grid.
//
// fp32 path (window attention only): plain FMA kernel, one workgroup per
// (window, head), K / V / scores in LDS.
//
// dwconv3x3_kernel: the depth-wise 3 x 3 positional encoding of the cross-shaped
// windows, token-major, taps masked at the border of the token's stripe.
#include <type_traits>
#include "device_common.h"
#include "kernels.h"

namespace sm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

typedef unsigned int au32x4 __attribute__((ext_vector_type(4)));
#define SM_GPTR_(p) ((const __attribute__((address_space(1))) void*)(p))
#define SM_LPTR_(p) ((__attribute__((address_space(3))) void*)(p))

struct WinGeom { int w, shift, H, W, nWx, nW, wy, wx; };

__device__ __forceinline__ int region(int c, int extent, int w, int s) { return c < extent - w ? 0 : (c < extent - s ? 1 : 2); }

// additive term for (query i, key j) of window `win` and head `hh`
template <typename T>
__device__ __forceinline__ float window_term(const WinGeom& g, const T* table, int heads, int hh, int win, int i, int j) {
  // token index -> (row, column) inside the window; exact for the small integers involved
  const float inv_w = 1.0f / (float)g.w;
  const int yi = (int)(((float)i + 0.5f) * inv_w), xi = i - yi * g.w;
  const int yj = (int)(((float)j + 0.5f) * inv_w), xj = j - yj * g.w;
  float t = Elem<T>::ld(table + ((yi - yj + g.w - 1) * (2 * g.w - 1) + (xi - xj + g.w - 1)) * heads + hh);
  if (g.shift > 0) {
    const int wy = g.wy, wx = g.wx;
    const int ri = 3 * region(wy * g.w + yi, g.H, g.w, g.shift) + region(wx * g.w + xi, g.W, g.w, g.shift);
    const int rj = 3 * region(wy * g.w + yj, g.H, g.w, g.shift) + region(wx * g.w + xj, g.W, g.w, g.shift);
    if (ri != rj) t += -100.f;
  }
  return t;
}

template <int DK, int DB, int KIND>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(sm_attention_desc a, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                        const bf16_t* __restrict__ v, bf16_t* __restrict__ o,
                                                        const bf16_t* __restrict__ table, int n_qblk, long total_waves) {
  const int lane = threadIdx.x & 63, l32 = lane & 31, hf = lane >> 5;
  const long wid = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wid >= total_waves) return;
  // query block fastest, then head, then batch: the waves of one workgroup share K and V
  const int qb = (int)(wid % n_qblk);
  const long bh = wid / n_qblk;
  const int hh = (int)(bh % a.heads);
  const int b = (int)(bh / a.heads);
  const bf16_t* qp = q + (int64_t)b * a.q_stride[0] + (int64_t)hh * a.q_stride[1];
  const bf16_t* kp = k + (int64_t)b * a.k_stride[0] + (int64_t)hh * a.k_stride[1];
  const bf16_t* vp = v + (int64_t)b * a.v_stride[0] + (int64_t)hh * a.v_stride[1];
  bf16_t* op = o + (int64_t)b * a.o_stride[0] + (int64_t)hh * a.o_stride[1];
  const int q0 = qb * 32, qi = q0 + l32;
  const bool q_ok = qi < a.nq;
  WinGeom wg;
  int win = 0;
  if (KIND == SM_ATT_WINDOW) {
    wg.w = a.window; wg.shift = a.shift; wg.H = a.H; wg.W = a.W; wg.nWx = a.W / a.window; wg.nW = (a.H / a.window) * wg.nWx;
    win = b % wg.nW;
    wg.wy = win / wg.nWx; wg.wx = win - wg.wy * wg.nWx;
  }
  const uint4 zero = make_uint4(0, 0, 0, 0);
  uint4 qf[DK];
#pragma unroll
  for (int ks = 0; ks < DK; ++ks) {
    const int e = 16 * ks + 8 * hf;
    qf[ks] = (q_ok && e < a.d) ? *(const uint4*)(qp + (int64_t)qi * a.q_stride[2] + e) : zero;
  }
  f32x16_t oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  int n_kblk = (a.nk + 31) / 32;
  if (KIND == SM_ATT_CAUSAL) { const int lim = (min(q0 + 31, a.nq - 1)) / 32 + 1; n_kblk = min(n_kblk, lim); }
  if (KIND == SM_ATT_WINDOW) n_kblk = 2;            // a window has at most 64 tokens: both key blocks unrolled

#pragma unroll
  for (int jb = 0; jb < (KIND == SM_ATT_WINDOW ? 2 : n_kblk); ++jb) {
    const int j0 = jb * 32;
    f32x16_t s;
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
    {
      const int kj = j0 + l32;
      const bool k_ok = kj < a.nk;
#pragma unroll
      for (int ks = 0; ks < DK; ++ks) {
        const int e = 16 * ks + 8 * hf;
        const uint4 kf = (k_ok && e < a.d) ? *(const uint4*)(kp + (int64_t)kj * a.k_stride[2] + e) : zero;
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf), __builtin_bit_cast(bf16x8_t, qf[ks]), s, 0, 0, 0);
      }
    }
    float bm = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int j = j0 + (i >> 2) * 8 + hf * 4 + (i & 3);
      float x = s[i] * a.scale;
      if (KIND == SM_ATT_WINDOW && q_ok && j < a.nk) x += window_term<bf16_t>(wg, table, a.heads, hh, win, qi, j);
      if (j >= a.nk || (KIND == SM_ATT_CAUSAL && j > qi)) x = -INFINITY;
      s[i] = x;
      bm = fmaxf(bm, x);
    }
    bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
    const float m_new = fmaxf(m_run, bm);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __expf(m_run - m_use);        // m_run = -inf gives 0
    float rs = 0.f;
    unsigned pk[8];
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
      const float p0 = __expf(s[i] - m_use), p1 = __expf(s[i + 1] - m_use);
      const bf16_t h0 = f2bf(p0), h1 = f2bf(p1);
      rs += bf2f(h0) + bf2f(h1);                      // the sum of what the MFMA will actually use
      pk[i >> 1] = (unsigned)h0 | ((unsigned)h1 << 16);
    }
    rs += __shfl_xor(rs, 32, 64);
    l_run = l_run * alpha + rs;
    m_run = m_new;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
      const uint4 pf = make_uint4(pk[4 * ks2], pk[4 * ks2 + 1], pk[4 * ks2 + 2], pk[4 * ks2 + 3]);
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const int e = 32 * db + l32;
        unsigned vw[4];
#pragma unroll
        for (int t = 0; t < 8; t += 2) {
          const int ja = j0 + (2 * ks2 + (t >> 2)) * 8 + hf * 4 + (t & 3);
          const unsigned lo = (ja < a.nk && e < a.d) ? vp[(int64_t)ja * a.v_stride[2] + e] : 0;
          const unsigned hi = (ja + 1 < a.nk && e < a.d) ? vp[(int64_t)(ja + 1) * a.v_stride[2] + e] : 0;
          vw[t >> 1] = lo | (hi << 16);
        }
        const uint4 vf = make_uint4(vw[0], vw[1], vw[2], vw[3]);
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vf), __builtin_bit_cast(bf16x8_t, pf), oacc[db], 0, 0, 0);
      }
    }
  }
  if (!q_ok) return;
  const float inv = 1.f / l_run;
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const int e = 32 * db + g4 * 8 + hf * 4;
      if (e < a.d) {
        const unsigned w0 = (unsigned)f2bf(oacc[db][4 * g4] * inv) | ((unsigned)f2bf(oacc[db][4 * g4 + 1] * inv) << 16);
        const unsigned w1 = (unsigned)f2bf(oacc[db][4 * g4 + 2] * inv) | ((unsigned)f2bf(oacc[db][4 * g4 + 3] * inv) << 16);
        *(uint2*)(op + (int64_t)qi * a.o_stride[2] + e) = make_uint2(w0, w1);
      }
    }
}

// Global attention (full or causal), bf16: a workgroup of four waves owns 128 consecutive queries of one
// (batch, head), 32 per wave, and walks the keys in tiles of 64.  A K tile and a V tile go from global memory
// straight into LDS (16-byte LDS-DMA loads, two stages: tile t+1 is in flight while tile t is consumed), each
// read from HBM / L2 once per workgroup instead of once per wave.  Rows sit in LDS at a pitch of an odd number
// of 16-byte chunks, which spreads both access patterns over all banks: the K fragments (one row per lane,
// ds_read_b128) and the V^T fragments, which the transposing LDS read (ds_read_b64_tr_b16: within 16 lanes,
// lane i receives element i % 4 of the 8 bytes addressed by lanes i / 4 + 4 j, j = 0..3) delivers directly in
// the operand layout of the second MFMA.  The softmax runs in the exp2 domain with the scale folded into one
// FMA per score, masks are applied only in tiles that cross the diagonal or the end of the keys, and the
// running output is rescaled only when some row maximum of the wave actually moved.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));

// MODE 0: every key visible; 1: causal; 2: stripes (a batch entry is one stripe of an image's token grid: its tokens
// lie in runs of a.run adjacent tokens, so the stripe partition and merge of cross-shaped windows are two more
// strides in the row addresses).
// bid: the workgroup's index among those of this attention (one launch may hold two attentions, below).
template <int DK, int MODE>
__device__ __forceinline__ void attn_flash_body(const sm_attention_desc& a, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                const bf16_t* __restrict__ v, bf16_t* __restrict__ o, int n_qt, int nbh, int bid, int pair = 0) {
  constexpr bool CAUSAL = MODE == 1, STRIPE = MODE == 2;
  constexpr int DB = (DK + 1) / 2;           // 32-wide output column blocks
  // Row pitches in 16-byte chunks, chosen for the 64-bank LDS.  K rows are read whole-chunk by 16 consecutive rows
  // at a time (ds_read_b128): an odd pitch spreads them over all banks.  V rows are read by the transposing load,
  // four rows of 64 contiguous bytes at a time: those tile the 256 bytes of banks when the pitch is 64 or 192 bytes
  // modulo 256, i.e. 4 or 12 chunks modulo 16 (the odd pitch measured 59 % of the kernel's LDS cycles as conflicts).
  constexpr int P = 2 * DK + 1;
  constexpr int PV = DK <= 2 ? 4 : (DK == 3 ? 7 : (DK <= 6 ? 12 : 20));      // DK = 3 (rows of 5 or 6 chunks): the odd pitch, where
                                                                            // 12 would double the tile for rows half empty (measured slower)
  constexpr int TILE = 64 * P, TILEV = 64 * PV;      // chunks per K tile, per V tile
  constexpr int STG = TILE + TILEV;                  // chunks per stage
  extern __shared__ au32x4 fl_lds[];                 // [2 stages][K tile, V tile]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hf = lane >> 5;
  // (batch, head) fastest: the workgroups that share K and V follow each other at a distance of nbh, which
  // keeps them on one XCD (one L2) whenever nbh is a multiple of 8.  Causal: the first half of the ranks takes
  // the long query tiles in descending order and the second half the short ones in ascending order, so that
  // co-resident workgroups of ranks r and r + n_qt / 2 carry about the same total work.
  // pair: heads narrower than a cache line share their lines with the next head; pairs of heads, not heads, then go
  // round the XCDs (both heads of a pair and all their query tiles on one L2), which needs nbh / 2 to be a multiple of 8
  int bh = bid % nbh, rank = bid / nbh;
  if (pair) { const int half = nbh >> 1, t = bid / half; bh = 2 * (bid - t * half) + (t & 1); rank = t >> 1; }
  int qt = rank;
  if (CAUSAL) { const int hq = (n_qt + 1) >> 1; qt = rank < hq ? n_qt - 1 - rank : rank - hq; }
  // stripes: heads whose rows share cache lines (head size 32 is half a line) follow each other at a distance of
  // a.nb workgroups, which keeps them on one XCD's L2 whenever a.nb is a multiple of 8
  const int hh = STRIPE ? bh / a.nb : bh % a.heads;
  int b = STRIPE ? bh - hh * a.nb : bh / a.heads;
  const bf16_t *qp = q, *kp = k, *vp = v;
  bf16_t* op = o;
  if (STRIPE) {
    const int img = b / a.stripes, j = b - img * a.stripes;
    qp += (int64_t)j * a.q_stripe[0]; kp += (int64_t)j * a.k_stripe[0]; vp += (int64_t)j * a.v_stripe[0]; op += (int64_t)j * a.o_stripe[0];
    b = img;
  }
  qp += (int64_t)b * a.q_stride[0] + (int64_t)hh * a.q_stride[1];
  kp += (int64_t)b * a.k_stride[0] + (int64_t)hh * a.k_stride[1];
  vp += (int64_t)b * a.v_stride[0] + (int64_t)hh * a.v_stride[1];
  op += (int64_t)b * a.o_stride[0] + (int64_t)hh * a.o_stride[1];
  // element offset of token s_ of the sequence
  auto row_off = [&](int s_, int64_t tok_stride, int64_t run_stride) -> int64_t {
    if (!STRIPE) return (int64_t)s_ * tok_stride;
    const int so = s_ / a.run;
    return (int64_t)so * run_stride + (int64_t)(s_ - so * a.run) * tok_stride;
  };
  const int Q0 = qt * 128, q0 = Q0 + wave * 32, qi = q0 + l32;
  const int chv = a.d >> 3;                  // valid chunks per row

  // loader: wave-load i covers chunks [64 i, 64 i + 64) of a tile; wave w issues loads w, w + 4, ...
  constexpr int NLW = (P + 3) / 4, NLV = (PV + 3) / 4;
  int ld_row[NLW], ld_col[NLW], lv_row[NLV], lv_col[NLV];
#pragma unroll
  for (int i = 0; i < NLW; ++i) {
    const int s = (wave + 4 * i) * 64 + lane;
    ld_row[i] = s / P;
    ld_col[i] = min(s - ld_row[i] * P, chv - 1) * 8;      // pad chunks repeat the last valid one (finite data)
  }
#pragma unroll
  for (int i = 0; i < NLV; ++i) {
    const int s = (wave + 4 * i) * 64 + lane;
    lv_row[i] = s / PV;
    lv_col[i] = (s - lv_row[i] * PV) * 8;                 // slots past the head size are not loaded: what the V^T reads
  }                                                       // find there only reaches output rows that are never stored
  auto issue = [&](int kt) {
    au32x4* st = fl_lds + (kt & 1) * STG;
#pragma unroll
    for (int i = 0; i < NLW; ++i) {
      if (wave + 4 * i < P) {                // wave-uniform
        const int key = min(kt * 64 + ld_row[i], a.nk - 1);        // rows past the end repeat the last key (masked below)
        __builtin_amdgcn_global_load_lds(SM_GPTR_(kp + row_off(key, a.k_stride[2], a.k_stripe[1]) + ld_col[i]), SM_LPTR_(st + (wave + 4 * i) * 64), 16, 0, 0);
      }
    }
#pragma unroll
    for (int i = 0; i < NLV; ++i) {
      if (wave + 4 * i < PV && lv_col[i] < a.d) {
        const int key = min(kt * 64 + lv_row[i], a.nk - 1);
        __builtin_amdgcn_global_load_lds(SM_GPTR_(vp + row_off(key, a.v_stride[2], a.v_stripe[1]) + lv_col[i]), SM_LPTR_(st + TILE + (wave + 4 * i) * 64), 16, 0, 0);
      }
    }
  };

  int n_kt = (a.nk + 63) >> 6;
  if (CAUSAL) n_kt = min(n_kt, (min(Q0 + 127, a.nq - 1) >> 6) + 1);
  issue(0);

  const au32x4 zero = {0u, 0u, 0u, 0u};
  au32x4 qf[DK];
  {
    const bf16_t* qrow = qp + row_off(min(qi, a.nq - 1), a.q_stride[2], a.q_stripe[1]);
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) {
      const int e = 16 * ks + 8 * hf;
      qf[ks] = *(const au32x4*)(qrow + min(e, a.d - 8));
      if (e >= a.d) qf[ks] = zero;           // zero columns past the head size: they cancel the K tile's pad chunks
    }
  }
  f32x16_t oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;      // l_run: this lane's half of the row sum
  const float sc = a.scale * 1.4426950408889634f;
  // per-lane LDS offsets (bytes): K fragment row l32, chunk hf; V^T fragment rows 4 hf + j, columns 16 eb + 4 aa
  const unsigned k_lane = (unsigned)(l32 * P + hf) * 16u;
  const unsigned v_lane = (unsigned)((4 * hf + ((lane & 15) >> 2)) * PV * 16 + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2);

  for (int kt = 0; kt < n_kt; ++kt) {
    __builtin_amdgcn_s_waitcnt(0x0f70);      // vmcnt(0): this wave's part of tile kt is in LDS
    __builtin_amdgcn_s_barrier();            // ... and everybody's; the other stage is no longer read
    if (kt + 1 < n_kt) issue(kt + 1);
    const int j0 = kt * 64;
    if (CAUSAL && j0 > q0 + 31) continue;    // wave-uniform: every key of the tile lies after every query of the wave
    const char* kt_l = (const char*)(fl_lds + (kt & 1) * STG);
    const char* vt_l = kt_l + TILE * 16;
    f32x16_t s[2];
#pragma unroll
    for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) s[jb][i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < DK; ++ks) {
        const au32x4 kf = *(const au32x4*)(kt_l + k_lane + (32 * jb * P + 2 * ks) * 16);
        s[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf), __builtin_bit_cast(bf16x8_t, qf[ks]), s[jb], 0, 0, 0);
      }
    }
    const bool masked = (CAUSAL && j0 + 63 > q0) || j0 + 64 > a.nk;      // wave-uniform
    float bm = -INFINITY;
    if (masked) {
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int j = j0 + 32 * jb + (i >> 2) * 8 + hf * 4 + (i & 3);
          if (j >= a.nk || (CAUSAL && j > qi)) s[jb][i] = -INFINITY;
          bm = fmaxf(bm, s[jb][i]);
        }
    } else {
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int i = 0; i < 16; ++i) bm = fmaxf(bm, s[jb][i]);
    }
    bm = fmaxf(bm, __shfl_xor(bm, 32, 64)) * sc;        // sc > 0: scaling commutes with the maximum
    const float m_new = fmaxf(m_run, bm);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);          // m_run = -inf gives 0
    const bool moved = m_new != m_run;
    m_run = m_new;
    float rs = 0.f;
    au32x4 pf[2][2];
#pragma unroll
    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[jb][i], sc, -m_use)), p1 = __builtin_amdgcn_exp2f(fmaf(s[jb][i + 1], sc, -m_use));
        rs += p0 + p1;
        const f32x2_t pp = {p0, p1};
        pf[jb][i >> 3][(i >> 1) & 3] = __builtin_bit_cast(unsigned, __builtin_convertvector(pp, bf16x2_t));
      }
    l_run = l_run * alpha + rs;
    if (__builtin_amdgcn_ballot_w64(moved) != 0) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
    }
#pragma unroll
    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const char* base = vt_l + v_lane + ((32 * jb + 16 * ks2) * PV * 16 + 64 * db);
          const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(base));
          const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(base + 8 * PV * 16));
          const s16x8_t vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vf), __builtin_bit_cast(bf16x8_t, pf[jb][ks2]), oacc[db], 0, 0, 0);
        }
  }
  if (qi >= a.nq) return;
  l_run += __shfl_xor(l_run, 32, 64);
  const float inv = 1.f / l_run;
  bf16_t* orow = op + row_off(qi, a.o_stride[2], a.o_stripe[1]);
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const int e = 32 * db + g4 * 8 + hf * 4;
      if (e < a.d) {
        f32x2_t x0 = {oacc[db][4 * g4] * inv, oacc[db][4 * g4 + 1] * inv}, x1 = {oacc[db][4 * g4 + 2] * inv, oacc[db][4 * g4 + 3] * inv};
        if (a.accumulate) {                   // O += result: what is there is an addend in the output's own layout
          const uint2 old = *(const uint2*)(orow + e);
          x0[0] += __uint_as_float(old.x << 16); x0[1] += __uint_as_float(old.x & 0xffff0000u);
          x1[0] += __uint_as_float(old.y << 16); x1[1] += __uint_as_float(old.y & 0xffff0000u);
        }
        *(uint2*)(orow + e) = make_uint2(__builtin_bit_cast(unsigned, __builtin_convertvector(x0, bf16x2_t)),
                                                                    __builtin_bit_cast(unsigned, __builtin_convertvector(x1, bf16x2_t)));
      }
    }
}

template <int DK, int MODE>
__global__ __launch_bounds__(256, 2) void attn_flash_kernel(sm_attention_desc a, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                            const bf16_t* __restrict__ v, bf16_t* __restrict__ o, int n_qt, int nbh, int pair) {
  attn_flash_body<DK, MODE>(a, q, k, v, o, n_qt, nbh, (int)blockIdx.x, pair);
}
// Two stripe attentions of one shape in one launch (the two halves of a cross-shaped window attention): workgroups
// [0, g0) belong to the first.  Each half has its own strides and pointers; nothing else differs.
struct FlashPairPtrs { const bf16_t *q, *k, *v; bf16_t* o; };
__global__ __launch_bounds__(256, 2) void attn_stripe_pair_kernel(sm_attention_desc a0, sm_attention_desc a1, FlashPairPtrs p0, FlashPairPtrs p1,
                                                                  int n_qt, int nbh, int g0) {
  if ((int)blockIdx.x < g0) attn_flash_body<2, 2>(a0, p0.q, p0.k, p0.v, p0.o, n_qt, nbh, (int)blockIdx.x);
  else attn_flash_body<2, 2>(a1, p1.q, p1.k, p1.v, p1.o, n_qt, nbh, (int)blockIdx.x - g0);
}

// Window attention, bf16, head size 32, at most 64 tokens per window: one wave per (window, head, block of 32
// queries); the four waves of a workgroup are the two query blocks of two adjacent heads of one window, so that
// their Q / K / V rows are adjacent in memory and the second reader of K and V hits the vector cache.  Short
// dependency chains matter more than total work here (a window is 49 tokens: the kernel is latency-bound), hence
// the split by query block.  Everything a wave needs is requested up front (Q and K fragments, V rows, its head's
// column of the relative-position table); V and the table go through wave-private LDS, from where the transposed
// V fragments and the bias values are read; the bias index is a difference of a per-query and a per-key term, the
// shift mask a comparison of two region ids, both prepared once per wave.  The softmax works on base-2 logits:
// scale and table are multiplied by log2 e on the way in.
// BOTH: one wave per (window, head) that works through both query blocks in turn (K, V, the table column and the
// per-key terms fetched once): half as many waves with a longer chain each, for grids of several rounds of residency,
// where the rounds, not the chain, set the time.
template <bool BOTH>
__global__ __launch_bounds__(256, 2) void attn_window32_kernel(sm_attention_desc a, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                            const bf16_t* __restrict__ v, bf16_t* __restrict__ o,
                                                            const bf16_t* __restrict__ table, long total_waves) {
  __shared__ bf16_t v_lds[4][64 * 32];
  __shared__ float t_lds[4][256];
  __shared__ int k_lds[4][64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, l32 = lane & 31, hf = lane >> 5;
  const unsigned wid = blockIdx.x * 4u + wave;       // < 2^31: checked by the launcher
  if ((long)wid >= total_waves) return;              // whole waves leave; no workgroup barrier is used below
  const int qb0 = BOTH ? 0 : (int)(wid & 1u);
  const unsigned pair = BOTH ? wid : wid >> 1;
  const int b = (int)(pair / (unsigned)a.heads);
  const int hh = (int)(pair - (unsigned)b * (unsigned)a.heads);
  const int w = a.window, n = a.nq, tw = 2 * w - 1;
  if (32 * qb0 >= n) return;                         // a window of at most 32 tokens has no second query block
  const bf16_t* qp = q + (int64_t)b * a.q_stride[0] + (int64_t)hh * a.q_stride[1];
  const bf16_t* kp = k + (int64_t)b * a.k_stride[0] + (int64_t)hh * a.k_stride[1];
  const bf16_t* vp = v + (int64_t)b * a.v_stride[0] + (int64_t)hh * a.v_stride[1];
  bf16_t* op = o + (int64_t)b * a.o_stride[0] + (int64_t)hh * a.o_stride[1];
  const au32x4 zero = {0u, 0u, 0u, 0u};
  constexpr float LOG2E = 1.4426950408889634f;
  // ---- all global loads first
  constexpr int NQB = BOTH ? 2 : 1;
  au32x4 qfa[NQB][2], kf[2][2], vrow[4];
  unsigned short tv[4];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int e = 16 * ks + 8 * hf;
#pragma unroll
    for (int qq = 0; qq < NQB; ++qq)
      qfa[qq][ks] = *(const au32x4*)(qp + (int64_t)min(32 * (qb0 + qq) + l32, n - 1) * a.q_stride[2] + e);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int j = 32 * kb + l32;
      kf[kb][ks] = *(const au32x4*)(kp + (int64_t)min(j, n - 1) * a.k_stride[2] + e);
      if (j >= n) kf[kb][ks] = zero;
    }
  }
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int c = lane + 64 * t, row = c >> 2, part = c & 3;
    vrow[t] = *(const au32x4*)(vp + (int64_t)min(row, n - 1) * a.v_stride[2] + part * 8);
    if (row >= n) vrow[t] = zero;                    // padded keys must contribute exact zeros
    const int ti = lane + 64 * t;
    tv[t] = ti < tw * tw ? table[ti * a.heads + hh] : (unsigned short)0;
  }
  // ---- per-wave LDS: V rows, table column as base-2 floats, per-key (bias term | region << 16)
  const int nWx = a.W / w, nW = (a.H / w) * nWx, win = b % nW, wy = win / nWx, wx = win - wy * nWx;
  const float inv_w = 1.0f / (float)w;
  {
    const int j = lane;
    const int yj = (int)(((float)j + 0.5f) * inv_w), xj = j - yj * w;
    int info = yj * tw + xj;
    if (a.shift > 0) info |= (3 * region(wy * w + yj, a.H, w, a.shift) + region(wx * w + xj, a.W, w, a.shift)) << 16;
    k_lds[wave][j] = info;
  }
  __builtin_amdgcn_sched_barrier(0);                 // the index terms above are computed while the loads are in flight
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int c = lane + 64 * t;
    *(au32x4*)(&v_lds[wave][c * 8]) = vrow[t];
    t_lds[wave][lane + 64 * t] = bf2f(tv[t]) * LOG2E;
  }
  __builtin_amdgcn_s_waitcnt(0xc07f);                // lgkmcnt(0): this wave's LDS writes are done (wave-private data)
  const float sc2 = a.scale * LOG2E;
  const bool shifted = a.shift > 0;                  // wave-uniform
#pragma unroll
  for (int qq = 0; qq < NQB; ++qq) {
  const int qb = qb0 + qq;
  if (32 * qb >= n) break;
  const int qi = 32 * qb + l32;                      // this lane's query
  const au32x4* qf = qfa[qq];
  // per-query terms
  const int yi = (int)(((float)qi + 0.5f) * inv_w), xi = qi - yi * w;
  const int qa = yi * tw + xi + (w - 1) * 2 * w;
  const int rq = a.shift > 0 ? 3 * region(wy * w + yi, a.H, w, a.shift) + region(wx * w + xi, a.W, w, a.shift) : 0;
  // ---- S^T[kb] = K_kb Q^T
  f32x16_t s[2];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
      s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf[kb][ks]), __builtin_bit_cast(bf16x8_t, qf[ks]), s[kb], 0, 0, 0);
  }
  // ---- bias, mask, softmax for this lane's query (keys: 16 per block in this lane, the other 16 in lane ^ 32)
  float mx = -INFINITY;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int j = 32 * kb + (i >> 2) * 8 + hf * 4 + (i & 3);
      const int info = k_lds[wave][j];
      float x = fmaf(s[kb][i], sc2, t_lds[wave][(qa - (info & 0xffff)) & 255]);
      if (shifted && rq != (info >> 16)) x += -100.f * LOG2E;
      if (j >= n) x = -INFINITY;
      s[kb][i] = x;
      mx = fmaxf(mx, x);
    }
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  au32x4 pf[2][2];
  float sum = 0.f;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
      const float p0 = __builtin_amdgcn_exp2f(s[kb][i] - mx), p1 = __builtin_amdgcn_exp2f(s[kb][i + 1] - mx);
      const f32x2_t pp = {p0, p1};
      const bf16x2_t ph = __builtin_convertvector(pp, bf16x2_t);
      const unsigned pw = __builtin_bit_cast(unsigned, ph);
      sum += __uint_as_float(pw << 16) + __uint_as_float(pw & 0xffff0000u);      // the sum of what the MFMA will actually use
      pf[kb][i >> 3][(i >> 1) & 3] = pw;
    }
  sum += __shfl_xor(sum, 32, 64);
  const float inv = 1.f / sum;
  // ---- O^T = V^T P^T
  f32x16_t oacc;
#pragma unroll
  for (int i = 0; i < 16; ++i) oacc[i] = 0.f;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
      au32x4 vf;
#pragma unroll
      for (int t = 0; t < 8; t += 2) {
        const int ja = 32 * kb + (2 * ks2 + (t >> 2)) * 8 + hf * 4 + (t & 3);
        const unsigned lo = v_lds[wave][ja * 32 + l32], hi = v_lds[wave][(ja + 1) * 32 + l32];
        vf[t >> 1] = lo | (hi << 16);
      }
      oacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vf), __builtin_bit_cast(bf16x8_t, pf[kb][ks2]), oacc, 0, 0, 0);
    }
  if (qi < n) {
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const int e = g4 * 8 + hf * 4;
      const f32x2_t x0 = {oacc[4 * g4] * inv, oacc[4 * g4 + 1] * inv}, x1 = {oacc[4 * g4 + 2] * inv, oacc[4 * g4 + 3] * inv};
      *(uint2*)(op + (int64_t)qi * a.o_stride[2] + e) = make_uint2(__builtin_bit_cast(unsigned, __builtin_convertvector(x0, bf16x2_t)),
                                                                  __builtin_bit_cast(unsigned, __builtin_convertvector(x1, bf16x2_t)));
    }
  }
  }
}

// Windows of 7 x 7 tokens, head size 32 (every Swin configuration).  Two things bound the general window kernel
// above at these sizes, neither of them HBM: the texture path (its loads and stores put the rows of a head slice in
// adjacent lanes, four cache lines per lane quad) and the vector ALU (index arithmetic per score).  This variant
//   * moves Q, K, V and O between global memory and LDS in 16-byte pieces with the four pieces of a row's 64-byte
//     head slice in adjacent lanes, and reads the MFMA fragments from LDS (rows at a pitch of 80 bytes);
//   * deals the keys to the MFMA rows so that the half-wave hf owns the window rows y with y & 1 == hf, in "slot"
//     order s = (y >> 1) * 7 + x (28 slots per half, 4 of them padding in the even half, 11 in the odd one): a
//     lane's 16 scores of key block kb are slots 16 kb .. 16 kb + 15 of its own half.  Then the relative-position
//     index of (query, slot) is a per-lane base minus a compile-time constant, i.e. one LDS read with an immediate
//     offset from the head's table column (pre-multiplied by log2 e); padding is known at compile time (slots >=
//     28) or per half-wave (odd half, slots 21 .. 27); the shifted-window mask is a 64-bit "same region" set per
//     query (two ballots over the keys), tested at constant bit positions, and only in the windows of the last row
//     or column, the only ones whose tokens lie in more than one region;
//   * keeps V transposed in LDS ([half][channel][slot]), so that a V^T fragment is one 16-byte read, shared by
//     both query blocks.
// All LDS data is private to its wave (the LDS queue keeps a wave's accesses in order): no workgroup barrier.
template <bool BOTH>
__global__ __launch_bounds__(256, 4) void attn_window7_kernel(sm_attention_desc a, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                           const bf16_t* __restrict__ v, bf16_t* __restrict__ o,
                                                           const bf16_t* __restrict__ table, long total_waves) {
  constexpr int RP = 80;                             // bytes per staged row: 64 + 16 keeps 16-byte reads of adjacent rows on distinct banks
  constexpr int PITCH = 40;                          // slots per channel row of V^T: 32 + 8, keeps the 16-byte reads aligned
  constexpr int TPAD = 16, TLEN = 208;               // the table column sits at [TPAD, TPAD + 169); padded slots read around it
  // per wave: Q rows [0, 3920) and K rows [K_OFF, K_OFF + 3920) first, then V^T in [0, 5120), then the O rows in [0, 5120)
  constexpr int K_OFF = 3968, T_OFF = 7936, WAVE_BYTES = T_OFF + TLEN * 4;
  __shared__ __attribute__((aligned(16))) unsigned char lds_all[4 * WAVE_BYTES];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, l32 = lane & 31, hf = lane >> 5;      // wave: scalar
  const unsigned wid = blockIdx.x * 4u + wave;       // < 2^31: checked by the launcher
  if ((long)wid >= total_waves) return;              // whole waves leave
  const int qb0 = BOTH ? 0 : (int)(wid & 1u);
  const unsigned pair = BOTH ? wid : wid >> 1;
  const int b = (int)(pair / (unsigned)a.heads);
  const int hh = (int)(pair - (unsigned)b * (unsigned)a.heads);
  const bf16_t* qp = q + (int64_t)b * a.q_stride[0] + (int64_t)hh * a.q_stride[1];
  const bf16_t* kp = k + (int64_t)b * a.k_stride[0] + (int64_t)hh * a.k_stride[1];
  const bf16_t* vp = v + (int64_t)b * a.v_stride[0] + (int64_t)hh * a.v_stride[1];
  bf16_t* op = o + (int64_t)b * a.o_stride[0] + (int64_t)hh * a.o_stride[1];
  const int qs = (int)a.q_stride[2], ksd = (int)a.k_stride[2], vs = (int)a.v_stride[2], os = (int)a.o_stride[2];      // < 2^24: checked by the launcher
  const au32x4 zero = {0u, 0u, 0u, 0u};
  constexpr float LOG2E = 1.4426950408889634f;
  constexpr int NQB = BOTH ? 2 : 1, QP = BOTH ? 4 : 2;      // query blocks of this wave; 64-lane rounds of 16-byte pieces that cover its query rows
  unsigned char* L = lds_all + wave * WAVE_BYTES;
  // ---- all global loads first: piece c = lane + 64 t is channels 8 (c & 3) .. of row c >> 2 (196 pieces per tensor)
  au32x4 qv[QP], kv[4], vv[4];
  unsigned short tv[3];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int c = lane + 64 * t, row = min(c >> 2, 48), part = c & 3;
    kv[t] = *(const au32x4*)(kp + (row * ksd + part * 8));
    vv[t] = *(const au32x4*)(vp + (row * vs + part * 8));
    if (t < QP) qv[t] = *(const au32x4*)(qp + (min(32 * qb0 + (c >> 2), 48) * qs + part * 8));
  }
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    const int ti = lane + 64 * t;
    tv[t] = ti < 169 ? table[ti * a.heads + hh] : (unsigned short)0;
  }
  // ---- index terms while the loads are in flight.  (n * 37) >> 8 == n / 7 for 0 <= n < 56.
  int krow[2];
  bool kok[2];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {                   // the key whose K row is MFMA row l32 of block kb
    const int s = 16 * kb + (l32 >> 3) * 4 + (l32 & 3), hk = (l32 >> 2) & 1;
    const int g = (s * 37) >> 8, y = 2 * g + hk;
    kok[kb] = s < 28 && y < 7;
    krow[kb] = kok[kb] ? y * 7 + (s - 7 * g) : 0;
  }
  int vdst[4];                                       // element index in V^T of this lane's piece t, channel part * 8
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int c = lane + 64 * t;                     // the 196 real pieces, then the 60 pieces of the 15 padded slots
    const bool real = c < 196;
    const int row = c >> 2, part = c & 3;
    const int y = (row * 37) >> 8, x = row - 7 * y;
    const int zs = (c - 196) >> 2;
    const int hk = real ? (y & 1) : (zs < 4 ? 0 : 1);
    const int s = real ? (y >> 1) * 7 + x : (zs < 4 ? 28 + zs : 17 + zs);
    vdst[t] = (hk * 32 + part * 8) * PITCH + s;
  }
  const int nWx = a.W / 7, nWy = a.H / 7, nW = nWy * nWx, win = b % nW, wy = win / nWx, wx = win - wy * nWx;
  const bool edge = a.shift > 0 && (wy == nWy - 1 || wx == nWx - 1);      // wave-uniform: elsewhere all tokens share region 0
  unsigned long long my = ~0ull, mxm = ~0ull;
  int ry0 = 0, rx0 = 0;
  if (edge) {
    const int j = min(lane, 48), yj = (j * 37) >> 8, xj = j - 7 * yj;
    ry0 = region(wy * 7, a.H, 7, a.shift); rx0 = region(wx * 7, a.W, 7, a.shift);
    my = __ballot(region(wy * 7 + yj, a.H, 7, a.shift) == ry0);
    mxm = __ballot(region(wx * 7 + xj, a.W, 7, a.shift) == rx0);
  }
  __builtin_amdgcn_sched_barrier(0);
  // ---- Q and K rows and the table column into LDS, the MFMA fragments out of it
  float* tw = (float*)(L + T_OFF);
  if (lane < TPAD) tw[lane] = 0.f;
#pragma unroll
  for (int t = 0; t < 3; ++t) tw[TPAD + lane + 64 * t] = bf2f(tv[t]) * LOG2E;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int c = lane + 64 * t, off = (c >> 2) * RP + (c & 3) * 16;
    if (c < 196) {
      *(au32x4*)(L + K_OFF + off) = kv[t];
      if (t < QP) *(au32x4*)(L + off) = qv[t];         // rows past the window's last repeat it (never stored)
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  au32x4 qfa[NQB][2], kf[2][2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
    for (int qq = 0; qq < NQB; ++qq) qfa[qq][ks] = *(const au32x4*)(L + min(32 * qq + l32, BOTH ? 48 : 31) * RP + (2 * ks + hf) * 16);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      kf[kb][ks] = *(const au32x4*)(L + K_OFF + krow[kb] * RP + (2 * ks + hf) * 16);
      if (!kok[kb]) kf[kb][ks] = zero;
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  // ---- V transposed over the Q / K rows, its fragments out
  bf16_t* vt = (bf16_t*)L;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    if (lane + 64 * t >= 196) vv[t] = zero;          // padded keys must contribute exact zeros
#pragma unroll
    for (int u = 0; u < 8; ++u) vt[vdst[t] + u * PITCH] = (bf16_t)(vv[t][u >> 1] >> (16 * (u & 1)));
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  au32x4 vf[2][2];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) vf[kb][ks2] = *(const au32x4*)(vt + (hf * 32 + l32) * PITCH + 16 * kb + 8 * ks2);
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const float sc2 = a.scale * LOG2E;
  auto queries = [&](auto edge_c) {
  constexpr bool EDGE = decltype(edge_c)::value;
#pragma unroll
  for (int qq = 0; qq < NQB; ++qq) {
    const int qi = 32 * (qb0 + qq) + l32;            // this lane's query
    const int qc = min(qi, 48), yi = (qc * 37) >> 8, xi = qc - 7 * yi;
    const float* tq = tw + (yi * 13 + xi + TPAD - 13 * hf);      // + 84 - (26 g + x) per slot, all >= 0
    // ---- S^T[kb] = K_kb Q^T
    f32x16_t s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf[kb][ks]), __builtin_bit_cast(bf16x8_t, qfa[qq][ks]), s[kb], 0, 0, 0);
    }
    // ---- bias, mask, softmax for this lane's query (28 slots here, the other half's 28 in lane ^ 32)
    unsigned same_lo = ~0u, same_hi = ~0u;
    if (EDGE) {
      const bool ysame = region(wy * 7 + yi, a.H, 7, a.shift) == ry0, xsame = region(wx * 7 + xi, a.W, 7, a.shift) == rx0;
      const unsigned long long same = ((ysame ? my : ~my) & (xsame ? mxm : ~mxm)) >> (7 * hf);
      same_lo = (unsigned)same; same_hi = (unsigned)(same >> 32);
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int sl = 16 * kb + i;
        if (sl >= 28) continue;
        const int g = sl / 7, x7 = sl - 7 * g;
        float x = fmaf(s[kb][i], sc2, tq[84 - (26 * g + x7)]);
        if (EDGE) {
          const int bit = 14 * g + x7;               // the key's natural index, less 7 hf
          const unsigned wd = bit < 32 ? same_lo : same_hi;
          if (!((wd >> (bit & 31)) & 1u)) x += -100.f * LOG2E;
        }
        if (g == 3 && hf) x = -INFINITY;             // window row 7 does not exist
        s[kb][i] = x;
        mx = fmaxf(mx, x);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    au32x4 pf[2][2];
    float sum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        unsigned pw = 0u;
        if (16 * kb + i < 28) {
          const float p0 = __builtin_amdgcn_exp2f(s[kb][i] - mx), p1 = __builtin_amdgcn_exp2f(s[kb][i + 1] - mx);
          const f32x2_t pp = {p0, p1};
          pw = __builtin_bit_cast(unsigned, __builtin_convertvector(pp, bf16x2_t));
          sum += p0 + p1;
        }
        pf[kb][i >> 3][(i >> 1) & 3] = pw;
      }
    sum += __shfl_xor(sum, 32, 64);
    const float inv = 1.f / sum;
    // ---- O^T = V^T P^T, then this lane's 4 x 4 channels of its query's row into the LDS copy of O
    f32x16_t oacc;
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[i] = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2)
        oacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vf[kb][ks2]), __builtin_bit_cast(bf16x8_t, pf[kb][ks2]), oacc, 0, 0, 0);
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const f32x2_t x0 = {oacc[4 * g4] * inv, oacc[4 * g4 + 1] * inv}, x1 = {oacc[4 * g4 + 2] * inv, oacc[4 * g4 + 3] * inv};
      *(uint2*)(L + (32 * qq + l32) * RP + g4 * 16 + hf * 8) = make_uint2(__builtin_bit_cast(unsigned, __builtin_convertvector(x0, bf16x2_t)),
                                                                          __builtin_bit_cast(unsigned, __builtin_convertvector(x1, bf16x2_t)));
    }
  }
  };
  if (edge) queries(std::true_type{}); else queries(std::false_type{});      // a scalar branch: edge is wave-uniform
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  // ---- O rows out, 64 contiguous bytes per lane quad
#pragma unroll
  for (int t = 0; t < QP; ++t) {
    const int c = lane + 64 * t, row = 32 * qb0 + (c >> 2);
    if (row < 49) *(au32x4*)(op + (row * os + (c & 3) * 8)) = *(const au32x4*)(L + (c >> 2) * RP + (c & 3) * 16);
  }
}

// fp32 window attention: nq, nk <= 64, d <= 4 DV.  One workgroup of 256 threads per (window, head); the four lanes of
// a quad own query i = tid / 4 and a quarter of the head's features each: a score is four partial dot products added
// across the quad, the product with V is taken per quarter.  K and V rows sit in LDS as 16-byte chunks (all quads read
// the same chunks at the same time: a broadcast), the head's column of the relative-position table as well; the
// scores of a query stay in its own LDS column between the two passes (maximum, then exponentials and the product
// with V in one sweep over the keys).
template <int DV>
__global__ __launch_bounds__(256) void attn_window_f32_kernel(sm_attention_desc a, const float* __restrict__ q, const float* __restrict__ k,
                                                              const float* __restrict__ v, float* __restrict__ o, const float* __restrict__ table) {
  constexpr int P = DV + 1;                  // row pitch in chunks, odd: the staging stores spread over the banks
  constexpr int CPL = DV / 4;                // chunks per lane
  __shared__ float4 ks[64 * P], vs[64 * P];
  __shared__ float ss[64 * 65];
  __shared__ float bias_s[232];              // (2 w - 1)^2 <= 225 entries (w <= 8)
  const int b = blockIdx.x / a.heads, hh = blockIdx.x % a.heads;
  const float* qp = q + (int64_t)b * a.q_stride[0] + (int64_t)hh * a.q_stride[1];
  const float* kp = k + (int64_t)b * a.k_stride[0] + (int64_t)hh * a.k_stride[1];
  const float* vp = v + (int64_t)b * a.v_stride[0] + (int64_t)hh * a.v_stride[1];
  float* op = o + (int64_t)b * a.o_stride[0] + (int64_t)hh * a.o_stride[1];
  const int tid = threadIdx.x, dv = a.d >> 2;
  const float4 zero4 = {0.f, 0.f, 0.f, 0.f};
  for (int idx = tid; idx < a.nk * DV; idx += 256) {
    const int j = idx / DV, c = idx - j * DV;
    float4 kk = zero4, vv = zero4;          // chunks past the head size: zeros, so that the sums below can run to DV
    if (c < dv) {
      kk = *(const float4*)(kp + (int64_t)j * a.k_stride[2] + 4 * c);
      vv = *(const float4*)(vp + (int64_t)j * a.v_stride[2] + 4 * c);
    }
    ks[j * P + c] = kk; vs[j * P + c] = vv;
  }
  if (a.kind == SM_ATT_WINDOW) {
    const int nt = (2 * a.window - 1) * (2 * a.window - 1);
    for (int t = tid; t < nt; t += 256) bias_s[t] = table[(int64_t)t * a.heads + hh];
  }
  __syncthreads();
  WinGeom wg;
  wg.w = a.window; wg.shift = a.shift; wg.H = a.H; wg.W = a.W; wg.nWx = a.W / a.window; wg.nW = (a.H / a.window) * wg.nWx;
  const int win = b % wg.nW;
  wg.wy = win / wg.nWx; wg.wx = win - wg.wy * wg.nWx;
  const int i = tid >> 2, c0 = (tid & 3) * CPL;       // the quad's query, this lane's first chunk
  const int iq = min(i, a.nq - 1);                    // quads past the last query repeat it and store nothing
  float4 qr[CPL];
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    qr[c] = zero4;
    if (c0 + c < dv) {
      const float4 t = *(const float4*)(qp + (int64_t)iq * a.q_stride[2] + 4 * (c0 + c));
      qr[c].x = t.x * a.scale; qr[c].y = t.y * a.scale; qr[c].z = t.z * a.scale; qr[c].w = t.w * a.scale;
    }
  }
  float mx = -INFINITY;
  for (int j = 0; j < a.nk; ++j) {
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
      const float4 kk = ks[j * P + c0 + c];
      s = fmaf(qr[c].x, kk.x, s); s = fmaf(qr[c].y, kk.y, s); s = fmaf(qr[c].z, kk.z, s); s = fmaf(qr[c].w, kk.w, s);
    }
    s += __shfl_xor(s, 1, 64);
    s += __shfl_xor(s, 2, 64);              // the whole dot product, the same bits in the four lanes
    if (a.kind == SM_ATT_WINDOW) s += window_term<float>(wg, bias_s, 1, 0, win, iq, j);
    ss[i * 65 + j] = s;                      // four lanes, one value, one address
    mx = fmaxf(mx, s);
  }
  float sum = 0.f;
  float4 acc[CPL];
#pragma unroll
  for (int c = 0; c < CPL; ++c) acc[c] = zero4;
  for (int j = 0; j < a.nk; ++j) {
    const float p = expf(ss[i * 65 + j] - mx);
    sum += p;
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
      const float4 vv = vs[j * P + c0 + c];
      acc[c].x = fmaf(p, vv.x, acc[c].x); acc[c].y = fmaf(p, vv.y, acc[c].y); acc[c].z = fmaf(p, vv.z, acc[c].z); acc[c].w = fmaf(p, vv.w, acc[c].w);
    }
  }
  if (i >= a.nq) return;
  const float inv = 1.f / sum;
#pragma unroll
  for (int c = 0; c < CPL; ++c)
    if (c0 + c < dv) {
      const float4 r = {acc[c].x * inv, acc[c].y * inv, acc[c].z * inv, acc[c].w * inv};
      *(float4*)(op + (int64_t)i * a.o_stride[2] + 4 * (c0 + c)) = r;
    }
}

// Depth-wise 3 x 3 cross-correlation on a token-major grid: one thread per (token, 8 channels); the 72 weights of its
// channels are 144 contiguous bytes.  Memory-bound: every value is read once from HBM and eight more times from cache.
// Workgroups are dealt to the 8 XCDs round-robin: XCD x takes the x-th eighth of the tokens, so that the rows above
// and below a token are fetched into the same L2 as the token's own.
__global__ __launch_bounds__(256) void dwconv3x3_kernel(DwconvArgs a, int64_t total) {
  const int64_t block = (int64_t)(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);      // the grid is a multiple of 8
  const int64_t idx = block * 256 + threadIdx.x;
  if (idx >= total) return;
  const int cv = a.Cn >> 3;
  const int c = (int)(idx % cv) * 8;
  const int64_t t = idx / cv;
  const int hw = a.H * a.W;
  const int img = (int)(t / hw), p = (int)(t - (int64_t)img * hw);
  const int y = p / a.W, x = p - y * a.W;
  const bool second = a.split_c > 0 && c >= a.split_c;                // channels from split_c on: the other stripe shape
  const int Hs = second ? a.Hs2 : a.Hs, Ws = second ? a.Ws2 : a.Ws;
  const int y_lo = (y / Hs) * Hs, x_lo = (x / Ws) * Ws;               // the token's stripe
  const bf16_t* vb = (const bf16_t*)a.v + (int64_t)img * a.v_img + c;
  float wv[72];
  {
    const au32x4* wp = (const au32x4*)((const bf16_t*)a.w + (int64_t)c * 9);
#pragma unroll
    for (int i = 0; i < 9; ++i) {
      const au32x4 u = wp[i];
#pragma unroll
      for (int j = 0; j < 4; ++j) { wv[8 * i + 2 * j] = __uint_as_float(u[j] << 16); wv[8 * i + 2 * j + 1] = __uint_as_float(u[j] & 0xffff0000u); }
    }
  }
  float acc[8];
  {
    const au32x4 u = *(const au32x4*)((const bf16_t*)a.bias + c);
#pragma unroll
    for (int j = 0; j < 4; ++j) { acc[2 * j] = __uint_as_float(u[j] << 16); acc[2 * j + 1] = __uint_as_float(u[j] & 0xffff0000u); }
  }
#pragma unroll
  for (int dy = 0; dy < 3; ++dy)
#pragma unroll
    for (int dx = 0; dx < 3; ++dx) {
      const int yy = y + dy - 1, xx = x + dx - 1;
      if (yy < y_lo || yy >= y_lo + Hs || xx < x_lo || xx >= x_lo + Ws) continue;          // beyond the stripe: zero
      const au32x4 u = *(const au32x4*)(vb + (int64_t)(yy * a.W + xx) * a.v_tok);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        acc[2 * j] = fmaf(__uint_as_float(u[j] << 16), wv[(2 * j) * 9 + dy * 3 + dx], acc[2 * j]);
        acc[2 * j + 1] = fmaf(__uint_as_float(u[j] & 0xffff0000u), wv[(2 * j + 1) * 9 + dy * 3 + dx], acc[2 * j + 1]);
      }
    }
  au32x4 r;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const f32x2_t pr = {acc[2 * j], acc[2 * j + 1]};
    r[j] = __builtin_bit_cast(unsigned, __builtin_convertvector(pr, bf16x2_t));
  }
  *(au32x4*)((bf16_t*)a.out + (int64_t)img * a.o_img + (int64_t)p * a.o_tok + c) = r;
}
int launch_dwconv3x3(const DwconvArgs& a, void* stream) {
  const int64_t total = (int64_t)a.n_img * a.H * a.W * (a.Cn / 8);
  if (total == 0) return 0;
  const int64_t blocks = ((total + 255) / 256 + 7) / 8 * 8;
  dwconv3x3_kernel<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream>>>(a, total);
  return (int)hipGetLastError();
}

// both descriptors: SM_ATT_STRIPE, bf16, head size <= 32, positive scale, the same nb, heads, nq (checked by the caller)
int launch_attention_stripe_pair(const sm_attention_desc& d0, const void* const* p0, const sm_attention_desc& d1, const void* const* p1, void* stream) {
  const int n_qt = (d0.nq + 127) / 128, nbh = d0.nb * d0.heads;
  const long g0 = (long)n_qt * nbh;
  if (2 * g0 >= (1L << 31)) return (int)hipErrorInvalidValue;
  const size_t smem = 2 * 64 * ((2 * 2 + 1) + 4) * 16 + 64;
  static const hipError_t attr = hipFuncSetAttribute((const void*)attn_stripe_pair_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (attr != hipSuccess) return (int)attr;
  const FlashPairPtrs a{(const bf16_t*)p0[0], (const bf16_t*)p0[1], (const bf16_t*)p0[2], (bf16_t*)p0[3]};
  const FlashPairPtrs b{(const bf16_t*)p1[0], (const bf16_t*)p1[1], (const bf16_t*)p1[2], (bf16_t*)p1[3]};
  attn_stripe_pair_kernel<<<dim3((unsigned)(2 * g0)), dim3(256), smem, (hipStream_t)stream>>>(d0, d1, a, b, n_qt, nbh, (int)g0);
  return (int)hipGetLastError();
}

int launch_attention(const sm_attention_desc& d, const void* q, const void* k, const void* v, void* o,
                     const void* rpb_table, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  if (d.dtype == SM_F32) {
    if (d.d <= 32) attn_window_f32_kernel<8><<<dim3((unsigned)(d.nb * d.heads)), dim3(256), 0, s>>>(d, (const float*)q, (const float*)k, (const float*)v,
                                                                                                     (float*)o, (const float*)rpb_table);
    else attn_window_f32_kernel<16><<<dim3((unsigned)(d.nb * d.heads)), dim3(256), 0, s>>>(d, (const float*)q, (const float*)k, (const float*)v,
                                                                                          (float*)o, (const float*)rpb_table);
    return (int)hipGetLastError();
  }
  if (d.kind == SM_ATT_WINDOW && d.d == 32 && d.nq <= 64 && d.window <= 8) {
    long waves = 2L * d.nb * d.heads;                 // one per (window, head, query block)
    if (waves >= (1L << 31)) return (int)hipErrorInvalidValue;
    // 256 CUs hold 20 of these waves each: beyond one round of residency a wave takes both query blocks
    const int64_t smax = 1 << 24;
    if (d.window == 7 && d.nq == 49 && d.nk == 49 && d.q_stride[2] < smax && d.k_stride[2] < smax && d.v_stride[2] < smax && d.o_stride[2] < smax) {
      if (waves > 256L * 20) {
        waves /= 2;
        attn_window7_kernel<true><<<dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s>>>(d, (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v,
                                                                                         (bf16_t*)o, (const bf16_t*)rpb_table, waves);
      } else {
        attn_window7_kernel<false><<<dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s>>>(d, (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v,
                                                                                          (bf16_t*)o, (const bf16_t*)rpb_table, waves);
      }
      return (int)hipGetLastError();
    }
    if (waves > 256L * 20 && d.nq > 32) {
      waves /= 2;
      attn_window32_kernel<true><<<dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s>>>(d, (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v,
                                                                                        (bf16_t*)o, (const bf16_t*)rpb_table, waves);
    } else {
      attn_window32_kernel<false><<<dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s>>>(d, (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v,
                                                                                         (bf16_t*)o, (const bf16_t*)rpb_table, waves);
    }
    return (int)hipGetLastError();
  }
  if (d.kind == SM_ATT_STRIPE && (d.d > 32 || d.scale <= 0.f)) return (int)hipErrorInvalidValue;      // one instantiation: head size <= 32
  if (d.kind != SM_ATT_WINDOW && d.scale > 0.f) {
    const int n_qt = (d.nq + 127) / 128, nbh = d.nb * d.heads, dk = (d.d + 15) / 16;
    const bf16_t *qq = (const bf16_t*)q, *kk = (const bf16_t*)k, *vv = (const bf16_t*)v;
    bf16_t* oo = (bf16_t*)o;
    const dim3 grid((unsigned)((long)n_qt * nbh)), block(256);
    // heads interleaved within a cache line (head stride under 128 bytes on the key side): see attn_flash_body
    const int64_t hs = d.k_stride[1] < 0 ? -d.k_stride[1] : d.k_stride[1];
    const int pair = (d.kind != SM_ATT_STRIPE && d.heads % 2 == 0 && hs * 2 < 128 && (nbh / 2) % 8 == 0) ? 1 : 0;
#define FLASH(DK_) do { \
      const size_t smem = 2 * 64 * ((2 * DK_ + 1) + (DK_ <= 2 ? 4 : (DK_ == 3 ? 7 : (DK_ <= 6 ? 12 : 20)))) * 16 + 64;      /* two stages of a K tile and a V tile */ \
      static const hipError_t attr_f = hipFuncSetAttribute((const void*)attn_flash_kernel<DK_, 0>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem); \
      static const hipError_t attr_c = hipFuncSetAttribute((const void*)attn_flash_kernel<DK_, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem); \
      if (attr_f != hipSuccess || attr_c != hipSuccess) return (int)(attr_f != hipSuccess ? attr_f : attr_c); \
      if (d.kind == SM_ATT_CAUSAL) attn_flash_kernel<DK_, 1><<<grid, block, smem, s>>>(d, qq, kk, vv, oo, n_qt, nbh, pair); \
      else attn_flash_kernel<DK_, 0><<<grid, block, smem, s>>>(d, qq, kk, vv, oo, n_qt, nbh, pair); } while (0)
    if (d.kind == SM_ATT_STRIPE) {
      const size_t smem = 2 * 64 * ((2 * 2 + 1) + 4) * 16 + 64;
      static const hipError_t attr_s = hipFuncSetAttribute((const void*)attn_flash_kernel<2, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      if (attr_s != hipSuccess) return (int)attr_s;
      attn_flash_kernel<2, 2><<<grid, block, smem, s>>>(d, qq, kk, vv, oo, n_qt, nbh, 0);
    }
    else if (dk <= 2) FLASH(2);
    else if (dk == 3) FLASH(3);
    else if (dk == 4) FLASH(4);
    else if (dk <= 6) FLASH(6);
    else FLASH(8);
#undef FLASH
    return (int)hipGetLastError();
  }
  const int n_qblk = (d.nq + 31) / 32;
  const long waves = (long)d.nb * d.heads * n_qblk;
  dim3 grid((unsigned)((waves + 3) / 4)), block(256);
  const bf16_t *qq = (const bf16_t*)q, *kk = (const bf16_t*)k, *vv = (const bf16_t*)v, *tt = (const bf16_t*)rpb_table;
  bf16_t* oo = (bf16_t*)o;
  const int dk = (d.d + 15) / 16;
#define ATT(DK_, DB_) do { \
    if (d.kind == SM_ATT_WINDOW) attn_bf16_kernel<DK_, DB_, SM_ATT_WINDOW><<<grid, block, 0, s>>>(d, qq, kk, vv, oo, tt, n_qblk, waves); \
    else if (d.kind == SM_ATT_CAUSAL) attn_bf16_kernel<DK_, DB_, SM_ATT_CAUSAL><<<grid, block, 0, s>>>(d, qq, kk, vv, oo, tt, n_qblk, waves); \
    else attn_bf16_kernel<DK_, DB_, SM_ATT_FULL><<<grid, block, 0, s>>>(d, qq, kk, vv, oo, tt, n_qblk, waves); } while (0)
  if (dk <= 2) ATT(2, 1);
  else if (dk == 3) ATT(3, 2);
  else if (dk == 4) ATT(4, 2);
  else if (dk <= 6) ATT(6, 3);
  else ATT(8, 4);
#undef ATT
  return (int)hipGetLastError();
}

}  // namespace sm
