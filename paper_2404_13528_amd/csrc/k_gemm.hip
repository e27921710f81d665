// Mapped Linear: C = epilogue(A . W^T) on the matrix cores (paper Table 3:
// MatMul is ILD & Variable; Sec. 3.2.2: both operands keep the reduction
// dimension K contiguous).  Eliminated layout transformations reach this
// kernel only as row programs: the offset of row r of A (gather side) and of
// row r of C / the residual (scatter side) are evaluated once per tile, outside
// the K loop, so the inner loop is plain 16-byte loads -> LDS -> MFMA.
//
// Tile: BM x 128 outputs per workgroup of 4 waves (2 x 2), BM = 64 * MI; each
// wave owns MI x 2 MFMA blocks of 32 x 32.  A K-tile is 128 bytes per row
// (64 bf16 / 32 fp32), staged through LDS in 16-byte chunks with an XOR swizzle
// (chunk c of row r sits in slot c ^ (r & 7)) so that the 32 rows read by one
// ds_read_b128 hit distinct banks.  Global loads of tile k+1 are issued before
// the MFMAs of tile k (register double buffering) and two LDS buffers alternate.
//
// Column pairing for gated activations and RoPE is done by permuting the
// logical column order of a wave's 64-column span (which W row feeds which
// MFMA block), so that the two partners sit in the same lane: the Slice /
// chunk operators of SwiGLU / GEGLU and the half-split of RoPE cost nothing.
#include <type_traits>
#include "device_common.h"
#include "kernels.h"

namespace sm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // native vector: stays in registers
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

struct ColMap {      // logical column n' -> physical W row / output column
  int mode;          // 0 identity, 1 gated halves, 2 rope
  int half;          // gated: N / 2
  int rope_cols, rope_dim;
};

__device__ __forceinline__ int phys_col(const ColMap& cm, int n) {
  if (cm.mode == 1) {
    const int p = n >> 6, w = n & 63;
    return w < 32 ? p * 32 + w : cm.half + p * 32 + (w - 32);
  }
  if (cm.mode == 2 && n < cm.rope_cols) {
    const int head = n / cm.rope_dim, u = n - head * cm.rope_dim;
    const int q = u >> 6, w = u & 63;
    const int e = w < 32 ? q * 32 + w : q * 32 + (w - 32) + (cm.rope_dim >> 1);
    return head * cm.rope_dim + e;
  }
  return n;
}

// erf by the rational approximation 7.1.26 of Abramowitz & Stegun (absolute error < 1.5e-7), which costs one
// reciprocal and one exponential instead of the library routine's long polynomial chain
__device__ __forceinline__ float erf_as(float x) {
  const float ax = fabsf(x);
  const float t = __frcp_rn(1.f + 0.3275911f * ax);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float r = 1.f - poly * __expf(-ax * ax);
  return copysignf(r, x);
}
__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.f + erf_as(x * 0.70710678118654752f)); }
__device__ __forceinline__ float silu_f(float x) { return x / (1.f + __expf(-x)); }

enum { EPI_PLAIN = 0, EPI_GELU = 1, EPI_GLU = 2, EPI_ROPE = 3 };

#define SM_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define SM_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

// DMA = true (bf16, K a multiple of 64): the K-tiles go from global memory straight into LDS
// (global_load_lds_dwordx4, no staging registers), one tile ahead of the MFMAs; the fragment reads are
// written as inline ds_read_b128 with explicit lgkmcnt waits and double-buffered registers, so that the
// LDS latency of step j+1 hides behind the MFMAs of step j.
// WM = waves along M (2 or 4): the workgroup has 2 * WM waves and a tile of 32 * MI * WM rows.  The 8-wave shape
// (256 x 128) halves the L2 -> LDS traffic per flop of the 4-wave one and is used where the grid is large enough.
template <typename T, int MI, int EPI, bool AGRAN, bool DMA, int WM>
__global__ __launch_bounds__(128 * WM) void gemm_kernel(GemmArgs g, ColMap cm, int tiles_n) {
  const SM_KARG GemmArgs* gk = kernarg_ptr<GemmArgs>();      // g is the first argument
  constexpr int VEC = Elem<T>::VEC;
  constexpr int BM = 32 * MI * WM, BN = 128, BK = 8 * VEC, NT = 128 * WM;
  constexpr int A_SLOTS = BM * 8, B_SLOTS = BN * 8;
  extern __shared__ u32x4 lds[];                     // [2][A_SLOTS + B_SLOTS]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, hf = lane >> 5;
  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2: give every XCD a contiguous range of
  // tiles (column tiles fastest) so that the tiles sharing an A row panel share one L2.
  const int n_tiles = gridDim.x;
  const int xcd = blockIdx.x & 7, q8 = n_tiles >> 3, r8 = n_tiles & 7;
  const int tile_id = xcd * q8 + min(xcd, r8) + (blockIdx.x >> 3);    // XCD x owns q8 (+1 if x < r8) consecutive tiles
  const int tile_m = tile_id / tiles_n, tile_n = tile_id - tile_m * tiles_n;
  const int64_t m0 = (int64_t)tile_m * BM;
  const int n0 = tile_n * BN;
  const T* A = (const T*)g.A;
  const T* W = (const T*)g.W;

  // loader assignment: chunk c of rows lr + 32*i
  const int lc = tid & 7, lr = tid >> 3;
  const T* a_ptr[2 * MI];
  bool a_ok[2 * MI];
#pragma unroll
  for (int i = 0; i < 2 * MI; ++i) {
    // rows past M are clamped to the last row: their products land in output rows that are never stored
    const int64_t r = min(m0 + lr + 32 * i, g.M - 1);
    a_ok[i] = true;
    a_ptr[i] = A + (g.a_rows.identity ? r * g.a_rows.ld : eval_rows_k(&gk->a_rows, r)) + lc * VEC;
  }
  const T* b_ptr[4];
  bool b_ok[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int n = min(n0 + lr + 32 * i, g.N - 1);          // clamped like the rows of A
    b_ok[i] = true;
    b_ptr[i] = W + (int64_t)phys_col(cm, n) * g.ldw + lc * VEC;
  }

  // row (and column) offsets of C: evaluated here, before the accumulators are live, into LDS behind the tiles
  constexpr int TILE_BYTES = 2 * (A_SLOTS + B_SLOTS) * 16, STAGE_BYTES = BM * 132 * 4;
  int64_t* c_off = (int64_t*)((char*)lds + (TILE_BYTES > STAGE_BYTES ? TILE_BYTES : STAGE_BYTES));
  if (tid < BM) {
    const int64_t r = m0 + tid;
    int64_t off = 0;
    if (r < g.M) {
      if (g.c_transposed) { const int64_t bi = r / g.c_batch_rows; off = bi * g.c_batch_rows * (cm.mode == 1 ? cm.half : g.N) + (r - bi * g.c_batch_rows); }
      else off = g.c_rows.identity ? r * g.c_rows.ld : eval_rows_k(&gk->c_rows, r);
    }
    c_off[tid] = off;
  }
  const int span0 = n0 + wn * 64;                    // logical start of this wave's 64 columns
  const int nl0 = span0 + l32, nl1 = span0 + 32 + l32;
  const int pc0 = phys_col(cm, nl0), pc1 = phys_col(cm, nl1);
  const bool ok0 = nl0 < g.N, ok1 = nl1 < g.N;
  const int64_t col_stride = g.c_transposed ? g.c_batch_rows : 1;
  int64_t co0 = pc0 * col_stride, co1 = pc1 * col_stride;
  if (g.c_cols_on) { co0 = ok0 ? eval_rows_k(&gk->c_cols, pc0) : 0; co1 = ok1 ? eval_rows_k(&gk->c_cols, pc1) : 0; }

  f32x16_t acc[MI][2];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;

  if constexpr (DMA) {
    // wave-load i of this wave fills rows g8*8 .. g8*8+7 of a tile (1 KiB, 64 consecutive 16-byte slots):
    // lane -> (row, slot position); the chunk that belongs in that slot is position ^ (row & 7)
    constexpr int LA = 2 * MI, LB = 8 / WM, STAGE = A_SLOTS + B_SLOTS;     // wave-loads per wave per stage
    const int lrow = lane >> 3, lpos = lane & 7;
    const T* a_src[LA];
    const T* b_src[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int rr = (wave * LA + i) * 8 + lrow;
      const int64_t r = min(m0 + rr, g.M - 1);
      a_src[i] = A + (g.a_rows.identity ? r * g.a_rows.ld : eval_rows_k(&gk->a_rows, r)) + (lpos ^ (rr & 7)) * VEC;
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      const int rr = (wave * LB + i) * 8 + lrow;
      const int n = min(n0 + rr, g.N - 1);
      b_src[i] = W + (int64_t)phys_col(cm, n) * g.ldw + (lpos ^ (rr & 7)) * VEC;
    }
    auto issue = [&](int kt) {
      u32x4* st = lds + (kt & 1) * STAGE;
      const int k0 = kt * BK;
#pragma unroll
      for (int i = 0; i < LA; ++i) __builtin_amdgcn_global_load_lds(SM_GPTR(a_src[i] + k0), SM_LPTR(st + (wave * LA + i) * 64), 16, 0, 0);
#pragma unroll
      for (int i = 0; i < LB; ++i) __builtin_amdgcn_global_load_lds(SM_GPTR(b_src[i] + k0), SM_LPTR(st + A_SLOTS + (wave * LB + i) * 64), 16, 0, 0);
    };
    unsigned fa_addr[MI], fb_addr[2];
    int fa_x[MI], fb_x[2];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) { const int r = wm * 32 * MI + mi * 32 + l32; fa_addr[mi] = r * 128; fa_x[mi] = r & 7; }
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) { const int r = wn * 64 + ni * 32 + l32; fb_addr[ni] = (A_SLOTS + r * 8) * 16; fb_x[ni] = r & 7; }
    auto read_frags = [&](unsigned sbase, int j, u32x4* fa, u32x4* fb) {
      const int c = 2 * j + hf;
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const unsigned ad = sbase + fa_addr[mi] + ((c ^ fa_x[mi]) << 4);
        asm volatile("ds_read_b128 %0, %1" : "=v"(fa[mi]) : "v"(ad));
      }
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) {
        const unsigned ad = sbase + fb_addr[ni] + ((c ^ fb_x[ni]) << 4);
        asm volatile("ds_read_b128 %0, %1" : "=v"(fb[ni]) : "v"(ad));
      }
    };
    auto compute = [&](int kt) {
      const unsigned sbase = (unsigned)((kt & 1) * STAGE * 16);
      u32x4 fa[2][MI], fb[2][2];
      read_frags(sbase, 0, fa[0], fb[0]);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int cur = j & 1;
        if (j < 3) {
          read_frags(sbase, j + 1, fa[cur ^ 1], fb[cur ^ 1]);
          // LDS returns in order: step j's MI + 2 reads have landed once only step j+1's are outstanding
          if constexpr (MI == 2) asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(fa[cur][0]), "+v"(fa[cur][1]), "+v"(fb[cur][0]), "+v"(fb[cur][1]));
          else asm volatile("s_waitcnt lgkmcnt(3)" : "+v"(fa[cur][0]), "+v"(fb[cur][0]), "+v"(fb[cur][1]));
        } else {
          if constexpr (MI == 2) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(fa[cur][0]), "+v"(fa[cur][1]), "+v"(fb[cur][0]), "+v"(fb[cur][1]));
          else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(fa[cur][0]), "+v"(fb[cur][0]), "+v"(fb[cur][1]));
        }
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < 2; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fa[cur][mi]),
                                                                  __builtin_bit_cast(bf16x8_t, fb[cur][ni]), acc[mi][ni], 0, 0, 0);
      }
    };
    // the row offsets of C written above must be visible before the epilogue: the loop's barriers order them
    const int nk = g.K / BK;
    issue(0);
    int kt = 0;
    for (; kt + 1 < nk; ++kt) {
      __builtin_amdgcn_s_waitcnt(0x0f70);        // vmcnt(0): this wave's part of tile kt is in LDS
      __builtin_amdgcn_s_barrier();              // ... and everybody's; buffer (kt + 1) & 1 is no longer read
      issue(kt + 1);
      compute(kt);
    }
    __builtin_amdgcn_s_waitcnt(0x0f70);
    __builtin_amdgcn_s_barrier();
    compute(kt);
    __syncthreads();
  } else {
  // global -> register staging, two K-tiles in flight (register sets 0 and 1)
    u32x4 ra[2][2 * MI], rb[2][4];
    bool kok[2] = {true, true};      // chunk of the staged tile lies inside K (zeroed when stored otherwise)
    const u32x4 zero = {0u, 0u, 0u, 0u};
    auto load_tile = [&](int k0, auto SET) {
      constexpr int S = decltype(SET)::value;
      const bool k_ok = k0 + lc * VEC < g.K;
      kok[S] = k_ok;
      if constexpr (AGRAN) {
        // K contiguous only in granules of 4 elements (an unfold folded into the load): the chunk is one
        // (fp32) or two (bf16) granules, each addressed through the column program
        const int kq = (k0 + lc * VEC) / 4;
        const int64_t c0 = eval_rows_k(&gk->a_cols, k_ok ? kq : 0);
        const int64_t c1 = VEC == 8 ? eval_rows_k(&gk->a_cols, k_ok ? kq + 1 : 0) : 0;
#pragma unroll
        for (int i = 0; i < 2 * MI; ++i) {
          const T* base = a_ptr[i] - lc * VEC;
          if constexpr (VEC == 4) ra[S][i] = *(const u32x4*)(base + c0);
          else {
            const u32x2 lo = *(const u32x2*)(base + c0), hi = *(const u32x2*)(base + c1);
            ra[S][i] = u32x4{lo.x, lo.y, hi.x, hi.y};
          }
        }
      } else {
        const int ks = k_ok ? k0 : 0;                          // a chunk past K is loaded from chunk 0 and zeroed
#pragma unroll
        for (int i = 0; i < 2 * MI; ++i) ra[S][i] = *(const u32x4*)(a_ptr[i] + ks);
      }
      const int ks = k_ok ? k0 : 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) rb[S][i] = *(const u32x4*)(b_ptr[i] + ks);
    };
    auto store_tile = [&](int buf, auto SET) {
      constexpr int S = decltype(SET)::value;
      u32x4* a_l = lds + buf * (A_SLOTS + B_SLOTS);
      u32x4* b_l = a_l + A_SLOTS;
#pragma unroll
      for (int i = 0; i < 2 * MI; ++i) { const int r = lr + 32 * i; a_l[r * 8 + (lc ^ (r & 7))] = kok[S] ? ra[S][i] : zero; }
#pragma unroll
      for (int i = 0; i < 4; ++i) { const int r = lr + 32 * i; b_l[r * 8 + (lc ^ (r & 7))] = kok[S] ? rb[S][i] : zero; }
    };
    auto compute_tile = [&](int buf) {
      const u32x4* a_l = lds + buf * (A_SLOTS + B_SLOTS);
      const u32x4* b_l = a_l + A_SLOTS;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = 2 * j + hf;
        u32x4 fa[MI], fb[2];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) { const int r = wm * 32 * MI + mi * 32 + l32; fa[mi] = a_l[r * 8 + (c ^ (r & 7))]; }
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) { const int r = wn * 64 + ni * 32 + l32; fb[ni] = b_l[r * 8 + (c ^ (r & 7))]; }
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < 2; ++ni) {
            if constexpr (sizeof(T) == 2) {
              acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fa[mi]),
                                                                    __builtin_bit_cast(bf16x8_t, fb[ni]), acc[mi][ni], 0, 0, 0);
            } else {
              const float* pa = (const float*)&fa[mi];
              const float* pb = (const float*)&fb[ni];
#pragma unroll
              for (int t = 0; t < 4; ++t)
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[t], pb[t], acc[mi][ni], 0, 0, 0);
            }
          }
      }
    };
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;

    // Software pipeline: while tile k is multiplied out of LDS buffer k&1, tile k+1 sits in registers and the
    // loads of tile k+2 are in flight.  Tile t always uses register set t&1 and LDS buffer t&1.
    const int nk = (g.K + BK - 1) / BK;
    load_tile(0, S0{});
    if (nk > 1) load_tile(BK, S1{});
    store_tile(0, S0{});
    __syncthreads();
    // steady state: every load and store of a trip is unconditional, so that the compiler's wait counters see
    // exactly one register set in flight at each store; the last one to three tiles are peeled below
    int kt = 0;
    for (; kt + 3 < nk; kt += 2) {
      load_tile((kt + 2) * BK, S0{});
      __builtin_amdgcn_sched_barrier(0);          // keep the loads at the top of the phase: they need its whole length
      compute_tile(0);
      store_tile(1, S1{});
      __syncthreads();
      load_tile((kt + 3) * BK, S1{});
      __builtin_amdgcn_sched_barrier(0);
      compute_tile(1);
      store_tile(0, S0{});
      __syncthreads();
    }
    const int left = nk - kt;                     // 1, 2 or 3 tiles: kt in LDS buffer 0, kt + 1 in register set 1
    if (left == 3) load_tile((kt + 2) * BK, S0{});
    compute_tile(0);
    if (left >= 2) {
      store_tile(1, S1{});
      __syncthreads();
      compute_tile(1);
      if (left == 3) {
        store_tile(0, S0{});
        __syncthreads();
        compute_tile(0);
      }
    }
    __syncthreads();
  }

  // ---- epilogue
  T* C = (T*)g.C;
  const T* R = (const T*)g.residual;
  const T* bias = (const T*)g.bias;
  const float b0 = (bias && ok0) ? Elem<T>::ld(bias + pc0) : 0.f;
  const float b1 = (bias && ok1) ? Elem<T>::ld(bias + pc1) : 0.f;
  const bool rope = EPI == EPI_ROPE && nl0 < cm.rope_cols;
  float theta = 0.f;
  if (rope) {
    const int e = pc0 % cm.rope_dim;                  // index of the pair, < rope_dim / 2
    theta = exp2f(-2.f * (float)e / (float)cm.rope_dim * log2f(g.rope_base));
  }
  // Staged epilogue: when the tile's output columns are one contiguous run and rows are stored whole, the values
  // (bias, activation, RoPE applied) go through LDS as fp32 so that the residual is read and the result written
  // in 16-byte row pieces; otherwise each lane stores its own elements.
  constexpr int EP = 132;                              // padded row pitch of the staging tile (floats)
  const bool staged = !g.c_cols_on && !g.c_transposed && (EPI != EPI_ROPE || cm.rope_dim <= 128);
  float* stage = (float*)lds;
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int rl = wm * 32 * MI + mi * 32 + (i >> 2) * 8 + hf * 4 + (i & 3);
      const int64_t r = m0 + rl;
      float v0 = acc[mi][0][i] + b0, v1 = acc[mi][1][i] + b1;
      if constexpr (EPI == EPI_GLU) {
        const float o = g.act == SM_ACT_SWIGLU ? silu_f(v0) * v1 : v0 * gelu_erf(v1);
        if (staged) { stage[rl * EP + wn * 32 + l32] = o; continue; }
        if (r < g.M && ok0 && pc0 < cm.half) {
          const int64_t off = c_off[rl] + co0;
          Elem<T>::st(C + off, R ? o + Elem<T>::ld(R + off) : o);
        }
        continue;
      }
      if constexpr (EPI == EPI_GELU) { v0 = gelu_erf(v0); v1 = gelu_erf(v1); }
      if (EPI == EPI_ROPE && rope) {
        const float ang = (float)(r % g.rope_seq) * theta;
        float sn, cs;
        sincosf(ang, &sn, &cs);
        const float a = v0, b = v1;
        v0 = a * cs - b * sn;
        v1 = b * cs + a * sn;
      }
      if (staged) {                                    // physical column inside the tile
        stage[rl * EP + (pc0 - n0)] = v0;
        stage[rl * EP + (pc1 - n0)] = v1;
        continue;
      }
      if (r >= g.M) continue;
      const int64_t ro = c_off[rl];
      if (ok0) {
        const int64_t off = ro + co0;
        if (R) v0 += Elem<T>::ld(R + off);
        Elem<T>::st(C + off, v0);
      }
      if (ok1) {
        const int64_t off = ro + co1;
        if (R) v1 += Elem<T>::ld(R + off);
        Elem<T>::st(C + off, v1);
      }
    }
  }
  if (staged) {
    __syncthreads();
    constexpr int TW = EPI == EPI_GLU ? 64 : 128;      // output columns of the tile
    constexpr int CPR = TW / VEC;                      // 16-byte pieces per row
    const int n_out = EPI == EPI_GLU ? cm.half : g.N;
    const int c_base = EPI == EPI_GLU ? n0 / 2 : n0;
    for (int p = tid; p < BM * CPR; p += NT) {
      const int rl = p / CPR, cl = (p - rl * CPR) * VEC;
      const int64_t r = m0 + rl;
      const int col = c_base + cl;
      if (r >= g.M || col >= n_out) continue;
      const int64_t off = c_off[rl] + col;
      float v[VEC];
#pragma unroll
      for (int e = 0; e < VEC; e += 4) {
        const float4 t = *(const float4*)(stage + rl * EP + cl + e);
        v[e] = t.x; v[e + 1] = t.y; v[e + 2] = t.z; v[e + 3] = t.w;
      }
      if (col + VEC <= n_out && (off & (VEC - 1)) == 0) {
        if (R) {
          const u32x4 rr = *(const u32x4*)(R + off);
          if constexpr (VEC == 8) {
#pragma unroll
            for (int e = 0; e < 4; ++e) { v[2 * e] += __uint_as_float(rr[e] << 16); v[2 * e + 1] += __uint_as_float(rr[e] & 0xffff0000u); }
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += __uint_as_float(rr[e]);
          }
        }
        u32x4 out;
        if constexpr (VEC == 8) {
#pragma unroll
          for (int e = 0; e < 4; ++e) out[e] = (unsigned)f2bf(v[2 * e]) | ((unsigned)f2bf(v[2 * e + 1]) << 16);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) out[e] = __float_as_uint(v[e]);
        }
        *(u32x4*)(C + off) = out;
      } else {
        for (int e = 0; e < VEC && col + e < n_out; ++e)
          Elem<T>::st(C + off + e, R ? v[e] + Elem<T>::ld(R + off + e) : v[e]);
      }
    }
  }
}

template <typename T, int MI, int EPI, bool AGRAN, bool DMA, int WM = 2>
static int gemm_launch2(const GemmArgs& g, const ColMap& cm, hipStream_t s) {
  constexpr int BM = 32 * MI * WM;
  const int tiles_n = (g.N + 127) / 128;
  const int64_t tiles_m = (g.M + BM - 1) / BM;
  const size_t tiles = 2 * (BM * 8 + 128 * 8) * sizeof(u32x4), stage = (size_t)BM * 132 * sizeof(float);
  const size_t smem = (tiles > stage ? tiles : stage) + BM * sizeof(int64_t);
  static const hipError_t attr = hipFuncSetAttribute((const void*)gemm_kernel<T, MI, EPI, AGRAN, DMA, WM>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (attr != hipSuccess) return (int)attr;
  gemm_kernel<T, MI, EPI, AGRAN, DMA, WM><<<dim3((unsigned)(tiles_m * tiles_n)), dim3(128 * WM), smem, s>>>(g, cm, tiles_n);
  return (int)hipGetLastError();
}

template <typename T, int MI, int EPI, bool AGRAN>
static int gemm_launch(const GemmArgs& g, const ColMap& cm, hipStream_t s) {
  if constexpr (sizeof(T) == 2 && !AGRAN) {
    if (g.K % 64 == 0) {
      if constexpr (MI == 2) {
        // 256 x 128 tiles when they fill the chip (one 8-wave workgroup per CU) about as well as the smaller ones
        const int64_t t256 = ((g.M + 255) / 256) * ((g.N + 127) / 128);
        const int64_t rounds = (t256 + 255) / 256;
        if (t256 >= 200 && (double)t256 / (double)(rounds * 256) >= 0.8) return gemm_launch2<T, 2, EPI, false, true, 4>(g, cm, s);
      }
      return gemm_launch2<T, MI, EPI, false, true>(g, cm, s);
    }
  }
  return gemm_launch2<T, MI, EPI, AGRAN, false>(g, cm, s);
}

template <typename T, int MI>
static int gemm_pick_epi(const GemmArgs& g, const ColMap& cm, hipStream_t s) {
  if (g.a_gran > 0) return gemm_launch<T, MI, EPI_PLAIN, true>(g, cm, s);     // checked by the caller: no activation with an unfold
  if (cm.mode == 1) return gemm_launch<T, MI, EPI_GLU, false>(g, cm, s);
  if (cm.mode == 2) return gemm_launch<T, MI, EPI_ROPE, false>(g, cm, s);
  if (g.act == SM_ACT_GELU) return gemm_launch<T, MI, EPI_GELU, false>(g, cm, s);
  return gemm_launch<T, MI, EPI_PLAIN, false>(g, cm, s);
}

template <typename T>
static int gemm_dispatch(const GemmArgs& g, const ColMap& cm, hipStream_t s) {
  // Tile height by how the grid fills the chip: 256 CUs hold 512 workgroups of the 128-row tile (64 KiB of LDS each)
  // or 768 of the 64-row tile; count rounds of residency, the 64-row tile being about 0.6 as efficient per row.
  const int64_t tn = (g.N + 127) / 128;
  const int64_t t128 = ((g.M + 127) / 128) * tn, t64 = ((g.M + 63) / 64) * tn;
  const double cost128 = (double)((t128 + 511) / 512) * 2.0, cost64 = (double)((t64 + 767) / 768) * 1.2;
  return (t128 >= 1024 || cost128 <= cost64) ? gemm_pick_epi<T, 2>(g, cm, s) : gemm_pick_epi<T, 1>(g, cm, s);
}

int launch_gemm(const GemmArgs& g, void* stream) {
  if (g.M == 0 || g.N == 0) return 0;
  ColMap cm;
  cm.mode = 0; cm.half = g.N / 2; cm.rope_cols = g.rope_cols; cm.rope_dim = g.rope_dim;
  if (g.act == SM_ACT_SWIGLU || g.act == SM_ACT_GEGLU) cm.mode = 1;
  else if (g.rope_cols > 0) cm.mode = 2;
  return g.dtype == SM_F32 ? gemm_dispatch<float>(g, cm, (hipStream_t)stream) : gemm_dispatch<bf16_t>(g, cm, (hipStream_t)stream);
}

}  // namespace sm
