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

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.f + erff(x * 0.70710678118654752f)); }
__device__ __forceinline__ float silu_f(float x) { return x / (1.f + __expf(-x)); }

enum { EPI_PLAIN = 0, EPI_GELU = 1, EPI_GLU = 2, EPI_ROPE = 3 };

template <typename T, int MI, int EPI, bool AGRAN>
__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs g, ColMap cm, int tiles_n) {
  const SM_KARG GemmArgs* gk = kernarg_ptr<GemmArgs>();      // g is the first argument
  constexpr int VEC = Elem<T>::VEC;
  constexpr int BM = 64 * MI, BN = 128, BK = 8 * VEC;
  constexpr int A_SLOTS = BM * 8, B_SLOTS = BN * 8;
  extern __shared__ u32x4 lds[];                     // [2][A_SLOTS + B_SLOTS]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, hf = lane >> 5;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x - tile_m * tiles_n;
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
    const int64_t r = m0 + lr + 32 * i;
    a_ok[i] = r < g.M;
    a_ptr[i] = A + (a_ok[i] ? (g.a_rows.identity ? r * g.a_rows.ld : eval_rows_k(&gk->a_rows, r)) : 0) + lc * VEC;
  }
  const T* b_ptr[4];
  bool b_ok[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int n = n0 + lr + 32 * i;
    b_ok[i] = n < g.N;
    b_ptr[i] = W + (int64_t)(b_ok[i] ? phys_col(cm, n) : 0) * g.ldw + lc * VEC;
  }

  f32x16_t acc[MI][2];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;

  u32x4 ra[2 * MI], rb[4];
  const u32x4 zero = {0u, 0u, 0u, 0u};
  auto load_tile = [&](int k0) {
    const bool k_ok = k0 + lc * VEC < g.K;
    if constexpr (AGRAN) {
      // K contiguous only in granules of 4 elements (an unfold folded into the load): the chunk is one
      // (fp32) or two (bf16) granules, each addressed through the column program
      const int kq = (k0 + lc * VEC) / 4;
      const int64_t c0 = k_ok ? eval_rows_k(&gk->a_cols, kq) : 0;
      const int64_t c1 = (k_ok && VEC == 8) ? eval_rows_k(&gk->a_cols, kq + 1) : 0;
#pragma unroll
      for (int i = 0; i < 2 * MI; ++i) {
        if (!(a_ok[i] && k_ok)) { ra[i] = zero; continue; }
        const T* base = a_ptr[i] - lc * VEC;
        if constexpr (VEC == 4) ra[i] = *(const u32x4*)(base + c0);
        else {
          const u32x2 lo = *(const u32x2*)(base + c0), hi = *(const u32x2*)(base + c1);
          ra[i] = u32x4{lo.x, lo.y, hi.x, hi.y};
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 2 * MI; ++i) ra[i] = (a_ok[i] && k_ok) ? *(const u32x4*)(a_ptr[i] + k0) : zero;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) rb[i] = (b_ok[i] && k_ok) ? *(const u32x4*)(b_ptr[i] + k0) : zero;
  };
  auto store_tile = [&](int buf) {
    u32x4* a_l = lds + buf * (A_SLOTS + B_SLOTS);
    u32x4* b_l = a_l + A_SLOTS;
#pragma unroll
    for (int i = 0; i < 2 * MI; ++i) { const int r = lr + 32 * i; a_l[r * 8 + (lc ^ (r & 7))] = ra[i]; }
#pragma unroll
    for (int i = 0; i < 4; ++i) { const int r = lr + 32 * i; b_l[r * 8 + (lc ^ (r & 7))] = rb[i]; }
  };

  const int nk = (g.K + BK - 1) / BK;
  load_tile(0);
  store_tile(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    if (kt + 1 < nk) load_tile((kt + 1) * BK);
    const u32x4* a_l = lds + (kt & 1) * (A_SLOTS + B_SLOTS);
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
    if (kt + 1 < nk) store_tile((kt + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue: row offsets of C once per tile (LDS is free now)
  int64_t* c_off = (int64_t*)lds;
  if (tid < BM) {
    const int64_t r = m0 + tid;
    int64_t off = 0;
    if (r < g.M) {
      if (g.c_transposed) { const int64_t bi = r / g.c_batch_rows; off = bi * g.c_batch_rows * (cm.mode == 1 ? cm.half : g.N) + (r - bi * g.c_batch_rows); }
      else off = g.c_rows.identity ? r * g.c_rows.ld : eval_rows_k(&gk->c_rows, r);
    }
    c_off[tid] = off;
  }
  __syncthreads();
  const int n_out = cm.mode == 1 ? cm.half : g.N;
  const int64_t col_stride = g.c_transposed ? g.c_batch_rows : 1;
  T* C = (T*)g.C;
  const T* R = (const T*)g.residual;
  const T* bias = (const T*)g.bias;
  const int span0 = n0 + wn * 64;                    // logical start of this wave's 64 columns
  const int nl0 = span0 + l32, nl1 = span0 + 32 + l32;
  const int pc0 = phys_col(cm, nl0), pc1 = phys_col(cm, nl1);
  const bool ok0 = nl0 < g.N, ok1 = nl1 < g.N;
  // column offsets: plain (n * stride) or through the column program of a store that splits the columns
  int64_t co0 = pc0 * col_stride, co1 = pc1 * col_stride;
  if (g.c_cols_on) { co0 = ok0 ? eval_rows_k(&gk->c_cols, pc0) : 0; co1 = ok1 ? eval_rows_k(&gk->c_cols, pc1) : 0; }
  const float b0 = (bias && ok0) ? Elem<T>::ld(bias + pc0) : 0.f;
  const float b1 = (bias && ok1) ? Elem<T>::ld(bias + pc1) : 0.f;
  const bool rope = EPI == EPI_ROPE && nl0 < cm.rope_cols;
  float theta = 0.f;
  if (rope) {
    const int e = pc0 % cm.rope_dim;                  // index of the pair, < rope_dim / 2
    theta = exp2f(-2.f * (float)e / (float)cm.rope_dim * log2f(g.rope_base));
  }
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int rl = wm * 32 * MI + mi * 32 + (i >> 2) * 8 + hf * 4 + (i & 3);
      const int64_t r = m0 + rl;
      if (r >= g.M) continue;
      float v0 = acc[mi][0][i] + b0, v1 = acc[mi][1][i] + b1;
      const int64_t ro = c_off[rl];
      if constexpr (EPI == EPI_GLU) {
        float o = g.act == SM_ACT_SWIGLU ? silu_f(v0) * v1 : v0 * gelu_erf(v1);
        if (ok0 && pc0 < cm.half) {
          const int64_t off = ro + co0;
          if (R) o += Elem<T>::ld(R + off);
          Elem<T>::st(C + off, o);
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
  (void)n_out;
}

template <typename T, int MI, int EPI, bool AGRAN>
static int gemm_launch(const GemmArgs& g, const ColMap& cm, hipStream_t s) {
  constexpr int BM = 64 * MI;
  const int tiles_n = (g.N + 127) / 128;
  const int64_t tiles_m = (g.M + BM - 1) / BM;
  const size_t smem = 2 * (BM * 8 + 128 * 8) * sizeof(u32x4);
  static const hipError_t attr = hipFuncSetAttribute((const void*)gemm_kernel<T, MI, EPI, AGRAN>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (attr != hipSuccess) return (int)attr;
  gemm_kernel<T, MI, EPI, AGRAN><<<dim3((unsigned)(tiles_m * tiles_n)), dim3(256), smem, s>>>(g, cm, tiles_n);
  return (int)hipGetLastError();
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
  // small problems take the 64-row tile so that the grid still covers the chip
  const int64_t tiles128 = ((g.M + 127) / 128) * ((g.N + 127) / 128);
  return tiles128 >= 512 ? gemm_pick_epi<T, 2>(g, cm, s) : gemm_pick_epi<T, 1>(g, cm, s);
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
