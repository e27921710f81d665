// Mapped Linear: C = epilogue(A . W^T) on the matrix cores (paper Table 3:
// MatMul is ILD & Variable; Sec. 3.2.2: both operands keep the reduction
// dimension K contiguous).  Eliminated layout transformations reach this
// kernel only as row programs: the offset of row r of A (gather side) and of
// row r of C / the residual (scatter side) are evaluated once per tile, outside
// the K loop, so the inner loop is plain 16-byte loads -> LDS -> MFMA.
//
// Tile: BM x 128 outputs per workgroup of 2 * WM waves (WM x 2), BM = 32 * MI * WM; each wave owns MI x 2 MFMA
// blocks of 32 x 32.  A K-tile is 128 bytes per row (64 bf16 / 32 fp32), held in LDS in 16-byte chunks with an XOR
// swizzle (chunk c of row r sits in slot c ^ ((r >> 1) & 7)): the LDS has 64 banks of 4 bytes, a ds_read_b128 is
// served 16 lanes (256 bytes) at a time, two rows span the banks once, so the sixteen consecutive rows read together
// must put their chunk at eight different positions per row parity (the r & 7 form, right for 32 banks, measured
// half of all LDS cycles as bank conflicts).  Two ways into LDS: straight from global memory (LDS-DMA, bf16 with
// K % 64 == 0: the fast path, see gemm_kernel) or through registers, two K-tiles in flight (fp32, ragged K, the
// unfolded A of the patch embedding, and the folded norm, which transforms A on the way).
//
// Column pairing for gated activations and RoPE is done by permuting the
// logical column order of a wave's 64-column span (which W row feeds which
// MFMA block), so that the two partners sit in the same lane: the Slice /
// chunk operators of SwiGLU / GEGLU and the half-split of RoPE cost nothing.
#include <atomic>
#include <map>
#include <mutex>
#include <tuple>
#include <algorithm>
#include <type_traits>
#include "device_common.h"
#include "kernels.h"

namespace sm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // native vector: stays in registers
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

struct TileOrder { int tiles_m, tiles_n, strip, group; };

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
template <typename T> __device__ __forceinline__ float gelu_t(float x) {
  if constexpr (sizeof(T) == 2) return gelu_poly(x);
  else return gelu_erf(x);
}
// sin and cos of an angle given in revolutions (position x frequency / 2 pi, up to a few hundred): the fraction goes to
// the hardware sine / cosine.  The fp32 product carries the angle to about 1e-7 of its size, i.e. 3e-4 rad at 2048
// positions, a tenth of a bf16 ulp of the rotated value; the library sincosf costs the 2048 x 12288 x 4096 projection
// a third of its time in argument reduction.
__device__ __forceinline__ void rope_sincos(float rev, float* sn, float* cs) {
  const float f = __builtin_amdgcn_fractf(rev);
  *sn = __builtin_amdgcn_sinf(f);
  *cs = __builtin_amdgcn_cosf(f);
}
__device__ __forceinline__ float silu_f(float x) { return x / (1.f + __expf(-x)); }

enum { EPI_PLAIN = 0, EPI_GELU = 1, EPI_GLU = 2, EPI_ROPE = 3 };

#define SM_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define SM_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

// The product is formed transposed, C^T = W A^T (the W fragment is the first MFMA operand), so that a lane ends up
// owning ONE output row and runs of four consecutive columns: after one v_permlane32_swap per value pair a lane
// holds eight consecutive bf16 columns, and bias, activation, RoPE, residual add and the 16-byte stores all happen
// in registers: the epilogue needs neither LDS nor a barrier, and LDS holds nothing but K-tile stages.
//
// DMA = true (bf16, K a multiple of 64): the K-tiles go from global memory straight into LDS
// (global_load_lds_dwordx4, no staging registers), NS - 1 tiles ahead of the MFMAs; the fragment reads are
// written as inline ds_read_b128 with explicit lgkmcnt waits and double-buffered registers, so that the
// LDS latency of step j+1 hides behind the MFMAs of step j.
// WM = waves along M (2 or 4): the workgroup has 2 * WM waves and a tile of 32 * MI * WM rows.  The 8-wave shape
// (256 x 128) halves the L2 -> LDS traffic per flop of the 4-wave one and is used where the grid is large enough.
// LNF (register path): LayerNorm / RMSNorm of A's rows folded into the load: row statistics in the prologue, the
// chunks normalised between their arrival in registers and the LDS store.
template <typename T, int MI, int EPI, bool AGRAN, bool DMA, int WM, int NS, bool LNF, bool GEN>
__global__ __launch_bounds__(128 * WM, 2) void gemm_kernel(GemmArgs g, ColMap cm, TileOrder ts) {
  const SM_KARG GemmArgs* gk = kernarg_ptr<GemmArgs>();      // g is the first argument
  // The kernel-argument fields that the per-tile code needs, read once and pinned in scalar registers.  Left to
  // itself the compiler re-reads them from the argument segment where they are used: one scalar load and one wait
  // each, strung one after the other by the branches between them, at every tile boundary.
#define SM_PIN(x) asm volatile("" : "+s"(x))
  int a_ident = g.a_rows.identity, c_ident = g.c_rows.identity, n_cols = g.N, c_cols_on = g.c_cols_on;
  int64_t a_ld = g.a_rows.ld, c_ld = g.c_rows.ld, m_rows = g.M;
  const int32_t* a_tab = g.a_rows.table;
  const int32_t* c_tab = g.c_rows.table;
  const void* bias_p = g.bias;
  const void* res_p = g.residual;
  void* c_p = g.C;
  SM_PIN(a_ident); SM_PIN(c_ident); SM_PIN(n_cols); SM_PIN(c_cols_on); SM_PIN(a_ld); SM_PIN(c_ld); SM_PIN(m_rows);
  SM_PIN(a_tab); SM_PIN(c_tab); SM_PIN(bias_p); SM_PIN(res_p); SM_PIN(c_p);
  int64_t ldw = g.ldw;
  SM_PIN(ldw);
  SM_PIN(cm.mode); SM_PIN(cm.half); SM_PIN(cm.rope_cols); SM_PIN(cm.rope_dim);
  SM_PIN(ts.tiles_m); SM_PIN(ts.tiles_n); SM_PIN(ts.strip); SM_PIN(ts.group);
#undef SM_PIN
  constexpr int VEC = Elem<T>::VEC;
  constexpr int BM = 32 * MI * WM, BN = 128, BK = 8 * VEC;
  constexpr int A_SLOTS = BM * 8, B_SLOTS = BN * 8;
  extern __shared__ u32x4 lds[];                     // [stages][A_SLOTS + B_SLOTS]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave: a scalar
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, hf = lane >> 5;
  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  The tiles are put in an order in which
  // (1) every XCD owns one contiguous run (so what it fetches through its L2 is a compact block of the tile grid:
  // the grid is cut into strips of `ts.strip` column tiles, as many strips as make the sum of the XCDs' A and W
  // panels smallest), and (2) inside a strip the tiles that are resident together form blocks of `ts.group` row
  // tiles by several column tiles rather than one long row, which shares both operands' panels between them.
  // The grid may be smaller than the tile count (a multiple of 8 then): the workgroup takes the virtual block ids
  // blockIdx.x, + gridDim.x, ..., which all fall to its own XCD, in the order of that XCD's run.
  const int n_tiles = ts.tiles_m * ts.tiles_n;
  const int q8 = n_tiles >> 3, r8 = n_tiles & 7;
  const int strip_tiles = ts.strip * ts.tiles_m;
  auto decode = [&](int vb_, int64_t& m0_, int& n0_) {
    const int xcd = vb_ & 7;
    const int t = xcd * q8 + min(xcd, r8) + (vb_ >> 3);          // XCD x owns q8 (+1 if x < r8) consecutive positions
    const int sidx = min(t / strip_tiles, (ts.tiles_n - 1) / ts.strip);
    const int rem = t - sidx * strip_tiles;
    const int sw = min(ts.strip, ts.tiles_n - sidx * ts.strip);         // width of this strip
    const int gidx = rem / (ts.group * sw), r2 = rem - gidx * ts.group * sw;
    const int gh = min(ts.group, ts.tiles_m - gidx * ts.group);         // height of this group of rows
    const int gcol = r2 / gh;
    m0_ = (int64_t)(gidx * ts.group + (r2 - gcol * gh)) * BM;
    n0_ = (sidx * ts.strip + gcol) * BN;
  };
  int vb = blockIdx.x;
  int64_t m0;
  int n0;
  decode(vb, m0, n0);
  const T* A = (const T*)g.A;
  const T* W = (const T*)g.W;
  int span0, pcb[2];                                 // logical start of this wave's 64 columns; W row / bias index of a block's first column
  auto set_cols = [&]() { span0 = n0 + wn * 64; pcb[0] = phys_col(cm, span0); pcb[1] = phys_col(cm, span0 + 32); };
  set_cols();
  // The bias words of this lane's columns (runs of four: 8 or 16 bytes each) are requested at the start of a tile;
  // the tile waits of the K loop (which count loads in issue order) have long since covered them when the epilogue
  // unpacks them.
  constexpr int BW = VEC == 8 ? 2 : 4;
  unsigned braw[2][4][BW];
  auto load_bias = [&]() {
    // unconditional loads (no select on the loaded words, which would make the prologue wait for them): without a
    // bias, or where a run is cut by the end of the columns, a valid address is read and the words are not used
    const bool bias_vec = bias_p && n_cols >= 4;
    const T* bp = bias_vec ? (const T*)bias_p : W;
    const int pmax = bias_vec ? ((n_cols - 4) & ~3) : 0;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int pc = min(pcb[ni] + g4 * 8 + hf * 4, pmax);
        if constexpr (VEC == 8) { const u32x2 b2 = *(const u32x2*)(bp + pc); braw[ni][g4][0] = b2.x; braw[ni][g4][1] = b2.y; }
        else { const u32x4 b4 = *(const u32x4*)(bp + pc); braw[ni][g4][0] = b4.x; braw[ni][g4][1] = b4.y; braw[ni][g4][2] = b4.z; braw[ni][g4][3] = b4.w; }
      }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };
  load_bias();
  // output offsets of this lane's MI rows (INT64_MIN past the last row), also requested at the start of the tile:
  // with a row table they are loads, and nothing in the epilogue should have to wait for them
  int64_t ro_t[MI];
  auto load_out_rows = [&]() {
    int rt[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int64_t r = m0 + (wm * MI + mi) * 32 + l32;
      if (c_ident) ro_t[mi] = r * c_ld;
      else if (c_tab) rt[mi] = c_tab[min(r, m_rows - 1)];
      else ro_t[mi] = eval_rows_k(&gk->c_rows, min(r, m_rows - 1));
    }
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int64_t r = m0 + (wm * MI + mi) * 32 + l32;
      if (!c_ident && c_tab) ro_t[mi] = (int64_t)rt[mi];
      if (r >= m_rows) ro_t[mi] = INT64_MIN;
    }
  };
  load_out_rows();

  f32x16_t acc[MI][2];
  auto zero_acc = [&]() {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;
  };
  zero_acc();

  // s_free: a stage nobody reads or fills any more; synced: a workgroup barrier has been passed since its last read
  auto epilogue = [&](int s_free, bool synced) __attribute__((always_inline)) {
  // ---- epilogue, in registers.  acc[mi][ni][i] is the output of row m0 + (wm MI + mi) 32 + l32 and logical
  // column span0 + 32 ni + cl(i), cl(i) = 8 (i / 4) + 4 hf + i % 4.  A block of 32 logical columns is a run of 32
  // physical columns in every column order (identity, gated halves, RoPE halves).
  T* C = (T*)c_p;
  const T* R = (const T*)res_p;
  const int n_out = EPI == EPI_GLU ? cm.half : n_cols;
  float bv[2][16];
  if constexpr (!GEN) {              // whole runs of four inside the columns, or columns that are never stored
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const unsigned b0 = bias_p ? braw[ni][g4][0] : 0u, b1 = bias_p ? braw[ni][g4][1] : 0u;
        bv[ni][4 * g4] = __uint_as_float(b0 << 16); bv[ni][4 * g4 + 1] = __uint_as_float(b0 & 0xffff0000u);
        bv[ni][4 * g4 + 2] = __uint_as_float(b1 << 16); bv[ni][4 * g4 + 3] = __uint_as_float(b1 & 0xffff0000u);
      }
  } else {
    const T* bias = (const T*)bias_p;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int pc = pcb[ni] + g4 * 8 + hf * 4;
        if (bias && pc + 4 <= n_cols) {
          if constexpr (VEC == 8) {
            const unsigned b0 = braw[ni][g4][0], b1 = braw[ni][g4][1];
            bv[ni][4 * g4] = __uint_as_float(b0 << 16); bv[ni][4 * g4 + 1] = __uint_as_float(b0 & 0xffff0000u);
            bv[ni][4 * g4 + 2] = __uint_as_float(b1 << 16); bv[ni][4 * g4 + 3] = __uint_as_float(b1 & 0xffff0000u);
          } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[ni][4 * g4 + j] = __uint_as_float(braw[ni][g4][j]);
          }
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) bv[ni][4 * g4 + j] = (bias && pc + j < n_cols) ? Elem<T>::ld(bias + pc + j) : 0.f;
        }
      }
  }
  float theta[16];
  const bool rope = EPI == EPI_ROPE && span0 < cm.rope_cols;
  if (rope) {
    // index of the pair, < rope_dim / 2: the block's 32 columns lie inside one half of a head (rope_dim is a multiple
    // of 64), so one scalar remainder serves the wave
    const int e0 = __builtin_amdgcn_readfirstlane(pcb[0]) % cm.rope_dim;
    const float k2 = -2.f / (float)cm.rope_dim * log2f(g.rope_base);
#pragma unroll
    for (int i = 0; i < 16; ++i)
      theta[i] = exp2f((float)(e0 + (i >> 2) * 8 + hf * 4 + (i & 3)) * k2) * 0.15915494309189535f;      // revolutions per position
  }
  const unsigned rope_m0 = EPI == EPI_ROPE ? (unsigned)(m0 % g.rope_seq) : 0u;      // position of the tile's first row (scalar)
  if constexpr (!GEN) {
    // The fast store (the launcher has checked: bf16, row-major, no second copy, the column count and every row /
    // column offset a multiple of 8 elements).  The wave's 32 rows x (one or two blocks of 32 columns) go through LDS
    // (free of K-tiles by now, a private region per wave) and leave as 16-byte pieces with the pieces of a row in
    // adjacent lanes: a store instruction then writes whole 64- or 128-byte runs of a few rows instead of 32 bytes of
    // each of 32 rows, which costs the texture path four cache lines per lane quad and the L2 four times the write
    // requests.  The residual is read in the same pattern and added, in fp32, to the bf16-rounded value.  The code
    // is kept short on purpose: a workgroup runs it once per tile, out of a cold instruction cache.
    constexpr int NBLK = EPI == EPI_GLU ? 1 : 2, ROWB = NBLK * 64, RPITCH = ROWB + 16;      // the pad holds the row's output offset
    constexpr int CPR = NBLK * 4, RPI = 64 / CPR;    // 16-byte pieces per row, rows per 64-lane round
    unsigned char* wreg = (unsigned char*)(lds + s_free * (A_SLOTS + B_SLOTS)) + wave * (32 * RPITCH);
    if (!synced) __syncthreads();                    // every wave has read its last K-tile fragments
    auto rows_fast = [&](auto MI_) __attribute__((always_inline)) {
      constexpr int mi = decltype(MI_)::value;
      const int64_t r = m0 + (wm * MI + mi) * 32 + l32;
      const int64_t ro = ro_t[mi];
      float v0[16], v1[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) { v0[i] = acc[mi][0][i] + bv[0][i]; v1[i] = acc[mi][1][i] + bv[1][i]; }
      if constexpr (EPI == EPI_GLU) {
#pragma unroll
        for (int i = 0; i < 16; ++i) v0[i] = g.act == SM_ACT_SWIGLU ? silu_f(v0[i]) * v1[i] : v0[i] * gelu_t<T>(v1[i]);
      } else if constexpr (EPI == EPI_GELU) {
#pragma unroll
        for (int i = 0; i < 16; ++i) { v0[i] = gelu_t<T>(v0[i]); v1[i] = gelu_t<T>(v1[i]); }
      } else if constexpr (EPI == EPI_ROPE) {
        if (rope) {
          const float pos = (float)((rope_m0 + (unsigned)((wm * MI + mi) * 32 + l32)) % (unsigned)g.rope_seq);
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            float sn, cs;
            rope_sincos(pos * theta[i], &sn, &cs);
            const float a = v0[i], b = v1[i];
            v0[i] = a * cs - b * sn;
            v1[i] = b * cs + a * sn;
          }
        }
      }
#pragma unroll
      for (int nb = 0; nb < NBLK; ++nb) {
        const float* v = nb ? v1 : v0;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {           // columns 8 g4 + 4 hf .. + 3 of the block
          const f32x2 p0 = {v[4 * g4], v[4 * g4 + 1]}, p1 = {v[4 * g4 + 2], v[4 * g4 + 3]};
          *(u32x2*)(wreg + l32 * RPITCH + nb * 64 + g4 * 16 + hf * 8) =
              u32x2{__builtin_bit_cast(unsigned, __builtin_convertvector(p0, bf16x2)), __builtin_bit_cast(unsigned, __builtin_convertvector(p1, bf16x2))};
        }
      }
      if (hf == 0) *(int64_t*)(wreg + l32 * RPITCH + ROWB) = ro;
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // wave-private data: the LDS queue keeps a wave's accesses in order
      __builtin_amdgcn_wave_barrier();
      // all LDS reads, then all residual loads, then the stores: one latency each, not one per round
      constexpr int NIT = 32 / RPI;
      const int c = lane % CPR, col = pcb[c >> 2] + (c & 3) * 8;
      const int64_t coff = c_cols_on ? eval_rows_k(&gk->c_cols, col >> 3) : (int64_t)col;
      u32x4 d[NIT], rr[NIT];
      int64_t off[NIT];
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int rl = it * RPI + lane / CPR;
        d[it] = *(const u32x4*)(wreg + rl * RPITCH + c * 16);
        const int64_t ro2 = *(const int64_t*)(wreg + rl * RPITCH + ROWB);
        off[it] = (ro2 == INT64_MIN || col >= n_out) ? INT64_MIN : ro2 + coff;
      }
      if (R) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) rr[it] = *(const u32x4*)(R + (off[it] == INT64_MIN ? 0 : off[it]));      // element 0: a valid address, not used
#pragma unroll
        for (int it = 0; it < NIT; ++it)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const f32x2 pr = {__uint_as_float(d[it][e] << 16) + __uint_as_float(rr[it][e] << 16), __uint_as_float(d[it][e] & 0xffff0000u) + __uint_as_float(rr[it][e] & 0xffff0000u)};
            d[it][e] = __builtin_bit_cast(unsigned, __builtin_convertvector(pr, bf16x2));
          }
      }
#pragma unroll
      for (int it = 0; it < NIT; ++it)
        if (off[it] != INT64_MIN) *(u32x4*)(C + off[it]) = d[it];
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    };
    rows_fast(std::integral_constant<int, 0>{});
    if constexpr (MI == 2) rows_fast(std::integral_constant<int, 1>{});
  } else {
  // VEC values w[] for columns col .. col + VEC - 1 of row r (output offset of the row: ro)
  int64_t cur_row = 0;               // the row the chunk belongs to (set by epilogue_rows), for the second copy
  auto store_chunk = [&](bool row_ok, int64_t ro, int col, const float* w) __attribute__((always_inline)) {
    if (!row_ok || col >= n_out) return;
    if (g.C2) {                      // the other layout: column-major, consecutive lanes (rows) write consecutive elements
      T* C2 = (T*)g.C2;
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        if (col + e < n_out) Elem<T>::st(C2 + (int64_t)(col + e) * g.M + cur_row, w[e]);
    }
    if (g.c_transposed) {
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        if (col + e < n_out) {
          const int64_t off = ro + (int64_t)(col + e) * g.c_batch_rows;
          Elem<T>::st(C + off, R ? w[e] + Elem<T>::ld(R + off) : w[e]);
        }
      return;
    }
    const bool whole = col + VEC <= n_out && (!g.c_cols_on || g.c_gran == VEC);
    const int64_t off = ro + (g.c_cols_on ? (g.c_gran == VEC ? eval_rows_k(&gk->c_cols, col / VEC) : 0) : col);
    if (whole && (off & (VEC - 1)) == 0) {
      float v[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[e] = w[e];
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
        for (int e = 0; e < 4; ++e) { const f32x2 pr = {v[2 * e], v[2 * e + 1]}; out[e] = __builtin_bit_cast(unsigned, __builtin_convertvector(pr, bf16x2)); }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = __float_as_uint(v[e]);
      }
      *(u32x4*)(C + off) = out;
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        if (col + e < n_out) {
          int64_t oe = off + e;
          if (g.c_cols_on && g.c_gran != VEC) oe = ro + eval_rows_k(&gk->c_cols, col + e);
          Elem<T>::st(C + oe, R ? w[e] + Elem<T>::ld(R + oe) : w[e]);
        }
    }
  };
  // one block of 32 output columns starting at ocb: a lane's sixteen values -> chunks of VEC consecutive columns
  auto store_block = [&](bool row_ok, int64_t ro, int ocb, const float* v) __attribute__((always_inline)) {
    if constexpr (VEC == 8) {
#pragma unroll
      for (int gp = 0; gp < 2; ++gp) {
        // lanes l and l + 32 own the same row: the lower one gives its second run of four and takes the partner's
        // first, so that it holds columns 16 gp .. 16 gp + 7 and the partner 16 gp + 8 .. 16 gp + 15
        float w[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const u32x2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v[8 * gp + j]), __float_as_uint(v[8 * gp + 4 + j]), false, false);
          w[j] = __uint_as_float(sw.x);
          w[4 + j] = __uint_as_float(sw.y);
        }
        store_chunk(row_ok, ro, ocb + (2 * gp + hf) * 8, w);
      }
    } else {
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) store_chunk(row_ok, ro, ocb + g4 * 8 + hf * 4, v + 4 * g4);
    }
  };
  auto epilogue_rows = [&](auto MI_) __attribute__((always_inline)) {
    constexpr int mi = decltype(MI_)::value;
    const int64_t r = m0 + (wm * MI + mi) * 32 + l32;
    const bool row_ok = r < g.M;
    cur_row = r;
    int64_t ro = 0;
    if (row_ok) {
      if (g.c_transposed) { const int64_t bi = r / g.c_batch_rows; ro = bi * g.c_batch_rows * n_out + (r - bi * g.c_batch_rows); }
      else ro = g.c_rows.identity ? r * g.c_rows.ld : eval_rows_k(&gk->c_rows, r);
    }
    float v0[16], v1[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) { v0[i] = acc[mi][0][i] + bv[0][i]; v1[i] = acc[mi][1][i] + bv[1][i]; }
    if constexpr (EPI == EPI_GLU) {
#pragma unroll
      for (int i = 0; i < 16; ++i) v0[i] = g.act == SM_ACT_SWIGLU ? silu_f(v0[i]) * v1[i] : v0[i] * gelu_t<T>(v1[i]);
      store_block(row_ok, ro, pcb[0], v0);
    } else {
      if constexpr (EPI == EPI_GELU) {
#pragma unroll
        for (int i = 0; i < 16; ++i) { v0[i] = gelu_t<T>(v0[i]); v1[i] = gelu_t<T>(v1[i]); }
      }
      if (EPI == EPI_ROPE && rope) {
        const float pos = (float)((rope_m0 + (unsigned)((wm * MI + mi) * 32 + l32)) % (unsigned)g.rope_seq);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          float sn, cs;
          rope_sincos(pos * theta[i], &sn, &cs);
          const float a = v0[i], b = v1[i];
          v0[i] = a * cs - b * sn;
          v1[i] = b * cs + a * sn;
        }
      }
      store_block(row_ok, ro, pcb[0], v0);
      store_block(row_ok, ro, pcb[1], v1);
    }
  };
  epilogue_rows(std::integral_constant<int, 0>{});
  if constexpr (MI == 2) epilogue_rows(std::integral_constant<int, 1>{});
  }
  };

  if constexpr (DMA) {
    // wave-load i of this wave fills rows g8*8 .. g8*8+7 of a tile (1 KiB, 64 consecutive 16-byte slots):
    // lane -> (row, slot position); the chunk that belongs in that slot is position ^ ((row >> 1) & 7)
    constexpr int LA = 2 * MI, LB = 8 / WM, STAGE = A_SLOTS + B_SLOTS;     // wave-loads per wave per stage
    const int lrow = lane >> 3, lpos = lane & 7;
    const T* a_src[LA];
    const T* b_src[LB];
    // the A rows of a tile: their offsets are requested early (pre: with a row table they are loads) and turned into
    // this lane's source pointers when the tile's first K-tiles are issued (fin)
    int a_off32[LA];
    auto src_pre = [&](int64_t m0_) {
      if (!a_ident && a_tab) {
#pragma unroll
        for (int i = 0; i < LA; ++i) a_off32[i] = a_tab[min(m0_ + (wave * LA + i) * 8 + lrow, m_rows - 1)];
      }
    };
    auto src_fin = [&](int64_t m0_, int n0_) {
#pragma unroll
      for (int i = 0; i < LA; ++i) {
        const int rr = (wave * LA + i) * 8 + lrow;
        const int64_t r = min(m0_ + rr, m_rows - 1);   // rows past M repeat the last row: their outputs are never stored
        const int64_t ao = a_ident ? r * a_ld : (a_tab ? (int64_t)a_off32[i] : eval_rows_k(&gk->a_rows, r));
        a_src[i] = A + ao + (lpos ^ ((rr >> 1) & 7)) * VEC;
      }
#pragma unroll
      for (int i = 0; i < LB; ++i) {
        const int rr = (wave * LB + i) * 8 + lrow;
        const int n = min(n0_ + rr, n_cols - 1);
        b_src[i] = W + (int64_t)phys_col(cm, n) * ldw + (lpos ^ ((rr >> 1) & 7)) * VEC;
      }
    };
    src_pre(m0);
    src_fin(m0, n0);
    // quarter `part` (0 .. 3) of the wave-loads of K-tile kt into `stage`; part < 0: all of them
    auto issue = [&](int kt, int stage, int part = -1) __attribute__((always_inline)) {
      u32x4* st = lds + stage * STAGE;
      const int k0 = kt * BK;
      constexpr int LPT_ = LA + LB;
#pragma unroll
      for (int i = 0; i < LPT_; ++i) {
        if (part >= 0 && i * 4 / LPT_ != part) continue;
        if (i < LA) __builtin_amdgcn_global_load_lds(SM_GPTR(a_src[i] + k0), SM_LPTR(st + (wave * LA + i) * 64), 16, 0, 0);
        else __builtin_amdgcn_global_load_lds(SM_GPTR(b_src[i - LA] + k0), SM_LPTR(st + A_SLOTS + (wave * LB + (i - LA)) * 64), 16, 0, 0);
      }
    };
    unsigned fa_addr[MI], fb_addr[2];
    int fa_x[MI], fb_x[2];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) { const int r = wm * 32 * MI + mi * 32 + l32; fa_addr[mi] = r * 128; fa_x[mi] = (r >> 1) & 7; }
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) { const int r = wn * 64 + ni * 32 + l32; fb_addr[ni] = (A_SLOTS + r * 8) * 16; fb_x[ni] = (r >> 1) & 7; }
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
    // The wave-loads of the K-tile that refills `fill_stage` go out a quarter at a time between the MFMA groups: the
    // L1 -> LDS path takes about as long for a tile's bytes as the matrix cores for its flops (64 bytes a clock against
    // 64 flops a byte at 128 x 128), and a wave that issues its loads in one go sits in the full queue, MFMA-less.
    auto compute = [&](int stage, int fill_kt = -1, int fill_stage = 0) __attribute__((always_inline)) {
      const unsigned sbase = (unsigned)(stage * STAGE * 16);
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
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fb[cur][ni]),
                                                                  __builtin_bit_cast(bf16x8_t, fa[cur][mi]), acc[mi][ni], 0, 0, 0);
        if (fill_kt >= 0) issue(fill_kt, fill_stage, j);
      }
    };
    // NS stages, tiles kt+1 .. kt+NS-2 in flight while tile kt is multiplied.  Per tile: wait until this wave's part
    // of it has landed (only the younger tiles' loads may still be outstanding), barrier (everybody's part has
    // landed, and nobody reads the stage of tile kt-1 any more), refill that stage with tile kt+NS-1, multiply.
    constexpr int LPT = LA + LB;                   // loads per wave per tile
    const int nk = g.K / BK;
#pragma unroll
    for (int t = 0; t < NS - 1; ++t)
      if (t < nk) issue(t, t);
    int sc = 0;                                    // stage of the K-tile about to be multiplied
    for (;;) {
      // this workgroup's next tile: its A-row offsets are requested now and arrive behind the K loop
      const int vb_n = vb + (int)gridDim.x;
      const bool more = vb_n < n_tiles;
      int64_t m0_n = 0;
      int n0_n = 0;
      if (more) { decode(vb_n, m0_n, n0_n); src_pre(m0_n); }
      int kt = 0;
      for (; kt + (NS - 1) < nk; ++kt) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * LPT) : "memory");
        __builtin_amdgcn_s_barrier();
        compute(sc, kt + NS - 1, sc == 0 ? NS - 1 : sc - 1);
        sc = sc == NS - 1 ? 0 : sc + 1;
      }
      // the last NS - 1 tiles (fewer if K is short): nothing left to issue, the wait count shrinks with the tiles in flight
#pragma unroll
      for (int left = NS - 2; left >= 0; --left) {
        if (nk > left) {
          if (left == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LPT) : "memory");
          else if (left == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPT) : "memory");
          else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          __builtin_amdgcn_s_barrier();
          compute(sc);
          sc = sc == NS - 1 ? 0 : sc + 1;
        }
      }
      // The next output tile of this workgroup: its first K-tiles are requested before the epilogue of this one, into
      // the stages sc .. sc + NS - 2 (all read for the last time before the barrier below); the epilogue shuffles
      // through the remaining stage, the last one multiplied, and its stores drain while the next tile's loads
      // arrive.  (The waits above count those stores as well: they are older than every load they wait for, so the
      // counts stay on the safe side.)
      __syncthreads();
      if (more) {
        src_fin(m0_n, n0_n);
#pragma unroll
        for (int t = 0; t < NS - 1; ++t)
          if (t < nk) issue(t, sc + t >= NS ? sc + t - NS : sc + t);
      }
      epilogue(sc == 0 ? NS - 1 : sc - 1, true);
      if (!more) break;
      vb = vb_n; m0 = m0_n; n0 = n0_n;
      set_cols();
      load_bias();
      load_out_rows();
      zero_acc();
    }
  } else {
    // global -> register staging, two K-tiles in flight (register sets 0 and 1)
    // loader assignment: chunk lc of rows lr + 32 i
    const int lc = tid & 7, lr = tid >> 3;
    const T* a_ptr[2 * MI];
#pragma unroll
    for (int i = 0; i < 2 * MI; ++i) {
      // rows past M are clamped to the last row: their products land in output rows that are never stored
      const int64_t r = min(m0 + lr + 32 * i, g.M - 1);
      a_ptr[i] = A + (g.a_rows.identity ? r * g.a_rows.ld : eval_rows_k(&gk->a_rows, r)) + lc * VEC;
    }
    const T* b_ptr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int n = min(n0 + lr + 32 * i, g.N - 1);          // clamped like the rows of A
      b_ptr[i] = W + (int64_t)phys_col(cm, n) * g.ldw + lc * VEC;
    }
    u32x4 ra[2][2 * MI], rb[2][4];
    bool kok[2] = {true, true};      // chunk of the staged tile lies inside K (zeroed when stored otherwise)
    const u32x4 zero = {0u, 0u, 0u, 0u};
    // folded norm: statistics of this thread's rows (the eight threads of a row each sum their chunks, then add up)
    float ln_mean[2 * MI], ln_rstd[2 * MI];
    u32x4 rg[2], rbt[2];             // gamma / beta chunk of the staged tile
    auto unpack8 = [&](const u32x4& v, float* f) {
      if constexpr (VEC == 8) {
#pragma unroll
        for (int e = 0; e < 4; ++e) { f[2 * e] = __uint_as_float(v[e] << 16); f[2 * e + 1] = __uint_as_float(v[e] & 0xffff0000u); }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] = __uint_as_float(v[e]);
      }
    };
    if constexpr (LNF) {
      const int nkt = (g.K + BK - 1) / BK;
      float acc1[2 * MI];
#pragma unroll
      for (int i = 0; i < 2 * MI; ++i) acc1[i] = 0.f;
      if (g.norm == 1) {
        for (int t = 0; t < nkt; ++t) {
          const int k0 = t * BK;
          if (k0 + lc * VEC < g.K) {
#pragma unroll
            for (int i = 0; i < 2 * MI; ++i) {
              float f[VEC];
              unpack8(*(const u32x4*)(a_ptr[i] + k0), f);
#pragma unroll
              for (int e = 0; e < VEC; ++e) acc1[i] += f[e];
            }
          }
        }
      }
#pragma unroll
      for (int i = 0; i < 2 * MI; ++i) {
        float v = acc1[i];
        v += __shfl_xor(v, 1, 64); v += __shfl_xor(v, 2, 64); v += __shfl_xor(v, 4, 64);
        ln_mean[i] = v / (float)g.K;         // 0 for RMSNorm
        acc1[i] = 0.f;
      }
      for (int t = 0; t < nkt; ++t) {        // second pass over rows that are in cache by now
        const int k0 = t * BK;
        if (k0 + lc * VEC < g.K) {
#pragma unroll
          for (int i = 0; i < 2 * MI; ++i) {
            float f[VEC];
            unpack8(*(const u32x4*)(a_ptr[i] + k0), f);
#pragma unroll
            for (int e = 0; e < VEC; ++e) { const float d = f[e] - ln_mean[i]; acc1[i] += d * d; }
          }
        }
      }
#pragma unroll
      for (int i = 0; i < 2 * MI; ++i) {
        float v = acc1[i];
        v += __shfl_xor(v, 1, 64); v += __shfl_xor(v, 2, 64); v += __shfl_xor(v, 4, 64);
        ln_rstd[i] = rsqrtf(v / (float)g.K + g.norm_eps);
      }
    }
    auto load_tile = [&](int k0, auto SET) {
      constexpr int S = decltype(SET)::value;
      const bool k_ok = k0 + lc * VEC < g.K;
      kok[S] = k_ok;
      if constexpr (AGRAN) {
        if (g.a_gran == 1) {
          // K not contiguous at all (e.g. a transposed operand read in place, the "sub-optimal read" of Sec. 3.2.2):
          // every element of the chunk is addressed through the column program and loaded on its own
          int64_t ce[VEC];
#pragma unroll
          for (int e = 0; e < VEC; ++e) ce[e] = eval_rows_k(&gk->a_cols, k_ok ? k0 + lc * VEC + e : 0);
#pragma unroll
          for (int i = 0; i < 2 * MI; ++i) {
            const T* base = a_ptr[i] - lc * VEC;
            if constexpr (VEC == 4) {
              ra[S][i] = u32x4{__float_as_uint(base[ce[0]]), __float_as_uint(base[ce[1]]), __float_as_uint(base[ce[2]]), __float_as_uint(base[ce[3]])};
            } else {
#pragma unroll
              for (int e = 0; e < 4; ++e) ra[S][i][e] = (unsigned)base[ce[2 * e]] | ((unsigned)base[ce[2 * e + 1]] << 16);
            }
          }
        } else {
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
        }
      } else {
        const int ks = k_ok ? k0 : -lc * VEC;                  // a chunk past K is loaded from the row's first chunk and zeroed
#pragma unroll
        for (int i = 0; i < 2 * MI; ++i) ra[S][i] = *(const u32x4*)(a_ptr[i] + ks);
      }
      const int ks = k_ok ? k0 : -lc * VEC;
#pragma unroll
      for (int i = 0; i < 4; ++i) rb[S][i] = *(const u32x4*)(b_ptr[i] + ks);
      if constexpr (LNF) {
        rg[S] = *(const u32x4*)((const T*)g.norm_gamma + ks + lc * VEC);
        rbt[S] = g.norm_beta ? *(const u32x4*)((const T*)g.norm_beta + ks + lc * VEC) : zero;
      }
    };
    auto store_tile = [&](int buf, auto SET) {
      constexpr int S = decltype(SET)::value;
      u32x4* a_l = lds + buf * (A_SLOTS + B_SLOTS);
      u32x4* b_l = a_l + A_SLOTS;
      if constexpr (LNF) {
        float gf[VEC], bf[VEC];
        unpack8(rg[S], gf);
        unpack8(rbt[S], bf);
#pragma unroll
        for (int i = 0; i < 2 * MI; ++i) {
          float f[VEC];
          unpack8(ra[S][i], f);
          const float sc_ = ln_rstd[i], sh_ = -ln_mean[i] * ln_rstd[i];
#pragma unroll
          for (int e = 0; e < VEC; ++e) f[e] = fmaf(fmaf(f[e], sc_, sh_), gf[e], bf[e]);
          if constexpr (VEC == 8) {
#pragma unroll
            for (int e = 0; e < 4; ++e) { const f32x2 pr = {f[2 * e], f[2 * e + 1]}; ra[S][i][e] = __builtin_bit_cast(unsigned, __builtin_convertvector(pr, bf16x2)); }
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) ra[S][i][e] = __float_as_uint(f[e]);
          }
        }
      }
#pragma unroll
      for (int i = 0; i < 2 * MI; ++i) { const int r = lr + 32 * i; a_l[r * 8 + (lc ^ ((r >> 1) & 7))] = kok[S] ? ra[S][i] : zero; }
#pragma unroll
      for (int i = 0; i < 4; ++i) { const int r = lr + 32 * i; b_l[r * 8 + (lc ^ ((r >> 1) & 7))] = kok[S] ? rb[S][i] : zero; }
    };
    auto compute_tile = [&](int buf) {
      const u32x4* a_l = lds + buf * (A_SLOTS + B_SLOTS);
      const u32x4* b_l = a_l + A_SLOTS;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = 2 * j + hf;
        u32x4 fa[MI], fb[2];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) { const int r = wm * 32 * MI + mi * 32 + l32; fa[mi] = a_l[r * 8 + (c ^ ((r >> 1) & 7))]; }
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) { const int r = wn * 64 + ni * 32 + l32; fb[ni] = b_l[r * 8 + (c ^ ((r >> 1) & 7))]; }
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < 2; ++ni) {
            if constexpr (sizeof(T) == 2) {
              acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fb[ni]),
                                                                    __builtin_bit_cast(bf16x8_t, fa[mi]), acc[mi][ni], 0, 0, 0);
            } else {
              const float* pa = (const float*)&fa[mi];
              const float* pb = (const float*)&fb[ni];
#pragma unroll
              for (int t = 0; t < 4; ++t)
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(pb[t], pa[t], acc[mi][ni], 0, 0, 0);
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
  }

  if constexpr (!DMA) epilogue(0, false);
}

template <typename T, int MI, int EPI, bool AGRAN, bool DMA, int WM, int NS, bool LNF, bool GEN>
static int gemm_launch3(const GemmArgs& g, const ColMap& cm, hipStream_t s) {
  constexpr int BM = 32 * MI * WM;
  const int tiles_n = (g.N + 127) / 128;
  const int64_t tiles_m = (g.M + BM - 1) / BM;
  if (tiles_m * tiles_n > INT32_MAX) return (int)hipErrorInvalidValue;
  const size_t smem = (size_t)NS * (BM * 8 + 128 * 8) * sizeof(u32x4);
  // strips: xn of them, 8 / xn XCDs per strip; an XCD then reads M / (8 / xn) rows of A and N / xn rows of W, in
  // total xn M + (8 / xn) N rows of K elements: take the xn that makes that smallest
  int xn = 1;
  double best = 1e300;
  for (int c = 1; c <= 8; c *= 2) {
    const double rows = (double)c * (double)g.M + (8.0 / c) * (double)g.N;
    if (rows < best && c <= tiles_n) { best = rows; xn = c; }
  }
  TileOrder ts;
  ts.tiles_m = (int)tiles_m; ts.tiles_n = tiles_n;
  ts.strip = (tiles_n + xn - 1) / xn;
  // row groups pay where the operand panels are long (they then exceed what the L2 keeps between tiles); with short
  // panels the plain row-major order inside a strip fetched less (measured on the K = 384 shapes)
  ts.group = g.K >= 1024 ? (int)std::min<int64_t>(4, tiles_m) : 1;
  static const hipError_t attr = hipFuncSetAttribute((const void*)gemm_kernel<T, MI, EPI, AGRAN, DMA, WM, NS, LNF, GEN>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (attr != hipSuccess) return (int)attr;
  int64_t grid = tiles_m * tiles_n;
  if constexpr (DMA) {
    // as many workgroups as are resident at once (a multiple of 8, so that a workgroup's tiles stay on its XCD): each
    // walks through its share of the tiles, prefetching across the tile boundary
    static const int resident = [&]() {
      int per_cu = 0, cus = 0, dev = 0;
      if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
          hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)gemm_kernel<T, MI, EPI, AGRAN, DMA, WM, NS, LNF, GEN>, 128 * WM, smem) != hipSuccess)
        return 0;
      return (per_cu * cus) & ~7;
    }();
    if (resident >= 8 && grid > resident) grid = resident;
  }
  gemm_kernel<T, MI, EPI, AGRAN, DMA, WM, NS, LNF, GEN><<<dim3((unsigned)grid), dim3(128 * WM), smem, s>>>(g, cm, ts);
  return (int)hipGetLastError();
}

// every offset the program yields is a multiple of `vec` elements (sufficient: its constant and coefficients are)
static bool rows_vec_aligned(const RowProg& p, int vec) {
  if (p.identity) return p.ld % vec == 0;
  if (p.c0 % vec) return false;
  for (int t = 0; t < p.nterm; ++t)
    if (p.t_coef[t] % vec) return false;
  return true;
}

// The short epilogue (whole 16-byte pieces, shuffled through LDS) where the store allows it; the general one otherwise.
template <typename T, int MI, int EPI, bool AGRAN, bool DMA, int WM = 2, int NS = 2, bool LNF = false>
static int gemm_launch2(const GemmArgs& g, const ColMap& cm, hipStream_t s) {
  if constexpr (sizeof(T) == 2) {
    const int n_out = EPI == EPI_GLU ? cm.half : g.N;
    const bool fast = !g.C2 && !g.c_transposed && n_out % 8 == 0 && g.N % 8 == 0 && rows_vec_aligned(g.c_rows, 8) &&
                      (!g.c_cols_on || (g.c_gran == 8 && rows_vec_aligned(g.c_cols, 8)));
    if (fast) return gemm_launch3<T, MI, EPI, AGRAN, DMA, WM, NS, LNF, false>(g, cm, s);
  }
  return gemm_launch3<T, MI, EPI, AGRAN, DMA, WM, NS, LNF, true>(g, cm, s);
}

static std::atomic<int> g_force_rows{0}, g_force_stages{0};       // sm_gemm_tuning (a process-wide sweep hook)
// tile height and stage count of one launch: 0 = the built-in choice.  Comes from sm_gemm_tuning (all shapes) or from
// the table sm_linear_autotune filled for this shape.
struct Tune { int rows, stages; };

// Two stages (one K-tile in flight) unless the tuning hook asks for more: within a chain of kernels the operands
// arrive from the memory-side cache, a workgroup's K step is bound by its own issue and fragment-read latencies
// rather than by the tile's arrival, and every further stage costs a resident workgroup per CU.
template <typename T, int MI, int EPI, int WM>
static int gemm_launch_dma(const GemmArgs& g, const ColMap& cm, hipStream_t s, Tune tn) {
  constexpr int BM = 32 * MI * WM;
  const int64_t stage = (BM + 128) * 128;
  const int ns = tn.stages ? std::min<int>(tn.stages, (int)((160 * 1024) / stage)) : 2;
  if (ns == 4) return gemm_launch2<T, MI, EPI, false, true, WM, 4>(g, cm, s);
  if (ns == 3) return gemm_launch2<T, MI, EPI, false, true, WM, 3>(g, cm, s);
  return gemm_launch2<T, MI, EPI, false, true, WM, 2>(g, cm, s);
}

template <typename T, int MI, int EPI, bool AGRAN>
static int gemm_launch(const GemmArgs& g, const ColMap& cm, hipStream_t s, Tune tn) {
  if constexpr (!AGRAN && (EPI == EPI_PLAIN || EPI == EPI_GELU)) {
    if (g.norm) return gemm_launch2<T, MI, EPI, false, false, 2, 2, true>(g, cm, s);      // checked by the caller: only these epilogues
  }
  if constexpr (sizeof(T) == 2 && !AGRAN) {
    if (g.K % 64 == 0) {
      if (tn.rows == 256 || tn.rows == 128) {
        if constexpr (MI == 2) return tn.rows == 256 ? gemm_launch_dma<T, 2, EPI, 4>(g, cm, s, tn) : gemm_launch_dma<T, 2, EPI, 2>(g, cm, s, tn);
      } else if (tn.rows == 64) {
        if constexpr (MI == 1) return gemm_launch_dma<T, 1, EPI, 2>(g, cm, s, tn);
      }
      if constexpr (MI == 2) {
        // 256 x 128 tiles when they fill the chip (one 8-wave workgroup per CU) about as well as the smaller ones; with a
        // short K loop only on grids of several rounds, where their lower L2 -> LDS traffic per flop pays
        const int64_t t256 = ((g.M + 255) / 256) * ((g.N + 127) / 128);
        const int64_t rounds = (t256 + 255) / 256;
        if (t256 >= (g.K >= 1024 ? 200 : 512) && (double)t256 / (double)(rounds * 256) >= 0.8) return gemm_launch_dma<T, 2, EPI, 4>(g, cm, s, tn);
      }
      return gemm_launch_dma<T, MI, EPI, 2>(g, cm, s, tn);
    }
  }
  return gemm_launch2<T, MI, EPI, AGRAN, false>(g, cm, s);
}

template <typename T, int MI>
static int gemm_pick_epi(const GemmArgs& g, const ColMap& cm, hipStream_t s, Tune tn) {
  if (g.a_gran > 0) return gemm_launch<T, MI, EPI_PLAIN, true>(g, cm, s, tn);     // checked by the caller: no activation with an unfold
  if (cm.mode == 1) return gemm_launch<T, MI, EPI_GLU, false>(g, cm, s, tn);
  if (cm.mode == 2) return gemm_launch<T, MI, EPI_ROPE, false>(g, cm, s, tn);
  if (g.act == SM_ACT_GELU) return gemm_launch<T, MI, EPI_GELU, false>(g, cm, s, tn);
  return gemm_launch<T, MI, EPI_PLAIN, false>(g, cm, s, tn);
}

// Shapes sm_linear_autotune has measured: (M, N, K, element type, epilogue class) -> the fastest (tile rows, stages)
struct TuneKey {
  int64_t M; int N, K, dtype, epi;
  bool operator<(const TuneKey& o) const { return std::tie(M, N, K, dtype, epi) < std::tie(o.M, o.N, o.K, o.dtype, o.epi); }
};
static std::mutex g_tune_mu;
static std::map<TuneKey, Tune> g_tuned;
static TuneKey tune_key(const GemmArgs& g) {
  return TuneKey{g.M, g.N, g.K, g.dtype, g.act * 4 + (g.residual ? 2 : 0) + (g.rope_cols ? 1 : 0)};
}
static bool tunable(const GemmArgs& g) { return g.dtype == SM_BF16 && g.K % 64 == 0 && g.a_gran == 0 && !g.norm; }

template <typename T>
static int gemm_dispatch(const GemmArgs& g, const ColMap& cm, hipStream_t s) {
  Tune tn{g_force_rows, g_force_stages};
  if (!tn.rows && !tn.stages && tunable(g)) {
    std::lock_guard<std::mutex> lock(g_tune_mu);
    auto it = g_tuned.find(tune_key(g));
    if (it != g_tuned.end()) tn = it->second;
  }
  if (tn.rows) return tn.rows >= 128 ? gemm_pick_epi<T, 2>(g, cm, s, tn) : gemm_pick_epi<T, 1>(g, cm, s, tn);
  // Tile height.  Large grids (several rounds of residency whatever the tile): the 128-row tile, or the 256-row one
  // where gemm_launch finds that it fills the chip.  Small grids are decided by rounds of residency (256 CUs hold
  // 768 workgroups of the 64-row tile, 512 of the 128-row one) times the time a workgroup lives: a fixed part plus
  // its K steps, both measured on the chip (microseconds; the 128-row step moves twice the rows in about twice the time,
  // so the smaller tile wins unless it needs an extra round).
  const int64_t tcols = (g.N + 127) / 128;
  const int64_t t128 = ((g.M + 127) / 128) * tcols, t64 = ((g.M + 63) / 64) * tcols;
  if (t128 >= 1024) return gemm_pick_epi<T, 2>(g, cm, s, tn);
  const double nk = (double)((g.K + 63) / 64);
  double cost64 = (double)((t64 + 767) / 768) * (3.0 + 0.78 * nk), cost128 = (double)((t128 + 511) / 512) * (3.6 + 1.6 * nk);
  // long K loops: the tile's L2 -> LDS traffic per flop decides, the 64-row tile being about 0.6 as efficient per row
  if (nk > 16) { cost64 = (double)((t64 + 767) / 768) * 1.2; cost128 = (double)((t128 + 511) / 512) * 2.0; }
  return cost128 <= cost64 ? gemm_pick_epi<T, 2>(g, cm, s, tn) : gemm_pick_epi<T, 1>(g, cm, s, tn);
}

int launch_gemm(const GemmArgs& g, void* stream) {
  if (g.M == 0 || g.N == 0) return 0;
  ColMap cm;
  cm.mode = 0; cm.half = g.N / 2; cm.rope_cols = g.rope_cols; cm.rope_dim = g.rope_dim;
  if (g.act == SM_ACT_SWIGLU || g.act == SM_ACT_GEGLU) cm.mode = 1;
  else if (g.rope_cols > 0) cm.mode = 2;
  return g.dtype == SM_F32 ? gemm_dispatch<float>(g, cm, (hipStream_t)stream) : gemm_dispatch<bf16_t>(g, cm, (hipStream_t)stream);
}

int gemm_tuning(int tile_rows, int stages) {
  if ((tile_rows != 0 && tile_rows != 64 && tile_rows != 128 && tile_rows != 256) || (stages != 0 && (stages < 2 || stages > 4))) return -1;
  g_force_rows = tile_rows; g_force_stages = stages;
  return 0;
}

// The tuner (paper Sec. 3.3 "Other optimizations": an auto-tuner picks tiling and unrolling per kernel; here the
// search space is small enough to be walked completely): every tile height x stage count the kernel has, timed on the
// caller's operands with HIP events; the fastest is remembered for the shape.  0 in *rows / *stages = the built-in choice won.
int gemm_autotune(const GemmArgs& g, int iters, void* stream, int* rows, int* stages, float* best_us, float* default_us) {
  if (!tunable(g)) return -2;
  hipStream_t s = (hipStream_t)stream;
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess) return -1;
  if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return -1; }
  { std::lock_guard<std::mutex> lock(g_tune_mu); g_tuned.erase(tune_key(g)); }
  const int cand_rows[] = {0, 64, 128, 256};
  Tune best{0, 0};
  float best_t = 1e30f, def_t = 0.f;
  int rc = 0;
  for (int ri = 0; ri < 4 && rc == 0; ++ri) {
    for (int st = (ri == 0 ? 0 : 2); st <= (ri == 0 ? 0 : 4) && rc == 0; ++st) {
      const Tune tn{cand_rows[ri], st};
      if (tn.rows) { std::lock_guard<std::mutex> lock(g_tune_mu); g_tuned[tune_key(g)] = tn; }
      for (int w = 0; w < 2 && rc == 0; ++w) rc = launch_gemm(g, stream);
      if (rc == 0 && hipEventRecord(a, s) != hipSuccess) rc = -1;
      for (int i = 0; i < iters && rc == 0; ++i) rc = launch_gemm(g, stream);
      if (rc == 0 && (hipEventRecord(b, s) != hipSuccess || hipEventSynchronize(b) != hipSuccess)) rc = -1;
      float ms = 0.f;
      if (rc == 0 && hipEventElapsedTime(&ms, a, b) != hipSuccess) rc = -1;
      const float us = ms * 1e3f / (float)iters;
      if (ri == 0) def_t = us;
      if (rc == 0 && us < best_t * (ri == 0 ? 1.f : 0.97f)) { best_t = us; best = tn; }     // a candidate has to win by 3 %
    }
  }
  (void)hipEventDestroy(a); (void)hipEventDestroy(b);
  {
    std::lock_guard<std::mutex> lock(g_tune_mu);
    g_tuned.erase(tune_key(g));
    if (rc == 0 && best.rows) g_tuned[tune_key(g)] = best;
  }
  if (rc) return rc;
  *rows = best.rows; *stages = best.stages; *best_us = best_t; *default_us = def_t;
  return 0;
}
void gemm_autotune_clear() { std::lock_guard<std::mutex> lock(g_tune_mu); g_tuned.clear(); }

}  // namespace sm
