// Launchers of the HIP kernels (C++ linkage, called by the C-ABI layer).
// Every launcher validates nothing: shapes and pointers are checked by the
// callers before anything is enqueued.  Each returns the hipError_t of the
// launch as an int (0 = success).
#pragma once
#include <cstdint>
#include "index_map.h"

namespace sm {

int launch_gather(const MapProg& prog, int64_t numel, int vec_elems, const void* src, void* dst, int esize, void* stream);

int launch_gather_add(const MapProg& prog, int64_t numel, int vec_elems, const void* src, const void* addend, void* dst, int dtype, void* stream);

// one wave that returns at once: what an event pair around a launch measures beyond the kernel's own run time
int launch_empty(void* stream);

// row copies: dst row r (inner contiguous elements) = src[rows(r) ...] (+ addend row r); rows(r) keeps 16-byte alignment
// Depth-wise 3 x 3 cross-correlation over the token grid of n_img images of H x W tokens with Cn channels (bf16):
// element (img, y, x, c) of v / out at img * *_img + (y * W + x) * *_tok + c; w [Cn][3][3], bias [Cn].  A tap
// contributes only when it lies in the token's own Hs x Ws stripe (Hs = H, Ws = W: plain zero padding).  split_c > 0
// (a multiple of 8): channels [split_c, Cn) use stripes of Hs2 x Ws2 instead.
struct DwconvArgs {
  const void* v; void* out; const void* w; const void* bias;
  int n_img, H, W, Cn, Hs, Ws;
  int64_t v_img, v_tok, o_img, o_tok;
  int split_c, Hs2, Ws2;
};
int launch_dwconv3x3(const DwconvArgs& a, void* stream);      // Cn a multiple of 8
// two stripe attentions of one shape in one launch; p0 / p1: {q, k, v, o}
int launch_attention_stripe_pair(const sm_attention_desc& d0, const void* const* p0, const sm_attention_desc& d1, const void* const* p1, void* stream);
// out [rows, 2 * cols] = [a | b] along the last axis; cols_bytes (of one input row) a multiple of 16
int launch_concat2_cols(const void* a, const void* b, void* out, int64_t rows, int cols_bytes, void* stream);
int launch_gather_rows(const RowProg& rows, int64_t n_rows, int inner, const void* src, const void* addend, void* dst, int dtype, void* stream);

// table[r] = offset of row r under `prog` (interpreted), r < n_rows: fills one per-row offset table
int launch_fill_rows(const RowProg& prog, int64_t n_rows, int32_t* table, void* stream);
// Several tables in one launch: the programs travel in the kernel-argument segment in a packed form (only the atoms
// and terms a program has), at most FILL_MAX_JOBS tables and FILL_MAX_WORDS words per launch.
constexpr int FILL_MAX_JOBS = 8, FILL_MAX_WORDS = 800;
struct FillBatch {
  int32_t n_jobs, total_blocks;
  int64_t dst[FILL_MAX_JOBS];
  int32_t n_rows[FILL_MAX_JOBS], first_block[FILL_MAX_JOBS], word_off[FILL_MAX_JOBS];
  int32_t words[FILL_MAX_WORDS];
};
int fill_pack(const RowProg& p, int32_t* words, int room);      // words used, or -1 if the program does not fit in `room`
int launch_fill_batch(const FillBatch& b, void* stream);
// collects the tables of several regions (a chain's plans) into as few fill launches as possible
class TableFiller {
 public:
  explicit TableFiller(void* stream) : stream_(stream), used_(0) { b_.n_jobs = 0; b_.total_blocks = 0; }
  int add(const TableRegion& r, void* region, uint64_t which);      // SM_OK or an error; may launch when a batch fills up
  int flush();
 private:
  FillBatch b_; void* stream_; int used_;
};

struct NormArgs {
  const void* x; const void* gamma; const void* beta; void* y;
  int64_t rows; int C; float eps; int rms; int dtype;
  int nseg;             // a logical row is nseg segments of C/nseg elements; segment j of row r is load-row r*nseg+j
  RowProg load, store;
};
int launch_norm(const NormArgs& a, void* stream);

struct GroupNormArgs {
  const void* x; const void* gamma; const void* beta; void* y; int B, C, HW, G; float eps; int tokens_out; int dtype;
  float* stats;      // device scratch of 2 * B * G floats, or null: with it the work is split into a statistics kernel and a
};                   // fully parallel apply kernel (two launches) instead of one workgroup per (image, group)
int launch_groupnorm(const GroupNormArgs& a, void* stream);      // returns the hip error; *launches (if given) = kernels enqueued
int groupnorm_launches(const GroupNormArgs& a);

struct GemmArgs {
  const void* A; const void* W; const void* bias; const void* residual; void* C;
  int64_t M; int N, K;          // N = rows of W (logical columns before gating)
  int dtype, act;
  int rope_cols, rope_dim, rope_seq; float rope_base;
  int c_transposed; int64_t c_batch_rows;
  int64_t ldw;                  // row pitch of W in elements
  RowProg a_rows, c_rows;       // c_rows.ld = pitch of C / residual
  int c_cols_on;                // 1: output column n is stored at c_rows(r) + c_cols(n) (a store that splits the
  RowProg c_cols;               //    column dimension, e.g. into heads)
  int c_gran;                   // c_cols takes n / c_gran and the store adds n % c_gran: 1, or the 16-byte vector width
  int norm;                     // 1 LayerNorm, 2 RMSNorm of every row of A over K, applied as the tile is staged (the norm
  float norm_eps;               //   that precedes the Linear, folded into its load); gamma / beta have K elements,
  const void* norm_gamma;       //   beta may be null
  const void* norm_beta;
  int a_gran;                   // > 0: A's K axis is contiguous only in granules of a_gran (4 or 1) elements;
  RowProg a_cols;               //      offset(r, k) = a_rows(r) + a_cols(k / a_gran) + k % a_gran
  void* C2;                     // non-null: a second copy of the result in the other layout, C2[n * M + r] = C[r][n]
};                              //   (the redundant copy a producer keeps for consumers with another reduction dimension)
int launch_gemm(const GemmArgs& a, void* stream);
int gemm_tuning(int tile_rows, int stages);      // 0 = automatic; -1 on values the kernel has no variant for
// times every (tile rows, stages) variant on g's operands and remembers the fastest for g's shape; synchronises.
// 0 ok, -2 shape has no variants (not the bf16 LDS-DMA path), other: hip error
int gemm_autotune(const GemmArgs& g, int iters, void* stream, int* rows, int* stages, float* best_us, float* default_us);
void gemm_autotune_clear();

// Fused MLP (bf16): Y = residual + W2 . gelu(W1 . norm(x) + b1) + b2 per token.  Wp: W1 [Hd, C] and W2 [C, Hd] packed
// by launch_mlp_pack into MFMA fragment order (2 * Hd * C elements).
struct MlpArgs {
  const void* X; const void* Wp; const void* b1; const void* b2; const void* residual; void* Y;
  int64_t M; int C, Hd;
  int norm; float norm_eps; const void* norm_gamma; const void* norm_beta;     // norm = 1: LayerNorm of X's rows first
  // Wproj_p != null: X is the input of a projection, x1 = X . Wproj^T + bproj + resid0 (resid0 read through y_rows),
  // and the MLP (with its norm and residual) works on x1; Wproj [C, C] packed by launch_lin_pack; `residual` unused
  const void* Wproj_p; const void* bproj; const void* resid0;
  // Y2 != null: a second output Y2 = LayerNorm(Y; ln2_gamma, ln2_beta, ln2_eps), row r stored at y2_rows(r) (the norm
  // that opens the next block, taken while the rows are in registers)
  void* Y2; const void* ln2_gamma; const void* ln2_beta; float ln2_eps;
  // Wq_p != null (with Wproj_p): Y2 is not that norm but the Linear that follows it, Y2 = LayerNorm(Y) . Wq^T + bq with
  // Wq [3 C, C] packed by launch_lin_pack, bq [3 C]; row r stored at 3 * y2_rows(r)
  const void* Wq_p; const void* bq;
  RowProg x_rows, y_rows;       // row r of X; row r of Y and of the residual
  RowProg y2_rows;
};
bool mlp_fused_supported(int C, int Hd, int dtype);
bool mlp_proj_supported(int C, int Hd, int dtype);
int launch_mlp_pack(const void* W1, const void* W2, int C, int Hd, void* packed, void* stream);
int launch_mlp_fused(const MlpArgs& a, void* stream);

// Linear for K in {128, 256, 384} (bf16) with the weight streamed into registers: Y = act(norm(X) . W^T + bias) (+ residual).
// Wp: W [N, K] packed by launch_lin_pack.  act: SM_ACT_NONE or SM_ACT_GELU.
struct Lin32Args {
  const void* X; const void* Wp; const void* bias; const void* residual; void* Y;
  int64_t M; int N, K; int act;
  int norm; float norm_eps; const void* norm_gamma; const void* norm_beta;
  RowProg x_rows, y_rows;       // row r of X; row r of Y and of the residual (pitch N when identity)
};
bool lin32_supported(int N, int K, int dtype);
int launch_lin_pack(const void* W, int N, int K, void* packed, void* stream);
int launch_lin32(const Lin32Args& a, void* stream);

// Decode step (k_decode.hip): bf16, at most 32 tokens, weights packed by launch_lin_pack.
struct DecodeInArgs {
  const unsigned short* x;                      // [B, E]
  const unsigned short *ln1_g, *ln1_b, *ln2_g, *ln2_b; float eps;
  const void *wqkv_p_, *w1_p_;                  // packed [3E, E] (rows ordered [head][q | k | v][d]) and [F, E]
  const unsigned short *bqkv, *b1;
  int B, E, h, d, F, rot, L; float rope_base;   // L: position of the new token (= number of cached tokens)
  unsigned short* dst[3]; int64_t dst_b[3], dst_h[3];   // feature e of head hh of token b of q / k / v goes to dst[t][b * dst_b[t] + hh * dst_h[t] + e]
  unsigned short* hid;                          // [B, F]
  int* counters; int n_counters;                // zeroed here for the two kernels that follow
};
struct DecodeAttnArgs {
  const unsigned short* q; int64_t q_b, q_h;    // query row of (b, hh) at q[b * q_b + hh * q_h]
  const unsigned short *K, *V; int64_t kv_b, kv_h;      // key row t of (b, hh) at K[b * kv_b + hh * kv_h + t * d]
  unsigned short* o; int64_t o_b, o_h;
  float* part; int* counters;                   // [B * h][splits][d + 2] floats; one counter per (b, hh), zero on entry
  int B, h, d, n_keys; float scale_log2e;
};
struct DecodeOutArgs {
  const unsigned short *o, *hid, *x; unsigned short* y;   // [B, E], [B, F], [B, E], [B, E]
  const void *wdense_p_, *w2_p_; const unsigned short *bdense, *b2;
  float* part; int* counters;                   // [splits][B][E] floats; one counter per 32 output features, zero on entry
  int B, E, F;
  int n_dense, per_max;                         // set by the launcher: K splits given to Wdense, most steps of any split
};
size_t decode_in_smem(int B, int E);
int launch_decode_in(const DecodeInArgs& a, void* stream);
int launch_decode_attn(const DecodeAttnArgs& a, int nsplit, void* stream);
int launch_decode_out(const DecodeOutArgs& a, int nks, void* stream);
// out [BH, L + 1, d] = Concat(cache [BH rows of pitch cache_bh_elems][L, d], fresh [BH, d]) along the token axis
int launch_decode_concat(const void* cache, int64_t cache_bh_elems, const void* fresh, void* out, int BH, int L, int d, void* stream);

int launch_attention(const sm_attention_desc& d, const void* q, const void* k, const void* v, void* o,
                     const void* rpb_table, void* stream);

// y[r] = sum over the n contiguous elements of row r (fp32 accumulation): a Reduce whose reduction dimension is innermost
int launch_reduce_last(const void* x, void* y, int64_t rows, int n, int dtype, void* stream);
// y[i] = sum over o < n_outer of x[o * inner + i]: a Reduce over the outermost dimension of a [n_outer, inner] tensor
int launch_reduce_first(const void* x, void* y, int n_outer, int64_t inner, int dtype, void* stream);

// mean over tokens: x [B, L, C] -> y [B, C]
int launch_mean_tokens(const void* x, void* y, int B, int L, int C, int dtype, void* stream);

}  // namespace sm

// validated wrappers shared by the single-operator entry points and the block executors
namespace sm {
int rows_of(const sm_map* m, int64_t rows, int64_t inner, int64_t identity_ld, RowProg* out, const char* who);
int norm_checked(NormArgs& a, void* stream, const char* who);
int gemm_checked(GemmArgs& g, void* stream, const char* who);
int mlp_checked(MlpArgs& a, void* stream, const char* who);
int lin32_checked(Lin32Args& a, void* stream, const char* who);
int attention_checked(const sm_attention_desc& d, const void* q, const void* k, const void* v, void* o, const void* table,
                      void* stream, const char* who);
int attention_stripe_pair_checked(const sm_attention_desc& d0, void* const* p0, const sm_attention_desc& d1, void* const* p1,
                                  void* stream, const char* who);
int map_vector_width(const sm_map& m, int esize);
}
