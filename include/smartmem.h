/* smartmem.h - C ABI of the MI355X layout-elided transformer-chain library.
 *
 * The library executes transformer operator chains with their explicit layout
 * transformations (Reshape, Transpose/Permute, cyclic roll, window partition and
 * reverse, head split and merge, patch merging, NCHW<->token rearrangement)
 * eliminated: a consumer kernel reads its producer's tensor in the producer's
 * layout through a composed index map (SmartMem, arxiv 2404.13528, Sec. 3).
 *
 * General conventions
 *   - Every function returns an int status (SM_OK or a negative SM_ERR_*);
 *     sm_last_error() gives a thread-local message for the last failure.
 *     No exception crosses this boundary.
 *   - "device pointer": memory of the current HIP device, owned by the caller,
 *     16-byte aligned.  "host pointer": ordinary process memory.
 *   - No entry point allocates, frees or copies device memory, and none
 *     synchronises: all device work is kernels enqueued on the hipStream_t passed
 *     as `void* stream` (NULL = the default stream), so any call, a first call
 *     included, may be captured into a HIP graph.  Scratch memory comes from the
 *     caller as `ws` / `ws_bytes`; the matching *_workspace_bytes() call gives
 *     the size needed (activation buffers plus the per-row offset tables of the
 *     call's index maps, which the executors fill with small kernels at the
 *     start of every call; nothing in `ws` has to survive between calls).  An
 *     undersized workspace returns SM_ERR_WORKSPACE before anything is launched.
 *     The executors keep the plans of the configurations they have seen in a
 *     bounded, mutex-guarded cache of host objects.  Two exceptions, both
 *     diagnostics a caller switches on: sm_timing_enable() brackets launches
 *     with HIP events and sm_timing_report() waits for them; sm_gemm_tuning()
 *     sets a process-wide tile override for sweeps.
 *   - Opaque handles (sm_map, sm_plan) are host objects created and destroyed by
 *     the library.  Descriptor structs are plain data owned by the caller and
 *     copied during the call.
 *   - Tensors are row-major.  Linear weights are [out_features, in_features]
 *     (the reduction dimension contiguous, Sec. 3.2.2).  All tensors of a call
 *     share the element type given by `dtype`.
 *   - Shapes that do not divide (H or W not a multiple of the window) return
 *     SM_ERR_SHAPE; there is no padding path.
 */
#ifndef SMARTMEM_H
#define SMARTMEM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SM_OK = 0, SM_ERR_INVALID_ARG = -1, SM_ERR_SHAPE = -2, SM_ERR_UNSUPPORTED = -3,
       SM_ERR_WORKSPACE = -4, SM_ERR_DEVICE = -5 };
enum { SM_F32 = 0, SM_BF16 = 1 };
enum { SM_ELIDED = 0, SM_EXPLICIT = 1 };
#define SM_MAX_RANK 8

const char* sm_last_error(void);
/* Version of this ABI (increments on incompatible change). */
int sm_abi_version(void);

/* ------------------------------------------------------------------------ */
/* Operator graph and layout planner (Sec. 3.1, 3.2; Tables 3, 5, 6)         */
/* ------------------------------------------------------------------------ */

/* Operator groups of Table 3: input layout dependent / independent x output
 * layout variable / fixed. */
enum { SM_ILD_VAR = 0, SM_ILI_VAR = 1, SM_ILD_FIX = 2, SM_ILI_FIX = 3 };
/* Pair actions of Table 5 and layout-search policies of Table 6. */
enum { SM_KEEP_BOTH = 0, SM_TRY_FUSE = 1, SM_ELIM_2ND = 2, SM_ELIM_1ST = 3, SM_ELIM_BOTH = 4 };
enum { SM_SEARCH_BOTH = 0, SM_SEARCH_FUSED = 1, SM_SEARCH_1ST = 2, SM_SEARCH_2ND = 3, SM_NO_SEARCH = 4 };
/* What became of an operator after planning. */
enum { SM_KEPT = 0, SM_FUSED = 1, SM_ELIMINATED_STORE = 2, SM_ELIMINATED_LOAD = 3, SM_MATERIALISED = 4 };

/* Operator kinds.  0..15 ILD&Variable, 16..31 ILD&Fixed, 32..47 ILI&Variable,
 * 48..63 ILI&Fixed.  The first four of each row are the paper's Table 3; the
 * others are classified by the definitions of Table 4. */
enum {
  SM_OP_CONV = 0, SM_OP_MATMUL = 1, SM_OP_LAYERNORM = 2, SM_OP_SOFTMAX = 3,
  SM_OP_GROUPNORM = 4, SM_OP_RMSNORM = 5, SM_OP_ATTENTION = 6, SM_OP_REDUCE = 7,
  SM_OP_RESHAPE = 16, SM_OP_TRANSPOSE = 17, SM_OP_DTOS = 18, SM_OP_STOD = 19,
  SM_OP_UNARY = 32, SM_OP_ADD = 33, SM_OP_MUL = 34, SM_OP_BIAS = 35, SM_OP_ROPE = 36,
  SM_OP_GATHER = 48, SM_OP_SLICE = 49, SM_OP_ROLL = 50, SM_OP_CONCAT = 51
};

typedef struct { int32_t rank; int64_t shape[SM_MAX_RANK]; int32_t dtype; } sm_tensor_desc;

/* One operator.  `in` are tensor ids (indices into the tensor array), `out` the
 * tensor it produces.  Operators must be given in topological order.
 * attr: TRANSPOSE attr[0..rank) = perm (output axis k is input axis perm[k]);
 *       ROLL attr = {axis, shift} (out[i] = in[(i - shift) mod n]);
 *       SLICE attr = {axis, start, stop, step}; RESHAPE none (shape of `out`);
 *       ILD&Variable kinds: attr[i] = reduction axis of operand i, -1 for none
 *       (Sec. 3.2.2 "reduction dimension"). */
typedef struct { int32_t kind; int32_t n_in; int32_t in[4]; int32_t out; int32_t n_attr; int64_t attr[16]; } sm_op_desc;

typedef struct sm_plan sm_plan;
typedef struct sm_map sm_map;

/* Table 3: group of an operator kind; SM_ERR_INVALID_ARG for an unknown kind. */
int sm_op_group(int kind, int* group);
/* Table 5 / Table 6 for a (first, second) pair of groups.  result_group is -1
 * for the N/A cells. */
int sm_pair_action(int first_group, int second_group, int* action);
int sm_pair_outcome(int first_group, int second_group, int* result_group, int* search);

/* Plans a producer-consumer operator graph: classifies every operator
 * (Table 3), merges Fixed-Fixed pairs, absorbs every run of Fixed operators
 * into the store of the preceding Variable operator or the load of the
 * following one (Table 5; write side when the run is the only reader of the
 * producer's tensor and is a bijection, Sec. 3.2.2; a run nothing reads is
 * stored by its producer as one more output), fuses ILI&Variable operators
 * pair by pair (consumers in graph order, latest producer first, never closing
 * a cycle) until only ILD&Variable operators survive, then selects the layout
 * of every stored tensor from its consumers' reduction dimensions with k
 * directly indexable dimensions (k = 1 on linear HBM; k = 2 reproduces the 2.5D
 * case).  Layout operators with several inputs (Concat) are not planned:
 * SM_ERR_UNSUPPORTED.  Host only.  *out is owned by the library until
 * sm_plan_destroy. */
int sm_layout_plan(const sm_tensor_desc* tensors, int n_tensors, const sm_op_desc* ops, int n_ops,
                   int k, sm_plan** out);
/* Per operator: group, the Table 5 action that decided it (-1 for a layout
 * operator that met no other operator), its status (SM_KEPT..),
 * the surviving operator that absorbed it (itself when kept, -1 when
 * materialised) and the group of the merged node (Table 6). Any out pointer
 * may be NULL. */
int sm_plan_op(const sm_plan*, int op, int* group, int* action, int* status, int* absorbed_by, int* node_group);
/* Per stored tensor: dimension order chosen (outermost first, length rank),
 * the reduction dimensions its consumers requested (up to SM_MAX_RANK, count in
 * *n_red) and the number of copies kept (> 1 when more than k are requested).
 * SM_ERR_INVALID_ARG if the tensor is never stored (eliminated view). */
int sm_plan_tensor(const sm_plan*, int tensor, int* dim_order, int* red_dims, int* n_red, int* n_copies);
/* Composed map seen by operand `operand` of surviving operator `consumer_op`
 * (view index -> element offset in the stored tensor).  *stored_tensor is the
 * tensor id the offsets refer to.  *borrowed is NULL when the operand is read
 * directly.  The map belongs to the plan. */
int sm_plan_load_map(const sm_plan*, int consumer_op, int operand, const sm_map** borrowed, int* stored_tensor);
/* Map applied by surviving operator `producer_op` when it stores its result:
 * natural output index -> element offset in the tensor it stores
 * (*stored_tensor, the output of the last absorbed operator).  NULL when the
 * result is stored as computed, or when the absorbed run is no bijection (a
 * graph output behind a Slice: *stored_tensor still names it).  A node that
 * stores several mapped tensors reports the first. */
int sm_plan_store_map(const sm_plan*, int producer_op, const sm_map** borrowed, int* stored_tensor);
void sm_plan_destroy(sm_plan*);

/* ------------------------------------------------------------------------ */
/* Index-map composer (Sec. 3.2.1: index comprehension and strength reduction) */
/* ------------------------------------------------------------------------ */

enum { SM_VIEW_RESHAPE = 0, SM_VIEW_PERMUTE = 1, SM_VIEW_ROLL = 2, SM_VIEW_SLICE = 3 };
/* RESHAPE: n = new rank, arg = new shape.  PERMUTE: n = rank, arg = perm.
 * ROLL: arg = {axis, shift}.  SLICE: arg = {axis, start, stop, step}, step >= 1. */
typedef struct { int32_t kind; int32_t n; int64_t arg[SM_MAX_RANK]; } sm_view_op;

/* Composes a chain of view operators applied to a contiguous row-major source
 * of shape `src` into one map: view multi-index -> source element offset, built
 * from identity / split (//, %) / merge (*, +) index dependencies and
 * simplified with exact strength-reduction rules. */
int sm_map_create(const sm_tensor_desc* src, const sm_view_op* chain, int n, sm_map** out);
/* outer is a map whose *source shape* equals inner's view shape; the result
 * maps outer's view index to inner's source offset. Not needed for chains
 * built in one go; provided for maps planned separately. */
int sm_map_compose(const sm_map* inner, const sm_map* outer, sm_map** out);
int sm_map_rank(const sm_map*);
int sm_map_shape(const sm_map*, int64_t* shape /* SM_MAX_RANK */);
int64_t sm_map_numel(const sm_map*);
/* Number of // and % operations left in the simplified map, and in the map
 * before simplification (what strength reduction removed). */
int sm_map_cost(const sm_map*, int* n_divmod, int* n_divmod_unsimplified);
/* offsets[o] = source element offset of view element o (row-major over the
 * view shape), o in [0, n); n must equal sm_map_numel.  Host pointer. */
int sm_map_eval_host(const sm_map*, int64_t* offsets, int64_t n);
/* 1 if the map is affine (no // or % left): then offset = base + sum stride[k]*i[k]. */
int sm_map_affine(const sm_map*, int64_t* base, int64_t* strides /* SM_MAX_RANK */);
/* Writes the simplified offset expression as text ("i0, i1, ..." are the view
 * indices) into buf (n bytes, truncated). */
int sm_map_describe(const sm_map*, char* buf, int n);
void sm_map_destroy(sm_map*);

/* The layout copy the paper removes (Sec. 2.2 "explicit" transformations;
 * Table 1 column "Exp."), kept as the materialised form of a composed map:
 * dst[o] = src[map(o)] for every view element o; dst is contiguous with the
 * view's shape.  on_device = 0: host pointers, executed on the host;
 * on_device = 1: device pointers, one HIP kernel on `stream`.  This is the
 * materialised form of an eliminated transformation (a test instrument and the
 * copy kernel of the explicit baseline). */
int sm_gather_mapped(const sm_map*, const void* src, void* dst, int dtype, int on_device, void* stream);

/* ------------------------------------------------------------------------ */
/* Single operators with mapped operands (device pointers)                    */
/* ------------------------------------------------------------------------ */

/* An ILD & Variable operator of Table 3 (LayerNorm) whose store takes a
 * composed map ("Eliminate 2nd", Table 5; Sec. 3.2.1).
 * y = LayerNorm(x) over the last dimension C of x [rows, C] (fp32 statistics,
 * biased variance).  rms != 0: RMSNorm (no mean subtraction, beta ignored).
 * store_map (nullable): a map with view shape [rows, C] (or any shape with
 * rows*C elements whose last dimension is C) giving the offset in y of each
 * natural output element; its last dimension must be contiguous. */
int sm_norm(const void* x, const void* gamma, const void* beta, void* y, int64_t rows, int C, float eps,
            int rms, int dtype, const sm_map* store_map, void* stream);
/* ILD & Variable by the definitions of Table 4 (the InstanceNorm example of
 * Fig. 1(b) is the same family); its output layout follows its consumer's
 * reduction dimension (Sec. 3.2.2).
 * GroupNorm over x NCHW [B, C, H, W] with G groups.  tokens_out = 0: y is NCHW;
 * tokens_out = 1: y is written token-major [B, H*W, C] (the layout a following
 * MatMul over C prefers).  stats_scratch (nullable): device memory for 2 * B * G
 * floats; with it the work runs as two fully parallel kernels (statistics, then
 * apply with whole-row stores) instead of one workgroup per (image, group). */
int sm_groupnorm(const void* x, const void* gamma, const void* beta, void* y, int B, int C, int HW, int G,
                 float eps, int tokens_out, int dtype, void* stats_scratch, void* stream);

/* Epilogue of sm_linear, applied in this order to acc = A.W^T:
 * +bias[n]; activation; RoPE; *gate; +residual. */
enum { SM_ACT_NONE = 0, SM_ACT_GELU = 1, SM_ACT_SWIGLU = 2, SM_ACT_GEGLU = 3 };
typedef struct {
  int64_t M; int32_t N, K;      /* C[M, N] = A[M, K] . W[N, K]^T */
  int32_t dtype;
  int32_t act;                  /* SM_ACT_*; SWIGLU / GEGLU: W has 2N' rows, output has N' = N/2 columns:
                                   SWIGLU out = silu(acc[:, j]) * acc[:, N' + j]; GEGLU out = acc[:, j] * gelu(acc[:, N' + j]) */
  int32_t rope_cols;            /* > 0: columns [0, rope_cols) are heads of size rope_dim rotated by RoPE (half-split pairs) */
  int32_t rope_dim; int32_t rope_seq;   /* position of row r is r mod rope_seq */
  float rope_base;
  int32_t c_transposed;         /* 1: C is stored column-major per batch of c_batch_rows rows:
                                   offset = (r / c_batch_rows) * N * c_batch_rows + n * c_batch_rows + r % c_batch_rows
                                   (NCHW store); residual is read the same way */
  int64_t c_batch_rows;
  int32_t norm;                 /* 0 none; 1 LayerNorm, 2 RMSNorm over K of every row of A, applied while A is loaded: the norm
                                   that precedes the Linear folded into it (activation none or GELU only, no RoPE).
                                   A's rows are normalised in fp32 and rounded to the element type before the product,
                                   exactly as a separate sm_norm would have stored them */
  float norm_eps;
  const void* norm_gamma;       /* [K], device; required when norm != 0 */
  const void* norm_beta;        /* [K], device; nullable (ignored by RMSNorm) */
  int32_t w_packed;             /* 1: W was rewritten by sm_linear_pack (see there); selects the kernel that streams the
                                   weight into registers */
} sm_linear_desc;
/* a_map / c_map (nullable): maps with view shape [M, K] / natural output shape
 * [M, Nout] whose last dimension is contiguous: row r of A is read at
 * a_map(r, 0); row r of the result is written at c_map(r, 0) and the residual
 * is read at the same offset.  bias, residual nullable.
 * An a_map whose last dimension is contiguous only in granules of 4 (an unfold)
 * or not at all (a transposed operand) is accepted when its offset separates
 * into a row part and a column part; the second case loads one element at a
 * time: the consumer-side ("read") folding that Sec. 3.2.2 advises against,
 * kept so that it can be measured against the producer-side fold (c_transposed). */
int sm_linear(const sm_linear_desc*, const void* A, const void* W, const void* bias, const void* residual,
              void* C, const sm_map* a_map, const sm_map* c_map, void* stream);
/* Weight layout for short reduction dimensions (Sec. 3.2.2's rule, the producer writes the layout its consumer reads
 * best, applied to a constant): for bf16, K in {128, 256, 384, 512} and N a multiple of 32 (sm_linear_pack_supported),
 * sm_linear_pack rewrites W [N, K] into `packed` (device, N * K elements, 16-byte aligned, caller-owned) in the order
 * of the matrix-core operand fragments.  sm_linear with w_packed = 1 and that buffer as W then runs a kernel in which
 * a workgroup keeps 32 rows of A (64 at K = 512) in LDS for all N outputs and the weight streams from L2 straight into registers: no
 * K-loop barriers, and a LayerNorm (norm = 1, beta required) costs one pass over the resident tile.  It pays most with
 * a folded LayerNorm and a short K against many rows (no norm kernel, no K-loop barriers).  Restrictions with w_packed: activation none or
 * GELU, no RoPE, no transposed store, row maps only (a map that splits columns returns SM_ERR_UNSUPPORTED). */
int sm_linear_pack_supported(int N, int K, int dtype);
int sm_linear_pack(const void* W, int N, int K, int dtype, void* packed, void* stream);

/* Fused two-layer MLP  Y = residual + gelu(norm(X) . W1^T + b1) . W2^T + b2  in one kernel, the hidden activation kept
 * in registers (an extension next to the paper's path: the paper keeps two MatMuls apart, Table 5; here the largest
 * intermediate of a transformer block, [M, hidden], never reaches memory).  bf16 only.
 * The kernel reads the two weight matrices in the order its matrix-core operands want them (Sec. 3.2.2's rule that
 * the producer writes the layout the consumer reads best, applied to constants): sm_mlp_pack writes W1 [hidden, C]
 * and W2 [C, hidden] (row-major, device) into `packed` (device, 2 * hidden * C elements, 16-byte aligned, owned by
 * the caller); call it once per weight pair, and again after the weights change.
 * sm_mlp_fused: X [M, C], b1 [hidden], b2 [C], residual (nullable) and Y [M, C] are device pointers, 16-byte
 * aligned.  norm = 1: LayerNorm over C of every row of X first (gamma, beta [C], device; rounded to bf16 as sm_norm
 * would store it).  The hidden activation is rounded to bf16 before the second product, as the two-kernel path
 * stores it.  x_map / y_map (nullable): row maps as in sm_linear (the residual is read through y_map).
 * sm_mlp_fused_supported: 1 if a shape has a kernel (bf16; C in {128, 256, 384} with hidden a multiple of 32 up to
 * 16384: 32-token tiles; C = 512 with hidden a multiple of 256: 64-token tiles, the MLP alone, i.e. no proj_packed);
 * other shapes return SM_ERR_UNSUPPORTED from both calls and nothing is enqueued. */
typedef struct {
  int64_t M; int32_t C, hidden, dtype;
  int32_t norm; float norm_eps;
  const void* norm_gamma; const void* norm_beta;
  /* proj_packed != null: the Linear in front of the MLP's residual stream runs in the same kernel (a transformer
   * block's attention output projection): x1 = X . Wproj^T + proj_bias + proj_residual, then
   * Y = x1 + MLP(norm(x1)); x1 (rounded to bf16) never reaches memory.  proj_packed = sm_linear_pack of
   * Wproj [C, C]; proj_bias [C]; proj_residual [M, C] is read through y_map like Y is written; the `residual`
   * argument is ignored.  Needs three token tiles in LDS: sm_mlp_proj_supported says whether a shape fits. */
  const void* proj_packed; const void* proj_bias; const void* proj_residual;
} sm_mlp_desc;
int sm_mlp_fused_supported(int C, int hidden, int dtype);
int sm_mlp_proj_supported(int C, int hidden, int dtype);
int sm_mlp_pack(const void* W1, const void* W2, int C, int hidden, int dtype, void* packed, void* stream);
int sm_mlp_fused(const sm_mlp_desc*, const void* X, const void* packed, const void* b1, const void* b2,
                 const void* residual, void* Y, const sm_map* x_map, const sm_map* y_map, void* stream);

/* MatMul + Softmax + MatMul of Table 3 as one ILD & Variable operator whose loads
 * and store take the head split / merge maps (Sec. 3.2.1; the paper keeps the
 * three apart and names tiled attention as complementary, Sec. 6).
 * Fused attention O = softmax(scale * Q K^T + bias + mask) V per (batch, head).
 * Q, K, V, O are 4-D strided views [nb, heads, n, d] (element strides, innermost
 * stride 1) so that head split / merge permutes are address arithmetic.
 * kind: SM_ATT_FULL, SM_ATT_CAUSAL (key j visible to query i iff j <= i), or
 * SM_ATT_WINDOW (Swin: n = window*window tokens, rel-pos bias gathered from
 * rpb_table [(2w-1)^2, heads], shifted-window mask computed from the window's
 * position on the H x W grid when shift > 0; masked logits get -100), or
 * SM_ATT_STRIPE (cross-shaped windows, CSwin: a batch entry is one stripe of an
 * image's token grid, whose n tokens lie in n / run runs of `run` adjacent
 * tokens; bf16, d <= 32, nq == nk): batch entry b is stripe b % stripes of image
 * b / stripes and starts (b / stripes) * stride[0] + (b % stripes) * stripe[0]
 * elements into the operand; its token s lies (s / run) * stripe[1] +
 * (s % run) * stride[2] elements further on. */
enum { SM_ATT_FULL = 0, SM_ATT_CAUSAL = 1, SM_ATT_WINDOW = 2, SM_ATT_STRIPE = 3 };
typedef struct {
  int32_t kind, dtype;
  int32_t nb, heads, nq, nk, d;
  float scale;
  int64_t q_stride[3], k_stride[3], v_stride[3], o_stride[3];   /* batch, head, token */
  int32_t window, shift, H, W;      /* SM_ATT_WINDOW only; batch index = (image, wy, wx) row-major */
  int32_t stripes, run;             /* SM_ATT_STRIPE only: stripes per image, adjacent tokens per run */
  int64_t q_stripe[2], k_stripe[2], v_stripe[2], o_stripe[2];   /* SM_ATT_STRIPE only: element strides (stripe, run) */
  int32_t accumulate, reserved;     /* accumulate != 0: O += the result (O is read; bf16 full / causal / stripe kinds with scale > 0) */
} sm_attention_desc;
int sm_attention(const sm_attention_desc*, const void* q, const void* k, const void* v, void* o,
                 const void* rpb_table, void* stream);

/* ------------------------------------------------------------------------ */
/* Block and chain executors                                                  */
/* ------------------------------------------------------------------------ */

/* The Swin block of Table 7 executed as Sec. 3.2 plans it: the executor writes
 * the block down as an operator graph, calls sm_layout_plan, and launches one
 * kernel per surviving ILD & Variable operator with the planned load / store
 * maps (SM_ELIDED), or the explicit chain the paper starts from (SM_EXPLICIT,
 * Table 1 "Exp.").  ws: sm_swin_block_workspace_bytes(cfg, mode) bytes.
 * One Swin block on x [B, H*W, C] -> y [B, H*W, C]:
 * LayerNorm -> (roll, window partition) -> QKV Linear -> window attention ->
 * proj Linear -> (reverse, roll back) -> +x -> LayerNorm -> MLP (GELU) -> +.
 * SM_ELIDED: 7 kernels (fewer where a norm is folded into the next Linear or the MLP is fused), the layout transformations are folded into their
 * neighbours' addressing as planned by sm_layout_plan.  SM_EXPLICIT: the same
 * 7 kernels with identity maps plus one copy kernel per transformation that
 * moves data (the baseline the paper's Table 1 calls explicit). */
typedef struct { int32_t B, H, W, C, heads, window, shift, mlp_ratio, dtype; float eps; } sm_swin_cfg;
typedef struct {
  const void *ln1_g, *ln1_b, *wqkv, *bqkv, *rpb_table, *wproj, *bproj,
             *ln2_g, *ln2_b, *w1, *b1, *w2, *b2;
  const void* mlp_packed;       /* nullable: sm_mlp_pack(w1, w2); with it (and a shape sm_mlp_fused_supported accepts)
                                   LayerNorm-2, FC1 + GELU and FC2 + residual run as the one fused MLP kernel */
  const void* proj_packed;      /* nullable: sm_linear_pack(wproj); with it and mlp_packed (and a shape
                                   sm_mlp_proj_supported accepts), SM_ELIDED also runs the output projection, its
                                   window-reverse store and the first residual inside that kernel.  SM_EXPLICIT cannot:
                                   its materialised reverse copy sits between the projection and the residual */
  const void* qkv_packed;       /* nullable: sm_linear_pack(wqkv); SM_ELIDED only.  LayerNorm-1 and the QKV Linear then
                                   run as one packed-weight kernel; in sm_run_chain, inside a stage, when the previous
                                   block runs the fused projection + MLP kernel, that kernel computes them instead and
                                   this block starts at attention */
} sm_swin_weights;
size_t sm_swin_block_workspace_bytes(const sm_swin_cfg*, int mode);
int sm_swin_block(const sm_swin_cfg*, const sm_swin_weights*, const void* x, void* y,
                  void* ws, size_t ws_bytes, int mode, void* stream);

/* For callers that cannot allocate (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): sm_swin_block with the library's own
 * workspace, a static device array of SM_STATIC_WS_BYTES (one copy per GPU the
 * library runs on, held until the process ends).  Same arguments, results and
 * errors as sm_swin_block without ws / ws_bytes; a block that needs more than
 * the static buffer returns SM_ERR_WORKSPACE and launches nothing.  Calls no
 * allocating routine.  All calls on one GPU share the buffer: calls that overlap
 * on one GPU (two streams, two threads) race; calls in stream order do not, and
 * nothing in the buffer has to be cleared between them. */
#define SM_STATIC_WS_BYTES (32u << 20)
size_t sm_swin_block_static_max_bytes(void);
int sm_swin_block_static(const sm_swin_cfg*, const sm_swin_weights*, const void* x, void* y, int mode, void* stream);

/* The global-attention blocks of Table 7 (a Pythia / Llama-style decoder layer,
 * an SD-UNet spatial transformer) planned and executed the same way (Sec. 3.2):
 * head split / merge permutes and the NCHW <-> token rearrangement become load /
 * store maps of the attention and Linear kernels.
 * Llama-style decoder layer (prefill) or diffusion-UNet spatial-transformer
 * block.  weights: array of device pointers in this order
 *   SM_ATTN_LLAMA (6): rms1_g, wqkv [3E, E] (rows q | k | v), wo, rms2_g,
 *                      w_gate_up [2F, E] (rows gate | up), wdown [E, F]
 *   SM_ATTN_SD (23): gn_g, gn_b, win, bin, ln1_g, ln1_b, a1_wqkv [3C, C], a1_wo, a1_bo,
 *                    ln2_g, ln2_b, a2_wq, a2_wkv [2C, Dc], a2_wo, a2_bo, ln3_g, ln3_b,
 *                    ff_w1 [2F, C], ff_b1, ff_w2, ff_b2, wout, bout
 *   SM_ATTN_VIT (12): a ViT encoder block (pre-norm, global attention over all S tokens, GELU MLP of width F):
 *                     ln1_g, ln1_b, wqkv [3E, E], bqkv, wo, bo, ln2_g, ln2_b, w1 [F, E], b1, w2 [E, F], b2
 * x: LLAMA, VIT [B, S, E]; SD NCHW [B, C, Hs, Ws]; context: SD only, [B, Sc, Dc]. */
enum { SM_ATTN_LLAMA = 0, SM_ATTN_SD = 1, SM_ATTN_VIT = 2 };
typedef struct {
  int32_t kind, dtype;
  int32_t B, S, E, heads, F;          /* LLAMA: S tokens, E hidden; SD: S = Hs*Ws, E = C channels */
  int32_t Hs, Ws, groups, Sc, Dc;     /* SD only */
  float rope_base, eps_norm, eps_gn;
} sm_attn_cfg;
size_t sm_attn_block_workspace_bytes(const sm_attn_cfg*, int mode);
int sm_attn_block(const sm_attn_cfg*, const void* const* weights, const void* x, const void* context,
                  void* y, void* ws, size_t ws_bytes, int mode, void* stream);

/* A GPT-NeoX / Pythia-style layer at a decode step (Table 7's decoder-only model at one new token per sequence:
 * every Linear is a matrix-vector product bound by its weight stream, so a materialised layout operator costs
 * relatively most; Sec. 3.2.1 elimination, Sec. 3.2.2 producer-writes-the-consumer's-layout).  bf16 only.
 *   y = x + dense(attention(q, [K; k], [V; v])) + W2 gelu(W1 LN2(x) + b1) + b2,   [q | k | v] = Wqkv LN1(x) + bqkv
 * with Wqkv's 3E output features ordered [head][q | k | v][d], the rotary embedding (half-split pairs (i, i + rot/2),
 * theta_i = rope_base^(-2i/rot), position L) on the first `rot` features of every query and key head, softmax scale
 * d^-1/2 over the L cached tokens and the new one, erf GELU, LayerNorm eps `eps`.
 * x, y: device [B, E].  Weights: device pointers; the four matrices in the fragment order sm_linear_pack writes
 * (wqkv_p from [3E, E], wdense_p from [E, E], w1_p from [F, E], w2_p from [E, F]); vectors as stored.
 * k_cache, v_cache: device [B, heads, cache_pitch, d], tokens 0 .. L-1 valid (keys already rotated).
 *   SM_ELIDED: cache_pitch > L; the new key / value rows are written at token L of k_cache / v_cache by the
 *     Linear that produces them (the Concat is its store address), the query is read in place from that Linear's
 *     result, the attention output is stored head-merged; k_out, v_out must be NULL.  Three kernels.
 *   SM_EXPLICIT: every Slice / Permute / Concat / Reshape of the exported graph that moves data is a copy kernel:
 *     k_out, v_out: device [B, heads, L + 1, d] receive the grown caches (k_cache / v_cache are only read).
 * Limits: B <= 32, E a multiple of 64 (<= 8192), d in {64, 128, 256}, F a multiple of 64, rot in {0, 32, 64}.
 * Workspace from sm_decode_step_workspace_bytes; nothing in it has to survive between calls.  Calls on one stream
 * are ordered; calls that share a workspace on different streams race. */
typedef struct {
  int32_t dtype, B, E, heads, F, rot, L, cache_pitch;
  float rope_base, eps;
} sm_decode_cfg;
typedef struct {
  const void *ln1_g, *ln1_b, *wqkv_p, *bqkv, *wdense_p, *bdense, *ln2_g, *ln2_b, *w1_p, *b1, *w2_p, *b2;
} sm_decode_weights;
/* W [N, K] (bf16, N a multiple of 32, K of 16) rewritten into `packed` (device, N * K elements, caller-owned) in the
 * fragment order of sm_linear_pack, without that call's limits on K: the layout sm_decode_step reads. */
int sm_decode_pack(const void* W, int N, int K, int dtype, void* packed, void* stream);
size_t sm_decode_step_workspace_bytes(const sm_decode_cfg*, int mode);
int sm_decode_step(const sm_decode_cfg*, const sm_decode_weights*, const void* x, void* k_cache, void* v_cache,
                   void* y, void* k_out, void* v_out, void* ws, size_t ws_bytes, int mode, void* stream);

/* Cross-shaped window self-attention of the CSwin Transformer (Table 1 counts its
 * Reshape / Transpose operators, Table 7 evaluates it): the stripe partition,
 * head split, head merge and stripe merge around the two attentions are Reshape /
 * Transpose / Slice runs that the planner turns into the attention kernel's load
 * and store addresses (Sec. 3.2.1).
 * qkv [B, H*W, 3C] (device; columns [q | k | v], each heads x d with d = C / heads)
 * as the fused Linear leaves it; out [B, H*W, C] (device).  Heads [0, heads/2)
 * attend inside vertical stripes (H x sw grid positions), the others inside
 * horizontal stripes (sw x W); scale d^-1/2.  lepe_w [C, 3, 3], lepe_b [C]
 * (device, bf16; both null: none): the locally-enhanced positional encoding,
 * a depth-wise 3 x 3 cross-correlation of each half's values inside their own
 * stripe (zero beyond the stripe's border), added to that half's attention
 * output; channel order as in out.
 *   SM_ELIDED: two attentions that read qkv in place and store into their half
 *     of out's channels (the Concat of the halves has two inputs and is not
 *     planned: it is applied as the store address, by hand); one launch holds
 *     both when H == W (the halves then have one shape), else two.  With the
 *     encoding: one convolution kernel first, which reads the values of both
 *     halves in place and writes out, to which the attentions then add.
 *   SM_EXPLICIT: per half one copy kernel for the Slice + partition + head split
 *     of q, k, v, the attention on contiguous operands, one copy for head merge +
 *     stripe merge, then one Concat kernel: 5 copies around the same 2 kernels
 *     (with the encoding 9 around 4: the values as stripe images and the
 *     encoding's head split are copies too).
 * Limits: bf16; heads even; d a multiple of 8, at most 32; H and W multiples of
 * sw; a stripe of at most 65536 tokens.  ws: device workspace of at least
 * sm_cswin_attention_workspace_bytes(cfg, mode) bytes, owned by the caller.
 * Nothing is allocated; SM_ERR_* with a message otherwise. */
typedef struct { int32_t dtype, B, H, W, C, heads, sw; } sm_cswin_cfg;
size_t sm_cswin_attention_workspace_bytes(const sm_cswin_cfg*, int mode);
int sm_cswin_attention(const sm_cswin_cfg*, const void* qkv, const void* lepe_w, const void* lepe_b, void* out,
                       void* ws, size_t ws_bytes, int mode, void* stream);

/* One CSwin block (Tables 1, 7): y = x1 + MLP(LayerNorm(x1)), x1 = x + proj(cross-shaped window attention of the fused
 * q | k | v Linear of LayerNorm(x)); x, y [B, H*W, C] (device, bf16).  Every layout operator of the block sits inside
 * the attention operator above (mode selects its elided or explicit form); around it the block is LayerNorm + Linear
 * (one kernel: the norm folded into the Linear's load, or the packed-weight Linear when qkv_packed is given), and the
 * output Linear + residual + LayerNorm + MLP + residual (one kernel when mlp_packed and proj_packed are given and
 * sm_mlp_proj_supported(C, mlp_ratio * C), else the Linears one by one).  Weights as in sm_swin_weights ([out, in],
 * packed forms from sm_mlp_pack / sm_linear_pack, optional); lepe_w [C, 3, 3], lepe_b [C].  Limits as for
 * sm_cswin_attention, C a multiple of 16.  Workspace from sm_cswin_block_workspace_bytes, caller-owned; nothing is
 * allocated. */
typedef struct { int32_t dtype, B, H, W, C, heads, sw, mlp_ratio; float eps; } sm_cswin_block_cfg;
typedef struct {
  const void *ln1_g, *ln1_b, *wqkv, *bqkv, *lepe_w, *lepe_b, *wproj, *bproj, *ln2_g, *ln2_b, *w1, *b1, *w2, *b2;
  const void *mlp_packed, *proj_packed, *qkv_packed;
} sm_cswin_weights;
size_t sm_cswin_block_workspace_bytes(const sm_cswin_block_cfg*, int mode);
int sm_cswin_block(const sm_cswin_block_cfg*, const sm_cswin_weights*, const void* x, void* y, void* ws, size_t ws_bytes,
                   int mode, void* stream);

/* A whole producer-consumer chain (Sec. 3.2: elimination and fusion alternate
 * over rounds, so removed layout operators leave compute operators adjacent):
 * A Swin chain: optional patch embedding (NCHW image, patch x patch stride
 * patch unfold folded into the Linear's A addressing), stages of blocks
 * (block k of a stage shifts by window/2 when k is odd and the stage is larger
 * than one window), patch merging between stages (2x2 gather folded into the
 * LayerNorm's load), optional head (LayerNorm, mean over tokens, Linear).
 * weights: device pointers in forward order: embed {w, b, ln_g, ln_b} if
 * has_embed; per stage: per block the 16 pointers of sm_swin_weights in
 * declaration order (mlp_packed, proj_packed and qkv_packed may be null), then (between stages) merge {ln_g, ln_b, w}; head
 * {ln_g, ln_b, w, b} if has_head.
 * x: image [B, in_ch, img, img] if has_embed else tokens [B, H0*W0, C0].
 * y: logits [B, n_cls] if has_head else tokens of the last stage.
 * y_feat (nullable): the normalised feature map [B, L_last, C_last] before pooling.
 * Inside a stage, SM_ELIDED, with a block's three packed weights given, a block costs two kernels: window attention,
 * and one kernel for projection + residual + LayerNorm-2 + MLP + residual that also computes the next block's
 * LayerNorm-1 and QKV Linear (stored through the composition of this block's window-reverse map and the next block's
 * partition map); the first block of a stage runs its own LayerNorm-1 and QKV. */
typedef struct { int32_t C, heads, depth, H, W; } sm_stage_desc;
typedef struct {
  int32_t B, dtype, window, mlp_ratio;
  int32_t has_embed, in_ch, img, patch;
  int32_t n_stages; sm_stage_desc stages[4];
  int32_t has_head, n_cls;
  float eps;
} sm_chain_desc;
size_t sm_run_chain_workspace_bytes(const sm_chain_desc*, int mode);
int sm_run_chain(const sm_chain_desc*, const void* const* weights, int n_weights, const void* x,
                 void* y, void* y_feat, void* ws, size_t ws_bytes, int mode, void* stream);

/* The multi-consumer example of the paper's global layout selection (Sec. 3.2.2, Fig. 4; memory cost of redundant
 * copies: Sec. 4.6), executed: T = A . W^T [D2*D3, D1] -> Transpose -> Reshape [D1, D2, D3] -> three consumers,
 *   reduce   [D1, D2]       = sum over D3,
 *   reduce_p [D2, D3]       = sum over D1,
 *   conv     [D1, D2, Cout] = contraction over D3 with wconv [Cout, D3].
 * The graph is planned with sm_layout_plan and k directly indexable dimensions.  SM_ELIDED: Transpose and Reshape
 * are eliminated into the MatMul's store; the consumers request two reduction dimensions, so with k = 1 the MatMul
 * keeps two copies of its result (one epilogue, two stores), each consumer reading the one whose innermost
 * dimension is its own; with k = 2 a single layout serves all three (Reduce' then reads with a stride on linear
 * memory).  SM_EXPLICIT: the Transpose runs as a copy kernel.  a [D2*D3, Kin], w [D1, Kin], wconv [Cout, D3]; device
 * pointers; Kin, D1, D3 multiples of the 16-byte vector.  sm_fanout_graph_plan reports what the planner decided and
 * what one redundant copy costs in bytes. */
typedef struct { int32_t dtype, D1, D2, D3, Kin, Cout, k; } sm_fanout_cfg;
int sm_fanout_graph_plan(const sm_fanout_cfg*, int* n_copies, int* red_dims /* 2 */, int* n_red, size_t* copy_bytes);
size_t sm_fanout_graph_workspace_bytes(const sm_fanout_cfg*, int mode);
int sm_fanout_graph(const sm_fanout_cfg*, const void* a, const void* w, const void* wconv, void* reduce_out,
                    void* reduce_p_out, void* conv_out, void* ws, size_t ws_bytes, int mode, void* stream);

/* Number of kernels the last sm_swin_block / sm_attn_block / sm_run_chain call
 * of this thread enqueued, split into compute and copy kernels. */
int sm_last_launch_counts(int* n_compute, int* n_copy);

/* Per-kernel timing for benchmarks.  sm_timing_enable(1) clears earlier records and makes every
 * kernel launch of this library record a HIP event before and after itself on its stream (a small
 * perturbation: do not enable it inside a region timed as a whole); sm_timing_enable(0) stops and
 * clears.  sm_timing_report waits for the recorded events and writes one line per kernel label,
 * "label<TAB>launches<TAB>total_ms", into buf (host pointer, n bytes). */
int sm_timing_enable(int on);
int sm_timing_report(char* buf, int n);
/* the labels of the launches recorded since sm_timing_enable(1), in launch order, one per line (host buffer; a label
 * stands for one kernel, sm_groupnorm's two-kernel form for two): lets a profiler's dispatch list be matched to them */
int sm_timing_sequence(char* buf, int n);
/* Launches n (1..1024) empty kernels on `stream`, each recorded like any other launch under the label
 * "empty_kernel" (only while timing is enabled): their average is what an event pair measures on top of a
 * kernel's own execution time (dispatch and completion), to be subtracted when comparing with a profiler. */
int sm_timing_calibrate(int n, void* stream);

/* The tuner (Sec. 3.3 "Other optimizations": the paper tunes block dimensions, unrolling and tiling with a genetic
 * search; this kernel's space is small enough to walk completely).  Times every (tile height x pipeline stages)
 * variant of the tiled Linear on the caller's operands (device pointers as for sm_linear, identity maps), `iters`
 * launches each between two HIP events on `stream`, and remembers the fastest for the shape (M, N, K, dtype,
 * epilogue): every later sm_linear / executor launch of that shape in this process uses it.  A set-up call like
 * sm_linear_pack, and unlike the other entry points it creates events and SYNCHRONISES with the stream; C is
 * overwritten with the Linear's result.  *tile_rows = *stages = 0: the built-in choice won (a variant has to be 3 %
 * faster) or the shape has a single variant (fp32, K not a multiple of 64).  sm_linear_autotune_clear forgets all. */
int sm_linear_autotune(const sm_linear_desc*, const void* A, const void* W, const void* bias, const void* residual,
                       void* C, int iters, void* stream, int* tile_rows, int* stages, float* best_us, float* default_us);
void sm_linear_autotune_clear(void);

/* Tuning hook for benchmarks: overrides the tile and pipeline choice of the bf16 Linear kernel for the calling
 * process.  tile_rows: 0 (automatic), 64, 128 or 256 output rows per workgroup; stages: 0 (automatic) or 2..4
 * K-tiles resident in LDS.  Returns SM_ERR_INVALID_ARG for other values.  Results do not depend on the choice. */
int sm_gemm_tuning(int tile_rows, int stages);

#ifdef __cplusplus
}
#endif
#endif
