/*
 * ecospa.h - C ABI of the MI355X (gfx950) library for EcoSpa's coupled structured
 * sparsification hot path: score -> select top-k -> compact -> reduced forward/backward.
 *
 * Notation follows the paper's Appendix A.1: a coupled pair is A in R^{m x n} with columns
 * a_j and B in R^{n x p} with rows b_j^T, sharing the inner dimension n; A B = sum_j a_j b_j^T.
 * Matrices are STORED in the Linear-layer layout W[out_features, in_features], row-major,
 * y = x W^T.  Hence a_j is stored ROW j of the first member (W_q, W_v, W_in, W_gate (.) W_up)
 * and b_j is stored COLUMN j of the second member (W_o, W_out, W_down); for the QK pair
 * (Eq. 4: W_i^Q W_i^K^T) b_j is stored ROW j of W_k.
 *
 * General rules for every entry point
 *   - Pointers are DEVICE pointers unless the comment says "host".  The caller owns every
 *     buffer; the library never allocates or frees device memory.  Scratch memory comes from
 *     the workspace the caller attaches with ecospa_set_workspace().
 *   - Calls are asynchronous on the context's HIP stream and never synchronise with the host.
 *   - Return value: ECOSPA_OK (0) or an error code > 0.  Arguments are validated on the host
 *     before any launch; on a validation error nothing is launched and no output is written.
 *   - Results are deterministic: no floating-point atomics, fixed reduction orders.
 *   - dtype is the storage type of weights/activations (ECOSPA_F32 or ECOSPA_BF16); all
 *     accumulation is fp32; scores are always fp32; indices are int32.
 *   - Leading dimensions (ld*) are in elements.  Buffers used by the reduced forward/backward
 *     must be 16-byte aligned with leading dimensions that are multiples of 8 elements.
 */
#ifndef ECOSPA_H
#define ECOSPA_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ECOSPA_OK = 0, ECOSPA_ERR_NULL = 1, ECOSPA_ERR_SHAPE = 2, ECOSPA_ERR_DTYPE = 3, ECOSPA_ERR_K = 4,
       ECOSPA_ERR_INDEX = 5, ECOSPA_ERR_WORKSPACE = 6, ECOSPA_ERR_ALIGN = 7, ECOSPA_ERR_HIP = 8 };
enum { ECOSPA_F32 = 0, ECOSPA_BF16 = 1 };
enum { ECOSPA_PAIR_QK = 0, ECOSPA_PAIR_VO = 1, ECOSPA_PAIR_FFN = 2, ECOSPA_PAIR_FFN_GATED = 3 };
enum { ECOSPA_BLOCK_ATTN = 0, ECOSPA_BLOCK_FFN = 1 };
enum { ECOSPA_ACT_GELU_ERF = 0, ECOSPA_ACT_GELU_TANH = 1, ECOSPA_ACT_SWIGLU = 2 };

typedef struct ecospa_ctx ecospa_ctx; /* host object */

/* Create a context bound to a HIP stream (hipStream_t passed as void*; NULL = default stream)
 * on the current device.  *out is a host object released by ecospa_destroy(). */
int ecospa_create(ecospa_ctx** out, void* hip_stream);
void ecospa_destroy(ecospa_ctx* ctx);
/* Attach caller-owned device scratch memory (256-byte aligned).  Entry points that need more
 * than `bytes` return ECOSPA_ERR_WORKSPACE.  The contents are clobbered by every call. */
int ecospa_set_workspace(ecospa_ctx* ctx, void* dev, size_t bytes);
/* Static, human-readable name of a status code. */
const char* ecospa_status_string(int code);
/* Text of the last HIP error seen by this context ("" if none); host string owned by ctx. */
const char* ecospa_last_error(const ecospa_ctx* ctx);

/* Measurement aid: time every launch of the bf16 MFMA contraction kernel with a pair of HIP events
 * recorded on the context's own stream.  enable != 0 starts a new window (at most 4096 launches
 * are kept); ecospa_profile_gemm_read waits for the recorded events and returns the number of
 * launches, the sum of their durations in ms and the sum of their 2*M*N*K flops (host pointers).
 * The events add a few microseconds per launch, so time throughput with profiling off. */
int ecospa_profile_gemm(ecospa_ctx* ctx, int enable);
int ecospa_profile_gemm_read(ecospa_ctx* ctx, int* launches, double* total_ms, double* total_flop);

/* Measurement aid: what a plain kernel reaches on this GPU's memory, the ceiling the HBM-bound steps (score: read
 * only; compaction: read and write) are priced against.  mode 0: `bytes` bytes of src are read once with 16-byte
 * loads and nothing is written (dst: at least 4 writable bytes, left as they are for any ordinary buffer content);
 * mode 1: src is copied to dst.  bytes a multiple of 16, pointers 16-byte aligned (dst in mode 0: 4-byte).
 * Errors: ERR_NULL, ERR_SHAPE (mode, bytes), ERR_ALIGN. */
int ecospa_hbm_probe(ecospa_ctx* ctx, const void* src, void* dst, size_t bytes, int mode);

/* Measurement aid: what the matrix units alone sustain on this GPU.  256 workgroups of four wavefronts (one per SIMD of
 * every compute unit) each issue `iters` rounds of 16 independent bf16 32x32x16 MFMAs on operand bits taken from src
 * (64 KiB, e.g. normally distributed bf16 values: the power the matrix units draw, and with it the clock the GPU
 * settles at, depends on the operand bits), with no memory traffic inside the loop.  sink: float[65536], written once.
 * *flop (host, may be NULL) receives the flops of the launch.  The caller times it.  Errors: ERR_NULL, ERR_SHAPE
 * (iters outside [1, 2^24]), ERR_ALIGN. */
int ecospa_mfma_probe(ecospa_ctx* ctx, const void* src, float* sink, int iters, double* flop /*host*/);

/* ------------------------------------------------------------------------------------------
 * Step 1 - per-dimension coupled importance score (paper Eq. 10; selection criterion Eq. 12).
 *
 * One ecospa_pair describes `groups` independent coupled pairs of one layer (the h heads of
 * Eq. 4, or 1 for the FFN pair of Eq. 7).  For unit u (= `unit` consecutive inner dimensions;
 * unit = 2 is the rotary 2x2 block of Eq. 6, whose Frobenius norm is position independent):
 *     r_u = sqrt(sum_{j in u} ||a_j||^2) * sqrt(sum_{j in u} ||b_j||^2),
 *     score[g][u] = r_u / sqrt(sum_{u' in group g} r_{u'}^2)       (0 if the group is all zero).
 * ECOSPA_PAIR_FFN_GATED scores a_j = row j of (w1 (.) w1b), the elementwise product of the
 * gate and up matrices (footnote to Eq. 8).
 * Grouped-query attention (Eq. 5): the rep1 query heads of a group pair with ONE key head, so inner
 * dimension j leaves all of them together and ||a_j||^2 adds the squared norms of row j of the rep1 heads
 * (QK pair: groups = key heads, w1 = W_q with groups*rep1 heads of n rows, the heads of a group side by
 * side; rep2 = 1).  In the same way rep2 heads of W_o share one value head (VO pair: w1 = W_v with
 * `groups` heads, w2 = W_o with groups*rep2 heads of n columns).  rep = 0 means 1; rep > 1 only for
 * the QK and VO kinds.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int kind;            /* ECOSPA_PAIR_*                                                      */
  int dtype;           /* ECOSPA_F32 | ECOSPA_BF16                                           */
  int groups;          /* independent pairs (heads); 1 for FFN                               */
  int n;               /* inner dimensions per group before pruning (d_h or d_ff)            */
  int unit;            /* 1, or 2 for rotary blocks; n % unit == 0                           */
  int d1, d2;          /* length of a_j and of b_j                                           */
  const void* w1;      /* [groups*rep1*n, d1], ld1: W_q | W_v | W_in | W_gate                */
  const void* w1b;     /* FFN_GATED: W_up [groups*n, d1], ld1b; otherwise NULL               */
  const void* w2;      /* QK: W_k [groups*rep2*n, d2]; VO/FFN*: W_o | W_out | W_down [d2, groups*rep2*n] */
  long long ld1, ld1b, ld2;
  int rep1, rep2;      /* heads of member 1 / member 2 per group (Eq. 5); 0 or 1: one each   */
  int w2_rows;         /* VO/FFN*: nonzero = the second member is stored with its units as rows,
                          [groups*rep2*n, d2] with ld2 >= d2 - b_j is row j, the orientation of B in
                          App. A.1 (and how GPT-2 checkpoints keep W_out) - so both members are read
                          along rows and the kept units are gathered as rows (axis 0)          */
} ecospa_pair;

/* Workspace bytes ecospa_coupled_score needs for this batch (host-only query; 0 on bad input). */
size_t ecospa_score_workspace_bytes(const ecospa_pair* pairs /*host*/, int n_pairs);
/* scores[p] (host array of device pointers) receives float[groups_p * n_p / unit_p].
 * All pairs of the batch are processed by shared launches (every weight is read once).
 * Errors: NULL pointers -> ERR_NULL; groups/n/d < 1, n % unit, ld < extent -> ERR_SHAPE;
 * unknown kind/dtype -> ERR_DTYPE; workspace too small -> ERR_WORKSPACE. */
int ecospa_coupled_score(ecospa_ctx* ctx, const ecospa_pair* pairs /*host*/, int n_pairs,
                         float* const* scores /*host*/);

/* ecospa_coupled_score for callers that cannot allocate device memory or attach a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same scores from the same kernels, with the
 * partial sums kept in a fixed array inside the library's device image (2 MiB per GPU, held until the process ends;
 * ecospa_coupled_score_static_max_bytes() returns the limit).  The call allocates nothing and does not touch the
 * context's workspace.  A batch whose ecospa_score_workspace_bytes() exceeds the limit -> ERR_WORKSPACE, before
 * anything is launched (2 MiB holds about six LLaMA-1B-shaped layers' pairs; larger batches go through
 * ecospa_coupled_score).  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two contexts) race; calls on one stream are ordered and safe.  Other errors as ecospa_coupled_score. */
size_t ecospa_coupled_score_static_max_bytes(void);
int ecospa_coupled_score_static(ecospa_ctx* ctx, const ecospa_pair* pairs /*host*/, int n_pairs,
                                float* const* scores /*host*/);

/* ------------------------------------------------------------------------------------------
 * Step 2 - keep the k most important units of every group (Sec. 3.2: "rank upsilon_i ... remove
 * those insignificant pairs"; Alg. 1's removal loop with the count fixed by the caller).
 * scores: float[groups * n_units]; idx: int32[groups * k], ascending within a group, values in
 * [0, n_units).  Order: larger score first, equal scores (-0 == +0) keep the lower index, NaN
 * ranks below every number - so exactly one result is correct.  Needs no workspace.
 * Errors: k < 1 or k > n_units -> ERR_K; groups/n_units < 1 -> ERR_SHAPE.
 * ------------------------------------------------------------------------------------------ */
int ecospa_select_topk(ecospa_ctx* ctx, const float* scores, int groups, int n_units, int k, int* idx);
/* The same for several score arrays (all coupled pairs of a layer) in one launch; `items` is a host
 * array.  Errors as above, checked for every item before anything is launched. */
typedef struct {
  const float* scores; /* float[groups * n_units] */
  int groups, n_units, k;
  int* idx;            /* int32[groups * k] */
} ecospa_select_item;
int ecospa_select_topk_batch(ecospa_ctx* ctx, const ecospa_select_item* items /*host*/, int n_items);

/* Steps 1 and 2 together (Eq. 10, then Sec. 3.2's ranking with the count fixed by the caller), for callers that
 * re-estimate few pairs at a time (one layer): scores[p] as ecospa_coupled_score writes them, and idx[p] (host array
 * of device pointers, int32[groups_p * k[p]]) the k[p] (host array) best units of every group of pair p, as
 * ecospa_select_topk would choose them from those scores.  The team that finishes a group's scores selects from
 * them in the same launch: two launches in all instead of three.  Workspace as ecospa_coupled_score.
 * Errors, before anything is launched: those of ecospa_coupled_score; ERR_NULL (k, idx, idx[p]);
 * k[p] < 1 or k[p] > n_p / unit_p -> ERR_K. */
int ecospa_score_select(ecospa_ctx* ctx, const ecospa_pair* pairs /*host*/, int n_pairs, float* const* scores /*host*/,
                        const int* k /*host*/, int* const* idx /*host*/);

/* ------------------------------------------------------------------------------------------
 * Pair-level importance and the cumulative-threshold rule (the two remaining pieces of Alg. 1).
 *
 * ecospa_pair_fisher - Eq. 8: the importance of a whole coupled pair from the loss gradients of its
 * two members, I = 1/2 * sum_{k=1,2} (1 / |W_k|) (1 / |D|) sum_ij (dL/dW_k)_ij^2.  `grads` describes
 * the gradient matrices exactly as an ecospa_pair describes the weights (w1 = dL/dW_1 ..., same
 * layouts, `unit` ignored); fisher[p] (host array of device pointers) receives float[groups_p], one
 * value per head / FFN pair.  For ECOSPA_PAIR_FFN_GATED the first member is (W_gate, W_up) together,
 * |W_1| counting both.  n_samples = |D| > 0.  Workspace and errors as ecospa_coupled_score.
 *
 * ecospa_select_theta - Alg. 1's inner loop for each of `groups` score rows: the unit with the smallest
 * score is removed while the remaining units still hold at least the fraction theta (0 <= theta <= 1)
 * of the row's total score; at least one unit stays.  Scores enter as integer masses
 * floor(clip(s, 0, 1) * 2^32) (NaN -> 0) and the bound is ceil(theta * total) in fp64, so all sums are
 * exact and exactly one result is correct.  Order of removal: ascending in the ordering of
 * ecospa_select_topk, higher index first among equal scores.  k_out: int32[groups] kept counts;
 * idx: int32[groups * n_units], row g holds its k_out[g] kept indices ascending, then -1.
 * Errors: ERR_NULL; groups/n_units < 1 -> ERR_SHAPE; theta outside [0, 1] (or NaN) -> ERR_K.
 * ------------------------------------------------------------------------------------------ */
int ecospa_pair_fisher(ecospa_ctx* ctx, const ecospa_pair* grads /*host*/, int n_pairs, float n_samples,
                       float* const* fisher /*host*/);
int ecospa_select_theta(ecospa_ctx* ctx, const float* scores, int groups, int n_units, float theta, int* idx, int* k_out);
/* ecospa_select_pairs - Alg. 1's choice among the coupled pairs of the model: of the n_pairs importance
 * values `fisher` (device float[n_pairs], as written by ecospa_pair_fisher into one array) the n_select
 * smallest are chosen (n_select = the top-K ratio times n_pairs, rounded by the caller); `chosen`
 * receives their indices, ascending (device int32[n_select]).  The order is that of ecospa_select_topk
 * reversed: smaller value first, NaN before every number, -0 == +0, equal values go to the lower index
 * - exactly one result is correct.  Errors: ERR_NULL; n_pairs < 1 -> ERR_SHAPE; n_select outside
 * [1, n_pairs] -> ERR_K. */
int ecospa_select_pairs(ecospa_ctx* ctx, const float* fisher, int n_pairs, int n_select, int* chosen);

/* ------------------------------------------------------------------------------------------
 * Step 3 - aligned gather of the kept inner dimensions into a smaller dense matrix (Def. 1:
 * the remaining terms keep their original pairing), and its inverse.
 *
 * The source axis holds groups*n inner dimensions; the destination axis holds, per group,
 * kp*unit slots of which the first k*unit receive the kept dimensions in ascending order and
 * the rest (padding for aligned tiles, kp >= k) are written as zeros:
 *   axis 0:  dst[g*kp*unit + i*unit + u, c] = src[g*n + idx[g*k+i]*unit + u, c],  c < other_extent
 *   axis 1:  dst[r, g*kp*unit + i*unit + u] = src[r, g*n + idx[g*k+i]*unit + u],  r < other_extent
 * Vectors (biases) are matrices with other_extent = 1 on axis 1.  Works for any dtype of 2 or 4
 * bytes (weights, moments, master copies).  idx must be ascending and in range (as written by
 * ecospa_select_topk); this is the caller's contract.
 * ecospa_scatter is the inverse: kept slots of src (compact layout) go back to their place in
 * dst (full layout) and every pruned row/column of dst is written as zero.
 * Errors: ERR_NULL, ERR_SHAPE (extents < 1, n % unit, ld too small), ERR_K (k < 1, k > n/unit,
 * kp < k), ERR_DTYPE.
 * ------------------------------------------------------------------------------------------ */
int ecospa_compact(ecospa_ctx* ctx, const void* src, void* dst, int dtype, int axis, int groups, int n,
                   int unit, int k, int kp, long long other_extent, long long ld_src, long long ld_dst,
                   const int* idx);
int ecospa_scatter(ecospa_ctx* ctx, const void* src, void* dst, int dtype, int axis, int groups, int n,
                   int unit, int k, int kp, long long other_extent, long long ld_src, long long ld_dst,
                   const int* idx);
/* Several gathers and/or scatters (every matrix, bias and moment of a layer) in one launch; the
 * fields have the meaning of the arguments above.  scatter: 0 = gather, 1 = the inverse direction with
 * zeros in every pruned row/column of dst, 2 = the inverse direction leaving pruned rows/columns of dst
 * as they are (compact parameters, master copies and moments written back into full-size arrays before
 * the importance is estimated again, Alg. 1); other values -> ERR_SHAPE.
 * `items` is a host array; all items are validated before anything is launched.  Items must not
 * overlap each other's destinations.
 * Reading contract of the column gathers (axis 1): rows are fetched in whole 16-byte pieces when src is 16-byte
 * aligned and ld_src is a multiple of 16 bytes that covers the inner extent rounded up to 16 bytes - a caller that
 * gives such an ld_src promises that every row, the last one included, is backed by memory up to that rounded extent
 * (a matrix with an odd inner width, stored with a padded leading dimension, then takes the fast path). */
/* Ragged kept counts (what the cumulative-threshold rule of Alg. 1 leaves: every head, every pair its
 * own k): k_group != NULL names a device int32[groups] array (k_out of ecospa_select_theta), ld_idx the
 * distance between the index lists of consecutive groups (idx: int32[groups * ld_idx], as written by
 * ecospa_select_theta with ld_idx = n_units).  Group g then keeps its first min(k_group[g], kp, ld_idx)
 * listed units and the remaining slots up to kp are zeros (scatter: its other rows/columns are
 * zeros), so all groups share the padded width kp and the compact matrices stay dense; `k` is not
 * used.  The counts live on the device and cannot be checked on the host: choosing kp >= max_g
 * k_group[g] is the caller's contract (units beyond kp would be dropped).  k_group == NULL: every
 * group keeps k units, ld_idx = 0 means k.  Errors for ragged items: kp < 1 or ld_idx < 1 -> ERR_K.
 * Grouped-query attention (Eq. 5): the idx_div query heads of a group keep the dimensions of their shared
 * key/value head, so W_q's rows and W_o's columns are gathered with groups = query heads and idx_div =
 * query heads per key/value head (idx: int32[(groups / idx_div) * ld_idx]); groups % idx_div != 0 -> ERR_SHAPE. */
typedef struct {
  const void* src;
  void* dst;
  int dtype, axis, groups, n, unit, k, kp, scatter;
  long long other_extent, ld_src, ld_dst;
  const int* idx;
  const int* k_group; /* device int32[groups / idx_div] or NULL */
  int ld_idx;
  int idx_div;        /* heads that share one index list: group g uses list (and count) g / idx_div; 0 or 1: its own */
  void* dst_t;        /* row gathers (axis 0, scatter 0) only, NULL: none - the transposed copy of dst written by the same
                         launch: dst_t[c * ld_dst_t + s] = dst[s * ld_dst + c] for every destination row s (padding
                         rows included) and c < other_extent; ld_dst_t >= groups * kp * unit.  It replaces an
                         ecospa_transpose_batch pass over the freshly gathered matrix.  Must not overlap src or dst. */
  long long ld_dst_t;
  const void* src_b;  /* row gathers of single rows (axis 0, scatter 0, unit 1) only, NULL: none - a second source of the
                         shape and leading dimension of src whose kept rows are interleaved with those of src:
                         destination row 2s is row map(s) of src, row 2s + 1 the same row of src_b, so dst has
                         2 * groups * kp rows (the (gate, up) row pairs of a gated FFN's first matrix from W_gate and
                         W_up in one copy); dst_t, if given, is the transposed copy of that interleaved matrix. */
} ecospa_map_item;
int ecospa_compact_batch(ecospa_ctx* ctx, const ecospa_map_item* items /*host*/, int n_items);

/* Debugging aid for the caller's contract on index lists (Def. 1 keeps the remaining terms in their original order:
 * ascending, in range).  Checks on the device, for each of `groups` lists (list g starts at idx + g*ld_idx), that its
 * first k entries - or k_group[g] entries when k_group != NULL (device int32[groups]; a count outside [0, ld_idx] is
 * itself an error) - lie in [0, n_units) and ascend strictly.  Unlike every other entry point it WAITS for the
 * context's stream (one flag word is copied back), so it belongs in tests and debug builds, not in timed paths.
 * Needs 4 bytes of workspace (its first word is clobbered).  Returns ECOSPA_ERR_INDEX if any list is bad.
 * Errors before anything is launched: ERR_NULL; groups/n_units/ld_idx < 1 -> ERR_SHAPE; k outside
 * [1, min(ld_idx, n_units)] with k_group == NULL -> ERR_K; no workspace -> ERR_WORKSPACE. */
int ecospa_check_indices(ecospa_ctx* ctx, const int* idx, int groups, int ld_idx, int k, const int* k_group, int n_units);

/* ------------------------------------------------------------------------------------------
 * Parameter update on the compact tensors (Alg. 1: "Update W", and the optimizer moments of a removed
 * row/column are removed with it - after ecospa_compact of the parameters, their master copies and both
 * moments with the same idx, all of them live in the compact layout).  AdamW, the optimizer of the
 * paper's GPT-2 and DeiT runs (Sec. 4.1), for step number `step` >= 1, elementwise:
 *   m <- beta1 m + (1 - beta1) g,   v <- beta2 v + (1 - beta2) g^2,
 *   w <- w - lr * ( (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps) + weight_decay * w )
 * in fp32 arithmetic, each result rounded once (to nearest even) to the type it is stored in.
 * Per tensor: w (device, n elements, updated in place; fp32 master weights or bf16 parameters), g
 * (gradient, read only), m and v (moments, updated in place, both of type s_dtype), and optionally
 * w_lp: a bf16 copy of the updated fp32 w, the working weights the contractions read (NULL: none; only
 * with w_dtype = ECOSPA_F32).  Tensors are contiguous and must not overlap; padding slots (w = g = m =
 * v = 0) stay exactly zero.  `items` and `hp` are host memory; all items are validated before anything
 * is launched, all tensors are updated by one launch (per 192 items).  Needs no workspace.
 * Errors: ERR_NULL; ERR_DTYPE (a type that is neither fp32 nor bf16; w_lp with bf16 w); ERR_SHAPE
 * (n < 1, n_items < 1, step < 1, beta outside [0, 1), negative lr / eps / weight_decay or NaN).
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  void* w;
  void* w_lp;      /* bf16[n] or NULL */
  const void* g;
  void* m;
  void* v;
  long long n;
  int w_dtype, g_dtype, s_dtype;
} ecospa_adamw_item;
typedef struct {
  float lr, beta1, beta2, eps, weight_decay;
  int step;
} ecospa_adamw_hyper;
int ecospa_adamw(ecospa_ctx* ctx, const ecospa_adamw_item* items /*host*/, int n_items,
                 const ecospa_adamw_hyper* hp /*host*/);

/* Transposed copies of (compact) matrices: dst[c, r] = src[r, c] for r < rows, c < cols, any 2- or 4-byte
 * dtype; all items in one launch; source and destination must not overlap.  The backward pass reads the
 * compact weights with the contraction index slow (dX = dY W); given a transposed copy beside the matrix
 * (the *_t fields of ecospa_block_desc) it runs the faster x W^T form.  A copy has to be refreshed
 * whenever its matrix changes (after ecospa_compact, after ecospa_adamw).
 * Errors: ERR_NULL, ERR_DTYPE, ERR_SHAPE (extents < 1, ld_src < cols, ld_dst < rows). */
typedef struct {
  const void* src;   /* [rows, cols], ld_src */
  void* dst;         /* [cols, rows], ld_dst */
  int dtype, rows, cols;
  long long ld_src, ld_dst;
} ecospa_transpose_item;
int ecospa_transpose_batch(ecospa_ctx* ctx, const ecospa_transpose_item* items /*host*/, int n_items);

/* cos/sin tables of the KEPT rotary blocks (Eq. 6; "position matrices are then adjusted to match
 * new dimensions", footnote to Eq. 10): for head g, position t < L, kept block i < k,
 *   angle = t * base^(-2 * idx[g*k+i] / d_h)   with d_h the ORIGINAL head width,
 * cos_out/sin_out: float[h, L, kp] (slots i >= k get cos = 1, sin = 0).  idx == NULL keeps
 * block i at slot i (dense layer).  Angles are evaluated in fp64. */
int ecospa_rope_table(ecospa_ctx* ctx, const int* idx, int h, int L, int k, int kp, int d_h, double base,
                      float* cos_out, float* sin_out);
/* The same with ragged kept counts: head g keeps its first min(k_group[g], kp, ld_idx) listed blocks
 * (idx: device int32[h * ld_idx], k_group: device int32[h]), the slots behind them get cos = 1, sin = 0. */
int ecospa_rope_table_ragged(ecospa_ctx* ctx, const int* idx, int ld_idx, const int* k_group, int h, int L, int kp,
                             int d_h, double base, float* cos_out, float* sin_out);
/* The gathers of ecospa_compact_batch and the tables of the kept rotary blocks in ONE launch (the tables follow from
 * the same index lists as the gathers, so a layer's compaction needs no launch of their own for them): `rope` (host,
 * NULL: plain ecospa_compact_batch) describes the tables as the arguments of ecospa_rope_table do (k_group == NULL;
 * ld_idx = 0 means k) or as those of ecospa_rope_table_ragged do (k_group != NULL, k unused).  Everything is validated
 * before anything is launched; errors as the separate calls. */
typedef struct {
  const int* idx;      /* device int32[h * ld_idx] kept blocks per head, or NULL (block i at slot i) */
  const int* k_group;  /* device int32[h] ragged kept counts, or NULL */
  int h, L, k, kp, d_h, ld_idx;
  double base;
  float *cos_out, *sin_out;   /* float[h, L, kp] */
} ecospa_rope_item;
int ecospa_compact_batch_rope(ecospa_ctx* ctx, const ecospa_map_item* items /*host*/, int n_items,
                              const ecospa_rope_item* rope /*host*/);

/* ------------------------------------------------------------------------------------------
 * Steps 4-5 - reduced forward and backward contractions on the compacted matrices (Eq. 1-3,
 * rewritten per head as Eq. 4; rotary form Eq. 6; gated FFN of the footnote to Eq. 8).
 *
 * Compact layouts (padding slots hold zeros, so results are exact):
 *   ATTN: w_qkv [((h + h_kv)*kp_qk + h_kv*kp_vo), d_model]: rows of W_q (head-major, kp_qk per head), then
 *         W_k, then W_v (kp_vo per head); b_qkv same length or NULL; w_o [d_model, h*kp_vo]; b_o.
 *         kp_qk, kp_vo are multiples of 16 and at most 128 (wider heads -> ERR_SHAPE, before anything is
 *         launched; the attention core runs a head in a 32-, 64- or 128-wide kernel, whichever holds it).  h_kv = key/value heads: h for multi-head
 *         attention (0 means h); under grouped-query attention (Eq. 5) h_kv divides h and query head i
 *         attends with key/value head i / (h / h_kv).
 *   FFN:  w_1 [kp_ff, d_model] (SWIGLU: [2*kp_ff, d_model], row 2i = gate unit i, row 2i+1 = up unit i, so that a
 *         tile of the first contraction holds whole (gate, up) pairs and the product is formed in its epilogue);
 *         b_1 same length and order or NULL; w_2 [d_model, kp_ff]; b_2.  kp_ff is a multiple of 16.
 * scale is the softmax scale (1/sqrt(original d_h) keeps "compact = masked dense").
 * rope_cos/rope_sin: float[h_kv, L, kp_qk/2] from ecospa_rope_table (one row of angles per key/value head:
 * the query heads that share it keep the same rotary blocks), or NULL for no rotation; pairs are
 * adjacent dimensions (2i, 2i+1).
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int block;                 /* ECOSPA_BLOCK_ATTN | ECOSPA_BLOCK_FFN */
  int dtype;
  int B, L, d_model;         /* tokens T = B*L, row-major [T, d_model] activations            */
  /* ATTN */
  int h, kp_qk, kp_vo;
  int causal;
  float scale;
  const float *rope_cos, *rope_sin;
  const void *w_qkv, *b_qkv, *w_o, *b_o;
  long long ld_wqkv, ld_wo;
  /* FFN */
  int kp_ff, act;
  const void *w_1, *b_1, *w_2, *b_2;
  long long ld_w1, ld_w2;
  /* ATTN, grouped-query attention */
  int h_kv;                  /* key/value heads; 0: as many as query heads                    */
  /* optional transposed copies of the weights for the backward pass (ecospa_transpose_batch), NULL: none.
   * w_qkv_t [d_model, nqkv], w_o_t [h*kp_vo, d_model], w_1_t [d_model, (1|2)*kp_ff], w_2_t [kp_ff, d_model];
   * leading dimensions multiples of 8, pointers 16-byte aligned.  Only the input-gradient contractions
   * read them; the results are those of the untransposed path up to the order of summation. */
  const void *w_qkv_t, *w_o_t, *w_1_t, *w_2_t;
  long long ld_wqkvt, ld_wot, ld_w1t, ld_w2t;
} ecospa_block_desc;

/* Activations the forward pass keeps for the backward pass; caller-allocated, dense row-major.
 *   ATTN: qkv [T, (h + h_kv)*kp_qk + h_kv*kp_vo] (Q and K after bias and rotation, V after bias),
 *         o [T, h*kp_vo] (per-head attention output), lse float[B*h*L] (log-sum-exp of the
 *         scaled, masked scores per query).
 *   FFN:  hpre [T, kp_ff] (SWIGLU: [T, 2*kp_ff], (gate, up) pre-activation pairs in the order of w_1's rows),
 *         act [T, kp_ff]. */
typedef struct {
  void *qkv, *o;
  float* lse;
  void *hpre, *act;
} ecospa_saved;

/* Gradients in the compact layouts of the weights they belong to (same dtype); any pointer may
 * be NULL to skip that gradient (bias gradients are skipped when NULL). */
typedef struct {
  void *dw_qkv, *db_qkv, *dw_o, *db_o;
  void *dw_1, *db_1, *dw_2, *db_2;
  long long ld_dwqkv, ld_dwo, ld_dw1, ld_dw2;
} ecospa_grads;

/* Workspace bytes forward+backward of this block need (host-only query; 0 on bad input). */
size_t ecospa_block_workspace_bytes(const ecospa_block_desc* desc /*host*/);
/* y[T, d_model] = block(x[T, d_model]); saved may be NULL for inference (ATTN still needs
 * workspace for q, k, v then).  Errors: ERR_NULL, ERR_SHAPE, ERR_DTYPE, ERR_ALIGN, ERR_WORKSPACE. */
int ecospa_coupled_fwd(ecospa_ctx* ctx, const ecospa_block_desc* desc /*host*/, const void* x, void* y,
                       const ecospa_saved* saved /*host*/);
/* From dy[T, d_model]: dx[T, d_model] and the compact weight gradients.  x, saved as in forward. */
int ecospa_coupled_bwd(ecospa_ctx* ctx, const ecospa_block_desc* desc /*host*/, const void* x, const void* dy,
                       const ecospa_saved* saved /*host*/, void* dx, const ecospa_grads* grads /*host*/);

/* ------------------------------------------------------------------------------------------
 * The dense contraction kernel behind steps 4-5, exposed for tests and tuning:
 *   C[m, n] = sum_k A(m, k) * B(n, k) (+ bias[n]),   m < M, n < N, k < K,   fp32 accumulation,
 *   A(m, k) = A[m*lda + k] (trans_a = 0) or A[k*lda + m] (trans_a = 1); B(n, k) likewise with ldb.
 * So x W^T is (0, 0), dY W is (0, 1) and dY^T X is (1, 1).  bias may be NULL.
 * tile (bf16 only; for tests and tuning): 0 = library's choice; 1 / 2 = 128x128 / 256x256 workgroup
 * tiles staged through registers, K-slow operands transposed on the way to LDS; 3 / 4 = the same with
 * K-slow operands read by transposing LDS reads; 10..19 and 21 = configurations 0..9 and 10 of the
 * software-pipelined kernel (direct global->LDS ring; needs K and K/splits to be multiples of its slab
 * depth, else the library falls back to its own choice); 20 = the register-prefetch kernel (256x256 tiles) for long
 * contractions with a K-slow B; 30..38 = the same kernel for dY^T X (both operands K-slow) with tiles 256x256,
 * 192x256, 256x192, 128x256, 256x128, 192x192, 128x192, 192x128, 128x128 (needs K and the K range of a split to be
 * multiples of 64).
 * splits: 0 = library's choice, otherwise the number of K splits (partials come from the
 * workspace and are added in a fixed order).
 * bf16 needs 16-byte aligned pointers, N % 8 == 0, leading dimensions % 8 == 0 and the
 * contiguous extent of each operand % 8 == 0 (-> ERR_ALIGN otherwise).
 * ------------------------------------------------------------------------------------------ */
int ecospa_contract(ecospa_ctx* ctx, int dtype, int M, int N, int K, const void* A, long long lda, int trans_a,
                    const void* B, long long ldb, int trans_b, void* C, long long ldc, const void* bias, int tile,
                    int splits);

/* The dY^T X form of ecospa_contract (bf16, both operands K-slow: A[K, M], B[K, N]) together with the column sums of
 * its A operand, colsum[m] = sum_k A(m, k) (float[M]) - the bias gradient that a backward pass gets from the weight-
 * gradient contraction that reads dY anyway.  Exposed for tests of every tile shape (tile: 0, 1..4, 20, 30..38 as in
 * ecospa_contract).  Workspace: splits * M floats (256-byte rounded) plus the partial products of a split contraction.
 * Errors as ecospa_contract. */
int ecospa_contract_colsum(ecospa_ctx* ctx, int M, int N, int K, const void* A, long long lda, const void* B,
                           long long ldb, void* C, long long ldc, float* colsum, int tile, int splits);

/* Workspace bytes ecospa_contract needs for this problem (host-only query): the fp32 partial sums of its K splits,
 * `splits` as passed to ecospa_contract (0 = the library's choice); 0 when K is not split or on bad input. */
size_t ecospa_contract_workspace_bytes(int dtype, int M, int N, int K, int splits);

/* ------------------------------------------------------------------------------------------
 * Layer glue.  The operators between the two blocks of a pre-norm decoder layer and around the stack: normalisation
 * with the residual addition in front of it, embedding lookup, mean cross-entropy.  The method leaves them as they
 * are - only the coupled pairs lose dimensions (Sec. 3.1; Alg. 1 touches the pairs' matrices alone) - and they are
 * the same for a dense and a sparse model; they are part of the library so that a whole training step of a stack
 * (the workloads of Sec. 4.1) runs in its kernels.  bf16 storage, fp32 arithmetic, every result rounded once; all
 * reductions in a fixed order (results repeat bit for bit).  Device pointers, rows contiguous (row r of a [T, d]
 * tensor at offset r * d), 16-byte aligned; everything asynchronous on the context's stream.
 * Errors, before any launch: ERR_NULL; ERR_DTYPE (dtype other than ECOSPA_BF16); ERR_SHAPE (T < 1, d < 8, d % 8,
 * d > 4096, unknown kind, V > 65536, a leading dimension below V, T % L != 0 with a position table);
 * ERR_ALIGN (a pointer off a 16-byte boundary, a leading dimension % 8); ERR_WORKSPACE (ecospa_norm_bwd).
 *
 * ecospa_norm_fwd: s = x + res (res NULL: s = x), rounded to bf16 and written to x_out when res is given (x_out may
 *   be x itself); kind RMS: y = s / sqrt(mean(s^2) + eps) * gain; kind LAYER: y = (s - mean(s)) / sqrt(var(s) + eps)
 *   * gain + bias (biased variance; bias NULL: none).  stat (NULL: not kept; float[T] for RMS: the reciprocal root,
 *   float[2T] for LAYER: mean, reciprocal root per row) is what ecospa_norm_bwd needs.
 * ecospa_norm_bwd: x = the s of the forward call.  dx = dres + the gradient through the normalisation (dres NULL:
 *   none; dx may be dres itself), dgain[d] (and dbias[d] for LAYER, NULL: not wanted) in bf16.  Workspace:
 *   ecospa_norm_bwd_workspace_bytes(T, d).
 * ecospa_embed_fwd: out[t] = table[ids[t]] (+ pos[t mod L], pos NULL: none; then T % L == 0); ids are int64; an id
 *   outside [0, vocab) reads as a zero row.
 * ecospa_embed_bwd: dtable[vocab, d] is written whole: row v = the sum of dx[t] over the positions t with
 *   ids[t] == v, added in position order in fp32 (zero for ids that do not occur; ids outside the table are
 *   skipped); dpos[L, d] = sum over the sequences of dx (NULL: not wanted).  d <= 4096.
 * ecospa_xent: row_loss[t] = log sum_j exp(logits[t, j]) - logits[t, targets[t]], *loss = mean over the T rows
 *   (device float), dlogits[t, j] = (softmax(logits[t])[j] - [j == targets[t]]) / T in bf16 (NULL: loss only;
 *   may be logits itself).  targets are int64; a target outside [0, V) makes its row count as zero loss and zero
 *   gradient (the mean still divides by T).  ldl, ldd: leading dimensions in elements.
 * ------------------------------------------------------------------------------------------ */
#define ECOSPA_NORM_RMS 0
#define ECOSPA_NORM_LAYER 1
int ecospa_norm_fwd(ecospa_ctx* ctx, int kind, int T, int d, int dtype, const void* x, const void* res, void* x_out,
                    const void* gain, const void* bias, float eps, void* y, float* stat);
int ecospa_norm_bwd(ecospa_ctx* ctx, int kind, int T, int d, int dtype, const void* x, const void* gain,
                    const float* stat, const void* dy, const void* dres, void* dx, void* dgain, void* dbias);
size_t ecospa_norm_bwd_workspace_bytes(int T, int d);
int ecospa_embed_fwd(ecospa_ctx* ctx, int T, int d, int vocab, int dtype, const long long* ids, const void* table,
                     const void* pos, int L, void* out);
int ecospa_embed_bwd(ecospa_ctx* ctx, int T, int d, int vocab, int dtype, const long long* ids, const void* dx,
                     void* dtable, void* dpos, int L);
int ecospa_xent(ecospa_ctx* ctx, int T, int V, int dtype, const void* logits, long long ldl, const long long* targets,
                void* dlogits, long long ldd, float* row_loss, float* loss);

#ifdef __cplusplus
}
#endif
#endif /* ECOSPA_H */
