/*
 * mosaic_prune.h -- C ABI of the MI355X (gfx950) projection-pruning hot path.
 *
 * The calls follow the problem statement of "Mosaic: Composite Projection
 * Pruning for Resource-efficient LLMs" (arXiv 2504.06323): the Parameter
 * Ranking Controller (Algorithm 1, Eq. 5, Eq. 6) and the unstructured /
 * structured / composite categories of the Parameter Pruning Controller
 * (Section 3.3, Section 4.1.3).
 *
 * Conventions shared by every entry point
 *   - Plain C, no exceptions.  Every call returns a prune_status (0 = ok,
 *     negative = error and nothing was launched).
 *   - Matrices are row-major.  A projection weight W is [rows = output
 *     features, cols = input features] with leading dimension ld_w (elements);
 *     its input activation X is [n_tokens, n_channels = cols] with ld_x.
 *   - Unless marked "host", a pointer is a DEVICE pointer owned by the caller.
 *     The library allocates nothing, frees nothing and keeps no state between
 *     calls.  Scratch memory is passed in as (ws, ws_bytes); its minimum size
 *     comes from prune_workspace_bytes() and it needs no initialisation.
 *     ws must be 16-byte aligned.
 *   - stream is a hipStream_t passed as void* (NULL = the default stream).
 *     All device work is enqueued asynchronously on it; nothing synchronises.
 *   - dtype is a prune_dtype: PRUNE_F32 (float) or PRUNE_BF16 (bfloat16 stored
 *     as 16-bit words).  bf16 is widened exactly to float before any arithmetic.
 *   - Results are deterministic: running a call twice on the same inputs gives
 *     bit-identical outputs (fixed reduction orders; only integer atomics).
 *   - Any shape is accepted.  Rows whose base address and width allow 128-bit
 *     accesses (pointer 16-byte aligned, cols and ld multiples of 8) take the
 *     vectorised kernels; everything else takes slower scalar kernels with the
 *     same results.
 */
#ifndef MOSAIC_PRUNE_H
#define MOSAIC_PRUNE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PRUNE_OK = 0,
    PRUNE_ERR_NULL = -1,      /* a required pointer is NULL */
    PRUNE_ERR_SHAPE = -2,     /* non-positive extent, or ld smaller than the row width */
    PRUNE_ERR_DTYPE = -3,     /* dtype is not a prune_dtype */
    PRUNE_ERR_ALIGNMENT = -4, /* ws not 16-byte aligned, or a pointer not aligned to its element size */
    PRUNE_ERR_WORKSPACE = -5, /* ws_bytes smaller than prune_workspace_bytes(), or (prune_stats_norms_static) the
                                 problem needs more scratch than PRUNE_STATIC_SCRATCH_BYTES */
    PRUNE_ERR_RANGE = -6,     /* scalar argument outside its documented range */
    PRUNE_ERR_DEVICE = -7     /* the HIP runtime refused a launch */
} prune_status;

typedef enum { PRUNE_F32 = 0, PRUNE_BF16 = 1 } prune_dtype;

typedef enum {
    PRUNE_OP_STATS = 0,   /* rows = n_tokens, cols = n_channels */
    PRUNE_OP_SCORE = 1,   /* rows, cols of W */
    PRUNE_OP_OUTLIER = 2, /* needs no workspace (returns 0) */
    PRUNE_OP_SELECT = 3,  /* rows, cols of W */
    PRUNE_OP_STRUCT = 4,  /* rows = inter, cols = hidden */
    PRUNE_OP_BATCH = 5    /* prune_score_outlier_batch: a constant, rows and cols are ignored (pass 1, 1) */
} prune_op;

/* Which entries of the table of outlier ratios are compared with one another when targets are
 * planned: all of them, those of one projection category across the layers, or -- layer pruning
 * (Section 4.1.3, Pruning Methods, item 2) -- whole layers, each with one target for all its
 * projections. */
typedef enum { PRUNE_SCOPE_GLOBAL = 0, PRUNE_SCOPE_CATEGORY = 1, PRUNE_SCOPE_LAYER = 2 } prune_scope;

/* Which mean an outlier is measured against: that of its own projection (Eq. 6, projection
 * outlier distribution) or that of all projections handed over together, i.e. of the layer
 * (Eq. 3 and Eq. 4, layer outlier distribution). */
typedef enum { PRUNE_OUTLIERS_PER_PROJECTION = 0, PRUNE_OUTLIERS_PER_LAYER = 1 } prune_outlier_scope;

/* One projection of a batch: weight [rows, cols] (device, pitch ld_w) and the norms [cols] (device)
 * of the activation it multiplies. */
typedef struct {
    const void *w;
    int64_t rows, cols, ld_w;
    const float *norms;
} prune_projection;

/* host, pure.  Library version as major * 10000 + minor * 100 + patch. */
int prune_version(void);

/* host, pure.  Static string naming a prune_status. */
const char *prune_status_string(int status);

/* host, pure.  Minimum ws_bytes for one call of `op` on a problem of the given
 * extents (see prune_op for what rows/cols mean).  Returns 0 for bad arguments. */
size_t prune_workspace_bytes(int op, int64_t rows, int64_t cols);

/*
 * Activation statistics (Algorithm 1, the loop that gathers A over the
 * calibration samples; the l2-norm term of Eq. 5).
 *   sumsq[j] += sum over t < n_tokens of x[t * ld_x + j]^2      for j < n_channels
 * x       [n_tokens, n_channels] of dtype, read once.
 * sumsq   [n_channels] float, in/out: the caller zeroes it before the first
 *         chunk of a tensor and may call repeatedly with further token chunks.
 * Squares and sums are formed in float (fixed order), the cross-block
 * reduction in double.  n_tokens == 0 is a valid no-op.
 */
int prune_stats_accumulate(const void *x, int dtype, int64_t n_tokens, int64_t n_channels, int64_t ld_x,
                           float *sumsq, void *ws, size_t ws_bytes, void *stream);

/*
 * The same statistics for a tensor that is handed over whole, in one call:
 *   sumsq[j] = sum over t < n_tokens of x[t * ld_x + j]^2 ;  norms[j] = sqrt(sumsq[j])
 * Both outputs are overwritten (no zeroing by the caller, no finalize call).
 * n_tokens == 0 writes zeros.  Workspace as for prune_stats_accumulate.
 */
int prune_stats_norms(const void *x, int dtype, int64_t n_tokens, int64_t n_channels, int64_t ld_x, float *sumsq,
                      float *norms, void *ws, size_t ws_bytes, void *stream);

/*
 * prune_stats_norms for callers that cannot allocate device memory and so have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments
 * (minus the workspace), same kernels, same results bit for bit.  The per-stripe partial sums live in
 * an array built into the library, PRUNE_STATIC_SCRATCH_BYTES per GPU, which each GPU the call runs on
 * holds until the process ends.  The call allocates and frees nothing; its first call on a device looks
 * up the address of that device's array.
 * A shape whose partial sums do not fit (prune_workspace_bytes(PRUNE_OP_STATS, n_tokens, n_channels)
 * above PRUNE_STATIC_SCRATCH_BYTES: more than 524288 channels) is refused with PRUNE_ERR_WORKSPACE and
 * nothing is launched.  All calls on one GPU share the array: calls that overlap in time on one GPU
 * (different streams, or different host threads) race and give wrong sums; calls on one stream, or
 * otherwise ordered, are safe.  Nothing needs clearing between calls: every partial sum that is read
 * was written by the same call.
 */
#define PRUNE_STATIC_SCRATCH_BYTES ((size_t)2 << 20)
int prune_stats_norms_static(const void *x, int dtype, int64_t n_tokens, int64_t n_channels, int64_t ld_x,
                             float *sumsq, float *norms, void *stream);

/* norms[j] = sqrt(sumsq[j]) (correctly rounded float sqrt).  In place allowed. */
int prune_stats_finalize(const float *sumsq, int64_t n_channels, float *norms, void *stream);

/*
 * Weight metric (Eq. 5; Algorithm 1, "Weight metric" step).
 *   omega[i, j] = float(|w[i, j]|) * norms[j]        one IEEE float multiply
 *   *score_sum  = sum over i, j of omega[i, j]       accumulated in double, fixed order
 * w          [rows, cols] of dtype, read once.
 * norms      [cols] float, as produced by prune_stats_finalize.
 * scores     optional [rows, cols] float, contiguous (ld = cols): receives omega.
 *            NULL in the hot mode (nothing but the sum is written).
 * score_sum  one double on the device.
 */
int prune_score(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld_w, const float *norms,
                float *scores, double *score_sum, void *ws, size_t ws_bytes, void *stream);

/*
 * Projection outliers (Eq. 6; Algorithm 1, the C / O steps).
 *   tau    = float(alpha * *score_sum / (rows * cols))   formed in double, rounded once
 *   *count = #{ (i, j) : omega[i, j] > tau }              strict, float compare
 * The projection rank is R = 100 * count / (rows * cols), formed by the caller.
 * omega is recomputed from (w, norms) exactly as in prune_score, or read from
 * `scores` when that is non-NULL (then w and norms may be NULL).
 * alpha >= 0.  count: one unsigned 64-bit on the device.  tau: optional float
 * on the device receiving the threshold that was used.
 */
int prune_outlier_ratio(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld_w,
                        const float *norms, const float *scores, float alpha, const double *score_sum,
                        unsigned long long *count, float *tau, void *stream);

/*
 * Weight metric and outliers of several projections at once (the loop over the
 * projections of a layer in Algorithm 1): three launches for the whole batch
 * instead of four per projection.
 * outlier_scope == PRUNE_OUTLIERS_PER_PROJECTION (Eq. 5, Eq. 6): for every i
 *   score_sums[i], taus[i], counts[i]
 * are what prune_score (without materialised scores) followed by
 * prune_outlier_ratio compute for projs[i]; the sums are accumulated in a
 * different fixed order, so they may differ from the single calls in the last
 * bits, and counts are exact for the threshold taus[i] that is reported.
 * outlier_scope == PRUNE_OUTLIERS_PER_LAYER (Eq. 3, Eq. 4, with the batch being
 * the projections of one layer, at most 16): score_sums[i] as above, but every
 *   taus[i] = float(alpha * sum_i score_sums[i] / sum_i rows_i * cols_i)
 * and counts[i] = #{omega in projs[i] : omega > that threshold}; the layer's
 * outlier count is the sum of counts[].
 * projs is a HOST array (read during the call); score_sums, counts, taus
 * (optional) are device arrays of n_proj entries.  All projections share dtype.
 * ws_bytes >= prune_workspace_bytes(PRUNE_OP_BATCH, 1, 1) (a constant).  If any
 * projection rules out 128-bit accesses the whole batch runs on scalar accesses.
 */
int prune_score_outlier_batch(const prune_projection *projs, int n_proj, int dtype, float alpha, int outlier_scope,
                              double *score_sums, unsigned long long *counts, float *taus, void *ws, size_t ws_bytes,
                              void *stream);

/*
 * host only, touches no device (Algorithm 1's normalize(R_LLM) and the
 * Projection Planner of Section 3.3; Eq. 1, Eq. 2).
 * Turns the n_layers x n_proj table of outlier counts into sparsity targets:
 *   R = 100 * counts / numels;  within a scope (all entries, or one projection
 *   category across layers) r_hat = (R - min) / (max - min) and
 *   s = p + 2 * lambda * (mean(r_hat) - r_hat);  s = p when max == min.
 * scope == PRUNE_SCOPE_LAYER (layer pruning, Section 4.1.3 Pruning Methods item
 * 2; Section 3.1): the ratio is taken per layer, R_n = 100 * (sum of the layer's
 * counts) / (sum of its numels) -- the counts then being those against the
 * layer's mean (PRUNE_OUTLIERS_PER_LAYER) --, the n_layers ratios are normalised
 * and spread by the same rule, and every projection of layer n gets s_n.
 * The unweighted mean of s is p, more outliers give a smaller s.  If cols is
 * non-NULL each s is clamped to [0, 1 - 1 / cols] and *clamped_out (optional)
 * is set to 1 when any clamp changed a value; zeros_per_row_out (optional,
 * needs cols) receives k = floor(s * cols), the per-row count handed to
 * prune_select_mask.  All arrays are host arrays of n_layers * n_proj entries,
 * row-major.  p in [0, 1), lambda >= 0.
 */
int prune_plan_sparsity(const unsigned long long *counts, const unsigned long long *numels, const int64_t *cols,
                        int n_layers, int n_proj, double p, double lambda, int scope, double *sparsity_out,
                        uint32_t *zeros_per_row_out, int *clamped_out);

/*
 * prune_plan_sparsity computed on the device (same arithmetic, same order of
 * operations, so the same bits), for callers that must not wait for the
 * outlier counts on the host: the counts stay where prune_score_outlier_batch
 * wrote them and the zeros-per-row land where prune_select_mask_batch can read
 * them (prune_select_item.k_dev).
 * DEVICE arrays of n_layers * n_proj entries: counts, numels (uint64), cols
 * (int64, required), sparsity_out (double), zeros_per_row_out (uint32).
 * flags_out: DEVICE int[2]; [0] = 1 iff some target was clamped, else 0;
 * [1] = 1 iff an input was invalid (numel == 0, count > numel, cols <= 0), in
 * which case the other outputs are unspecified, else 0.
 * One small launch on `stream`; returns once it is enqueued.  n_layers * n_proj <= 1048576.
 */
int prune_plan_sparsity_device(const unsigned long long *counts, const unsigned long long *numels,
                               const int64_t *cols, int n_layers, int n_proj, double p, double lambda, int scope,
                               double *sparsity_out, uint32_t *zeros_per_row_out, int *flags_out, void *stream);

/*
 * Unstructured projection pruning (Section 4.1.3, category 1: pruned
 * parameters are set to zero).  In every row the k entries with the smallest
 * omega are zeroed; among equal omega the lower column goes first, so the
 * result is unique.  omega is recomputed from (w, norms) as in prune_score, or
 * read from `scores` (contiguous [rows, cols], non-negative) when non-NULL.
 *   w_out[i, j] = pruned(i, j) ? 0 : w[i, j]          same dtype as w, pitch ld_out
 * w_out may equal w (in place, then ld_out == ld_w) or be a separate buffer;
 * partial overlap is not allowed.  mask_bits is optional: uint32 [rows, ceil(cols / 32)], bit b of
 * word q of a row is 1 iff column 32 * q + b is kept; bits past cols are 0.
 * 0 <= k <= cols; k == 0 copies w to w_out.
 */
int prune_select_mask(const void *w, void *w_out, int dtype, int64_t rows, int64_t cols, int64_t ld_w,
                      int64_t ld_out, const float *norms, const float *scores, uint32_t k, uint32_t *mask_bits, void *ws,
                      size_t ws_bytes, void *stream);

/*
 * One projection of a prune_select_mask_batch call; fields as the arguments of prune_select_mask.
 * k_dev (nullable): DEVICE pointer to this projection's k, read by the kernels when they run (for
 * example an element of prune_plan_sparsity_device's zeros_per_row_out); when set, the field k is
 * ignored and a value above cols counts as cols.
 * row_sumsq (nullable): DEVICE float [rows]; receives, for every row, the sum of the squares of the row
 * as it is written to w_out (float arithmetic, fixed order).  For the gate and up projections these
 * are the row terms of prune_struct_compact's group magnitude, formed here while the masked row is
 * still in registers instead of by another pass over the two matrices.
 */
typedef struct {
    const void *w;
    void *w_out;
    int64_t rows, cols, ld_w, ld_out;
    const float *norms;
    uint32_t k;
    uint32_t *mask_bits; /* nullable */
    const uint32_t *k_dev; /* nullable */
    float *row_sumsq; /* nullable */
} prune_select_item;

/*
 * prune_select_mask for several projections (Section 4.1.3, category 1, applied to
 * the projections of a layer): projections whose rows have the same width class
 * share one launch.  Every item is processed exactly as by prune_select_mask with
 * scores == NULL (the metric is recomputed from w and norms); the whole batch is
 * validated before anything is launched.  items is a HOST array of n_items <= 1024
 * entries, read during the call; all items share dtype.  Needs no workspace.
 */
int prune_select_mask_batch(const prune_select_item *items, int n_items, int dtype, void *ws, size_t ws_bytes,
                            void *stream);

/*
 * Structured removal of MLP intermediate channels (Section 4.1.3, categories
 * 2 and 3; Fig. 4: the nodes between projections are pruned as a group).
 * Run on the already masked weights for the composite category.
 *   group_mag[c] = sum_j gate[c, j]^2 + sum_j up[c, j]^2 + sum_i down[i, c]^2
 * the r channels with the smallest group_mag (lower c first among equals) are
 * removed; kept_idx receives the remaining inter - r channel indices in
 * ascending order, and, when the three *_out pointers are non-NULL,
 *   gate_out = gate[kept, :]  [inter - r, hidden]
 *   up_out   = up[kept, :]    [inter - r, hidden]
 *   down_out = down[:, kept]  [hidden, inter - r]
 * gate, up are [inter, hidden], down is [hidden, inter]; all inputs and
 * outputs are contiguous.  Pass all three outputs or none (rank only).
 * 0 <= r < inter.  Outputs must not overlap inputs.
 * gate_rowsq, up_rowsq (DEVICE float [inter], both or neither): the row sums of squares of gate and up
 * when the caller already has them (prune_select_item.row_sumsq of the masking pass that produced the
 * two matrices); the call then reads gate and up only for the gather.  They must belong to the gate
 * and up handed in: the call does not check.
 */
int prune_struct_compact(const void *gate, const void *up, const void *down, int dtype, int64_t inter,
                         int64_t hidden, uint32_t r, const float *gate_rowsq, const float *up_rowsq,
                         float *group_mag, int32_t *kept_idx, void *gate_out, void *up_out, void *down_out,
                         void *ws, size_t ws_bytes, void *stream);

/*
 * Structured removal of coupled groups that span several projections (Section
 * 4.1.3, categories 2 and 3: attention heads and feed-forward channels; Fig. 4:
 * nodes between projections pruned as a group).  Group g < n_groups owns
 *   rows [g * row_per[i], (g + 1) * row_per[i])  of row_mats[i]  ([n_groups * row_per[i], row_width[i]])
 *   cols [g * col_per[i], (g + 1) * col_per[i])  of col_mats[i]  ([col_height[i], n_groups * col_per[i]])
 * e.g. one group per key/value head of grouped-query attention: rows of q (all
 * query heads of the group), k and v as row matrices, columns of o as a column
 * matrix; or one feed-forward channel: gate and up rows, down column.
 *   group_mag[g] = sum of squares of everything group g owns
 * The r groups of lowest magnitude are removed (lower g first among equals);
 * kept_idx gets the other n_groups - r indices ascending; when row_outs and
 * col_outs are given, row_outs[i] = the kept groups' rows of row_mats[i] and
 * col_outs[i] = the kept groups' columns of col_mats[i], in kept order.
 * The pointer arrays and the extent arrays are HOST arrays of n_row (n_col)
 * entries, at most 8 each; the matrices, group_mag, kept_idx and outputs are
 * contiguous device buffers that do not overlap.  Pass both output arrays or
 * neither (rank only).  0 <= r < n_groups.
 * ws_bytes >= prune_struct_groups_workspace_bytes(same extents).
 */
size_t prune_struct_groups_workspace_bytes(const int64_t *row_per, const int64_t *row_width, int n_row,
                                           const int64_t *col_per, const int64_t *col_height, int n_col,
                                           int64_t n_groups);
int prune_struct_groups(const void *const *row_mats, const int64_t *row_per, const int64_t *row_width, int n_row,
                        const void *const *col_mats, const int64_t *col_per, const int64_t *col_height, int n_col,
                        int dtype, int64_t n_groups, uint32_t r, float *group_mag, int32_t *kept_idx,
                        void *const *row_outs, void *const *col_outs, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * The Hessian-based one-shot pruner with weight compensation that the paper's experiments run with
 * the planner's targets (Section 4.1.3, "Pruning Methods"; Section 4.1.4, "Calibration": the same
 * 128 samples give the Hessian).  Built in stages; each stage is an entry point of its own.
 * ------------------------------------------------------------------------------------------------ */

/*
 * Hessian of the layer-wise reconstruction problem of one projection input:
 *   h[i, j] += sum_t x[t, i] * x[t, j]          0 <= i, j < channels
 * x: DEVICE [n_tokens, channels] of dtype, pitch ld_x (elements).  h: DEVICE fp32 [channels, channels],
 * pitch ld_h, in/out: zero it before the first chunk of tokens; both triangles are written and stay
 * bitwise symmetric.  Products are exact for bf16 input, sums are fp32 within a block's share of the
 * tokens and double across shares, in a fixed order (reproducible bit for bit).
 * ws_bytes >= prune_hessian_workspace_bytes(n_tokens, channels).  n_tokens == 0 is a no-op.
 */
size_t prune_hessian_workspace_bytes(int64_t n_tokens, int64_t channels);
int prune_hessian_accumulate(const void *x, int dtype, int64_t n_tokens, int64_t channels, int64_t ld_x, float *h,
                             int64_t ld_h, void *ws, size_t ws_bytes, void *stream);

/*
 * Factor of the damped Hessian.  In place on h (DEVICE fp32 [n, n], pitch ld_h, symmetric, as left by
 * prune_hessian_accumulate):
 *   1. dead[j] = (h[j, j] == 0) (DEVICE uint8 [n], nullable); such channels get h[j, j] = 1
 *   2. h[j, j] += damp * mean_j(h[j, j])
 *   3. the upper triangle of h (diagonal included) becomes R, upper triangular with positive diagonal and
 *      R R^T = h; R is the inverse of the upper Cholesky factor U of h^-1 (h^-1 = U^T U) that the published
 *      pruner is written with.  The strictly lower triangle is left unspecified.
 * info (DEVICE int, nullable): 0, or the 1-based index of a pivot that was not positive (the factor then
 * holds NaNs).  n and ld_h must be multiples of 4, h 16-byte aligned.
 * ws_bytes >= prune_hessian_factor_workspace_bytes(n).  fp32 throughout.
 */
size_t prune_hessian_factor_workspace_bytes(int64_t n);
int prune_hessian_factor(float *h, int64_t n, int64_t ld_h, double damp, uint8_t *dead, int *info, void *ws,
                         size_t ws_bytes, void *stream);

/*
 * The compensated sweep of the one-shot pruner over one projection, with the sparsity target the planner
 * assigned to it.  Columns are processed left to right in blocks of 128.  When a block starts, the saliency of
 * entry (i, j) is (current w[i, j] / U[j, j])^2 with U = R^-1; the floor(sparsity * rows * width) entries of the
 * block with the smallest saliency are pruned (all rows compete together; equal saliencies go by row-major
 * position in the block); column by column a pruned entry becomes 0, a kept one keeps its current value, and the
 * error is spread over all later columns so that the layer's output on the calibration data changes least.
 *   w, w_out: DEVICE [rows, cols] of dtype, pitches ld_w / ld_out; w_out may equal w (then ld_out == ld_w).
 *   r: DEVICE fp32, the factor left by prune_hessian_factor in the upper triangle of [cols, cols], pitch ld_r.
 *   dead: DEVICE uint8 [cols], nullable: columns whose weights count as zero (from prune_hessian_factor).
 *   first_block, n_blocks: the range of 128-column blocks to process in this call (n_blocks < 0: all the rest).
 *     A projection may be swept in several calls, in order, starting at block 0.  Between the calls v (or, when v
 *     is NULL, the workspace, which then holds it) must be left untouched.  The workspace also holds the changes
 *     of the current group of four blocks: a call with first_block % 4 != 0 continues such a group and must be
 *     given the workspace of the previous call, untouched; a call that starts a group (first_block % 4 == 0) with
 *     a caller-owned v may be given any workspace.
 *   v: DEVICE fp32 [rows, cols] contiguous, nullable: the working matrix G.  For every column j not yet processed
 *     it holds sum over the finished columns i of (w[:, i] - w_out[:, i]) * R[i, j]; zeroed by the call that
 *     processes block 0.  Given by callers that sweep in several calls and want the state in a buffer of their own.
 *   saliency: DEVICE fp32 [rows, cols] contiguous, nullable: receives, for the columns of every block processed,
 *     the saliencies the selection of that block was taken on (fp32, as computed when the block started).
 *   mask_bits: nullable, uint32 [rows, ceil(cols / 32)] keep-bits as written by prune_select_mask (only the words
 *     of the processed blocks are written).
 * cols and ld_r must be multiples of 4; r 16-byte, ws 256-byte aligned.  fp32 arithmetic throughout.
 * ws_bytes >= prune_obs_sweep_workspace_bytes(rows, cols, v == NULL).
 */
size_t prune_obs_sweep_workspace_bytes(int64_t rows, int64_t cols, int own_v);
int prune_obs_sweep(const void *w, void *w_out, int dtype, int64_t rows, int64_t cols, int64_t ld_w, int64_t ld_out,
                    const float *r, int64_t ld_r, const uint8_t *dead, double sparsity, int64_t first_block,
                    int64_t n_blocks, float *v, float *saliency, uint32_t *mask_bits, void *ws, size_t ws_bytes,
                    void *stream);

/* ------------------------------------------------------------------------------------------------
 * Forward pass of the feed-forward block (LLaMA-style layers of Table 2, Section 4.1.1):
 *   h = silu(x gate^T) * (x up^T),   y = h down^T.
 * The down projection's input h, whose per-channel norms enter its weight metric (Eq. 5), thereby comes from
 * a real forward pass, and the block can be run at full and at structurally pruned size (Section 4.1.3,
 * categories 2 and 3).
 * ------------------------------------------------------------------------------------------------ */

/*
 * y[t, j] = sum_k x[t, k] * w[j, k]: a bias-free projection with weights [n, k].
 * x [tokens, k] pitch ld_x, w [n, k] pitch ld_w, y [tokens, n] pitch ld_y, all DEVICE and of dtype; fp32
 * accumulation, the result rounded once to dtype.  bf16 data with k a multiple of 32, pitches multiples of 8 and
 * 16-byte aligned x and w runs on the matrix cores; anything else on a plain kernel with the same semantics.
 */
int prune_linear(const void *x, const void *w, void *y, int dtype, int64_t tokens, int64_t n, int64_t k, int64_t ld_x,
                 int64_t ld_w, int64_t ld_y, void *stream);

/*
 * h[t, c] = silu(sum_k x[t, k] gate[c, k]) * (sum_k x[t, k] up[c, k]),  silu(a) = a / (1 + exp(-a)),
 * rounded once to dtype; gate, up [inter, hidden] with the same pitch ld_w.
 * sumsq (DEVICE fp32 [inter], nullable, in/out): sumsq[c] += sum_t h[t, c]^2 over the stored (rounded) values --
 * the statistic prune_stats_accumulate would give on h, produced where h is produced; fixed summation order.
 * ws: needed only with sumsq on the matrix-core path, ws_bytes >= prune_mlp_workspace_bytes(tokens, inter).
 */
size_t prune_mlp_workspace_bytes(int64_t tokens, int64_t inter);
int prune_mlp_gate_up(const void *x, const void *gate, const void *up, void *h, int dtype, int64_t tokens,
                      int64_t hidden, int64_t inter, int64_t ld_x, int64_t ld_w, int64_t ld_h, float *sumsq, void *ws,
                      size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * The attention half of a LLaMA-style layer (Table 2, Section 4.1.1), so that the inputs of the q / k / v, o and
 * gate / up projections can come from a forward pass as well.  Token rows hold their heads side by side.
 * ------------------------------------------------------------------------------------------------ */

/* y[t, :] = x[t, :] / sqrt(mean_j x[t, j]^2 + eps) * weight[:]; x, y [tokens, channels] with pitches, weight [channels]. */
int prune_rmsnorm(const void *x, const void *weight, void *y, int dtype, int64_t tokens, int64_t channels, int64_t ld_x,
                  int64_t ld_y, float eps, void *stream);

/* out[t, j] = a[t, j] + b[t, j] (a residual connection); out may be a or b. */
int prune_add(const void *a, const void *b, void *out, int dtype, int64_t rows, int64_t cols, int64_t ld_a, int64_t ld_b,
              int64_t ld_out, void *stream);

/*
 * Rotary position embedding, in place on x [tokens, heads * head_dim] (pitch ld): in every head, dimension
 * i < head_dim / 2 is paired with i + head_dim / 2 and the pair (a, b) becomes (a cos - b sin, b cos + a sin) with
 * the angle (t mod seq_len) * base^(-2 i / head_dim).  head_dim even, base > 1 (the models use 10000).
 */
int prune_rotary(void *x, int dtype, int64_t tokens, int64_t heads, int64_t head_dim, int64_t ld, int64_t seq_len,
                 float base, void *stream);

/*
 * Causal attention per sequence and head:
 *   o[s, h, :] = sum_{t <= s} softmax_t(q[s, h, :] . k[t, g, :] / sqrt(head_dim)) v[t, g, :],  g = h / (heads / kv_heads)
 * q, o [n_seqs * seq_len, heads * head_dim], k, v [n_seqs * seq_len, kv_heads * head_dim], with pitches; heads a
 * multiple of kv_heads, head_dim <= 256.  bf16 with head_dim 128, pitches multiples of 8 and 16-byte aligned bases
 * runs on the matrix cores; anything else on a plain kernel with the same semantics.
 */
int prune_causal_attention(const void *q, const void *k, const void *v, void *o, int dtype, int64_t n_seqs,
                           int64_t seq_len, int64_t heads, int64_t kv_heads, int64_t head_dim, int64_t ld_q, int64_t ld_k,
                           int64_t ld_v, int64_t ld_o, void *stream);

/* ------------------------------------------------------------------------------------------------
 * Measurement aid (nothing of the paper): the streaming rates this card delivers to the plainest
 * kernels, which the benchmark reports beside the published HBM peak so that every pass of the path
 * can be held against both (the paper reports means over repeated trials, Section 4.1.5; so does the
 * benchmark).
 *   PRUNE_PROBE_READ: reads `bytes` from src in 128-bit non-temporal loads; dst receives one checksum
 *     word per thread, prune_bandwidth_probe_sink_bytes(blocks) bytes.
 *   PRUNE_PROBE_COPY: dst[0 .. bytes) = src[0 .. bytes).
 * src, dst: DEVICE, 16-byte aligned, not overlapping; bytes a positive multiple of 16; blocks: the
 * number of 256-thread workgroups that share the range (1 .. 1048576).  One launch on `stream`.
 * ------------------------------------------------------------------------------------------------ */
typedef enum { PRUNE_PROBE_READ = 0, PRUNE_PROBE_COPY = 1 } prune_probe_mode;
size_t prune_bandwidth_probe_sink_bytes(int blocks);
int prune_bandwidth_probe(const void *src, void *dst, size_t bytes, int mode, int blocks, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOSAIC_PRUNE_H */
