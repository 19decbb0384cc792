/*
 * aes_spmm.h - C ABI of the MI355X (gfx950) adaptive-edge-sampling SpMM library.
 *
 * The library computes Y = A_s * X, where A_s is the CSR matrix A after the
 * per-row adaptive edge sampling of the AES-SpMM paper (Sec. 3.2 Algorithm 1,
 * Sec. 3.3 Table 1 and Eq. 3), and X is a dense feature matrix in float32 or in
 * 8-bit quantised form (Sec. 2.3 Eq. 1-2) that is dequantised while it is
 * gathered.
 *
 * Conventions for every entry point
 *   - Pointers marked [dev] are DEVICE pointers on the current HIP device;
 *     [host] pointers are ordinary host memory.  The library never allocates,
 *     frees or keeps device memory: all buffers, workspaces included, are owned
 *     by the caller and may be released once the stream has passed the call
 *     (the one exception, a fixed array inside the code object, is described
 *     with aes_sample_build_noalloc).
 *   - Every call is asynchronous: it enqueues kernels on `stream` (a
 *     hipStream_t passed as void*, NULL = the default stream) and returns.  It
 *     never synchronises.  Calls on different streams may run concurrently as
 *     long as their output buffers and workspaces do not overlap.
 *   - Return value: AES_OK (0) or a negative aes_status.  Argument errors
 *     (NULL where not allowed, negative sizes, bad enum, too small workspace,
 *     misaligned leading dimension) are found on the host BEFORE anything is
 *     launched.  AES_ERR_HIP reports a launch failure.  Contents of CSR arrays
 *     are not validated on the device: a monotone rowptr with rowptr[0] == 0,
 *     rowptr[n_rows] == nnz and 0 <= colidx < n_cols is the caller's contract.
 *   - aes_last_error() returns a static, thread-local, human-readable message
 *     for the last failing call of the calling thread.
 *   - Matrices are row-major.  Leading dimensions (ldx, ldq, ldy) are counted
 *     in elements and must be >= the row length; the leading dimension of a
 *     gathered feature matrix (X, Xq) must be below 2^32 (AES_ERR_UNSUPPORTED).
 *   - Within-row order of CSR entries is the caller's; the sampling takes runs
 *     of consecutive entries, so results depend on it.  Nothing is sorted.
 */
#ifndef AES_SPMM_H
#define AES_SPMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum aes_status {
    AES_OK = 0,
    AES_ERR_INVALID_ARG = -1,  /* NULL pointer, negative size, bad enum, bad ld  */
    AES_ERR_UNSUPPORTED = -2,  /* size beyond what the kernels index             */
    AES_ERR_WORKSPACE = -3,    /* workspace NULL or smaller than the query says  */
    AES_ERR_HIP = -4           /* HIP reported an error at launch                */
} aes_status;

/* Group that shares one (scale, zero) pair. */
typedef enum aes_q_granularity {
    AES_Q_PER_TENSOR = 0,      /* 1 group                                        */
    AES_Q_PER_COLUMN = 1,      /* F groups, one per feature column               */
    AES_Q_PER_ROW = 2,         /* n groups, one per node                         */
    AES_Q_PER_ROW_FOLDED = 3,  /* aes_spmm_q8 only: per-node constants already    */
                               /* folded into the plan's values, see              */
                               /* aes_plan_fold_row_constants                     */
    AES_Q_PER_ROW_INLINE = 4   /* n groups, one per node, the constants stored in  */
                               /* the node's own row of codes: see below           */
} aes_q_granularity;

/*
 * AES_Q_PER_ROW_INLINE: per-node constants that travel with the node's codes.
 * Row i of Xq holds its F codes, padding up to byte 4*ceil(F/4), there the
 * float32 scale of node i and, for AES_Q_AFFINE_FLOOR_U8, its float32 zero
 * point in the next four bytes.  It needs ldq >= 4*ceil(F/4) + 4 (+ 8 for the
 * affine scheme), ldq a multiple of 4 and Xq 4-byte aligned (else
 * AES_ERR_INVALID_ARG); the scale / zero arguments are ignored and may be NULL.
 * Why: with AES_Q_PER_ROW the multiply gathers scale[col] for every slot from
 * an array of its own, a second memory line per slot.  Inside the row the
 * constants come with a line the gather fetches anyway WHEN THE ROW HAS ROOM
 * for them in its last 128-byte line (F = 100, 500, 602 ... with ldq rounded up
 * to a multiple of 128); a row of exactly 128 or 256 codes has none, its
 * constants would start a line of their own, and AES_Q_PER_ROW (or the folded
 * plan) is the better choice there.  aes_quantize_inline_ld gives the smallest
 * such leading dimension that is a multiple of 128.
 */
int64_t aes_quantize_inline_ld(int32_t F, int32_t scheme);

typedef enum aes_q_scheme {
    /* Sec. 2.3 Eq. 1-2 with b = 8: q = floor((x-x_min)/(x_max-x_min)*255) in
     * 0..255 (uint8 bit pattern), x_hat = q*scale + zero with
     * scale = (x_max-x_min)/255, zero = x_min.  x_max == x_min gives q = 0. */
    AES_Q_AFFINE_FLOOR_U8 = 0,
    /* Symmetric variant: a = max|x|, scale = a/127 (1 if a == 0),
     * q = round-half-even(x/scale) clamped to -127..127, x_hat = q*scale. */
    AES_Q_SYMMETRIC_RNE_I8 = 1
} aes_q_scheme;

/* How a row with more than W entries is sampled (Sec. 3.3). */
typedef enum aes_strategy {
    AES_STRATEGY_ADAPTIVE = 0, /* Table 1: (N, sample_cnt) from R = row_nnz / W    */
    AES_STRATEGY_AFS = 1,      /* N = 1, sample_cnt = W: fine-grained, the paper's  */
                               /* description of ES-SpMM's accuracy-first strategy  */
    AES_STRATEGY_SFS = 2       /* N = W, sample_cnt = 1: coarse-grained, speed-first */
} aes_strategy;

enum { AES_MAX_W = 1 << 20 };

/* Message of the calling thread's last failing call ("" if none). */
const char *aes_last_error(void);

/* ------------------------------------------------------------------------- */
/* Sampling: CSR -> sampled plan (Algorithm 1 sampling loop, Table 1, Eq. 3)  */

/*
 * Upper bound, computable without reading device memory, on the number of
 * slots aes_sample_build writes: min(nnz, n_rows * W), or nnz when W == 0.
 * s_col / s_val / s_eid must have at least this many elements.
 * Returns a negative aes_status on bad arguments.
 */
int64_t aes_sample_capacity(int64_t n_rows, int64_t nnz, int32_t W);

/* Bytes of device workspace aes_sample_build needs for n_rows rows. */
size_t aes_sample_workspace_bytes(int64_t n_rows);

/*
 * Builds the sampled matrix A_s of CSR matrix A (Sec. 2.2 format).
 *
 * For each row r with row_nnz = rowptr[r+1] - rowptr[r]:
 *   (N, sample_cnt) follow Table 1 from R = row_nnz / W (real ratio), with
 *   N >= 1 and sample_cnt <= W; rows with row_nnz <= W keep every entry.
 *   Sample i (0 <= i < sample_cnt) starts at
 *       start_i = ((i + s_r) * 1429) mod (row_nnz - N + 1)            (Eq. 3)
 *   and slot i + j*sample_cnt (0 <= j < N) receives entry start_i + j of the
 *   row (Algorithm 1, sampling loop).  s_r is a per-row offset derived from
 *   `seed` (low 32 bits of seed*(2r+1)*2654435761); seed == 0 gives s_r == 0,
 *   i.e. exactly Eq. 3.  Overlapping samples are kept; nothing de-duplicates.
 *   Row r owns N*sample_cnt slots (== min(row_nnz, W) when W is a power of
 *   two), stored at s_rowptr[r] .. s_rowptr[r+1]-1.
 * W == 0 selects "no sampling": the plan is a copy of the CSR matrix.
 *
 *   n_rows, n_cols  matrix shape; n_rows >= 0, 0 <= n_cols < 2^31
 *   nnz             stored entries of A; >= 0
 *   rowptr   [dev]  n_rows+1 int64
 *   colidx   [dev]  nnz int32
 *   val      [dev]  nnz float32
 *   W               sampling width, 0 or 1..AES_MAX_W (any integer)
 *   seed            see above
 *   strategy        aes_strategy; ADAPTIVE is the paper's method, AFS / SFS
 *                   replace Table 1 by the fixed (N, sample_cnt) named there
 *   s_rowptr [dev]  out, n_rows+1 int64
 *   s_col    [dev]  out, aes_sample_capacity() int32
 *   s_val    [dev]  out, same count, float32 (bit copies of val)
 *   s_eid    [dev]  out or NULL, same count, int64: index into colidx/val each
 *                   slot was taken from
 *   row_perm [dev]  out or NULL, n_rows int32: the rows ordered by decreasing
 *                   slot-count class (class = bit length of the slot count),
 *                   original order kept within a class.  A scheduling hint for
 *                   the SpMM entry points; requires n_rows < 2^31.
 *   workspace[dev]  aes_sample_workspace_bytes(n_rows) bytes, 8-byte aligned
 */
int aes_sample_build(int64_t n_rows, int64_t n_cols, int64_t nnz,
                     const int64_t *rowptr, const int32_t *colidx, const float *val,
                     int32_t W, uint64_t seed, int32_t strategy,
                     int64_t *s_rowptr, int32_t *s_col, float *s_val, int64_t *s_eid,
                     int32_t *row_perm,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * aes_sample_build for callers that cannot allocate device memory and have no
 * workspace to hand over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments (minus the workspace), same
 * kernels, same results bit for bit; the workspace is a fixed array inside the
 * library's code object (2 228 232 bytes, resident on every GPU the library is
 * used on until the process ends) whose device address is looked up once per
 * device, on the first call made with that device current.  The call allocates
 * and frees nothing.
 *
 *   n_rows          at most AES_NOALLOC_MAX_ROWS, else AES_ERR_UNSUPPORTED
 *                   (nothing is launched)
 * All calls on one GPU share that GPU's array: calls that may overlap in time
 * (different streams, different host threads) race on it and must be
 * serialised by the caller.  Nothing in it has to survive or be cleared between
 * calls: every element a kernel reads is written earlier in the same call.
 */
enum { AES_NOALLOC_MAX_ROWS = 1 << 24 };
int aes_sample_build_noalloc(int64_t n_rows, int64_t n_cols, int64_t nnz,
                             const int64_t *rowptr, const int32_t *colidx, const float *val,
                             int32_t W, uint64_t seed, int32_t strategy,
                             int64_t *s_rowptr, int32_t *s_col, float *s_val, int64_t *s_eid,
                             int32_t *row_perm, void *stream);

/* ------------------------------------------------------------------------- */
/* Multiply stage (Algorithm 1, accumulation loop) on a plan                   */

/*
 * Y[r, c] = sum_k s_val[k] * X[s_col[k], c] over the slots k of row r, for
 * 0 <= c < F.  float32 accumulation by fused multiply-add in slot order (float64
 * for the long rows described under W); the summation order within a row is
 * fixed, so results are bit-reproducible from run to run.
 * Rows without slots give zero rows.  Every element of Y[0..n_rows, 0..F) is
 * written; padding columns F..ldy are not touched.
 *
 *   n_rows, n_cols  shape of A_s; X has n_cols rows
 *   W               the width the plan was built with: an upper bound on the
 *                   slots of any row, or 0 when there is none (unsampled plan,
 *                   plain CSR).  It only selects the kernel variant: with
 *                   W == 0 or W > 2048 rows longer than 2048 slots are shared by
 *                   all wavefronts of a workgroup (partial sums carried in
 *                   float64 and added in a fixed order) instead of being left
 *                   to one lane group.  A row with more slots than a non-zero
 *                   W states is still computed correctly, only without that
 *                   sharing.
 *   s_rowptr/s_col/s_val [dev]  a plan from aes_sample_build (or any CSR with
 *                   int64 rowptr, int32 colidx, float32 val); s_col / s_val may
 *                   be NULL only when the plan has no slots at all
 *   row_perm [dev]  NULL, or a permutation of 0..n_rows-1 giving the order in
 *                   which rows are handed to wavefronts (from aes_sample_build)
 *   X        [dev]  n_cols x F float32, leading dimension ldx
 *   Y        [dev]  out, n_rows x F float32, leading dimension ldy; must not
 *                   overlap X
 *   F               1 <= F < 2^24
 * No alignment beyond that of a float is required of X, Y, ldx or ldy (rows that
 * start on 16-byte boundaries touch the fewest memory lines).  Columns
 * 0 .. 4*floor(F/4) - 1 are computed four per lane; the last F % 4 columns, if
 * any, by a second, element-wise launch over the same plan (same results).
 */
int aes_spmm_f32(int64_t n_rows, int64_t n_cols, int32_t W,
                 const int64_t *s_rowptr, const int32_t *s_col, const float *s_val,
                 const int32_t *row_perm,
                 const float *X, int64_t ldx, int32_t F,
                 float *Y, int64_t ldy, void *stream);

/* ------------------------------------------------------------------------- */
/* Feature quantisation (Sec. 2.3 Eq. 1; once per feature matrix)              */

/* Bytes of device workspace aes_quantize_features needs (0 for PER_ROW). */
size_t aes_quantize_workspace_bytes(int64_t n, int32_t F, int32_t granularity);

/*
 * Quantises X (n x F float32) to 8 bits per value, see aes_q_scheme.  All
 * arithmetic is IEEE binary32 with one rounding per operation (subtract,
 * divide, multiply, floor / divide, round-half-even), so the codes are
 * bit-reproducible on any conforming implementation.  NaN/Inf inputs give
 * unspecified codes.
 *
 *   X     [dev]  n x F float32, leading dimension ldx
 *   Xq    [dev]  out, n x F bytes, leading dimension ldq (uint8 bit pattern
 *                for AFFINE_FLOOR_U8, int8 for SYMMETRIC_RNE_I8)
 *   scale [dev]  out, 1 | F | n float32 according to granularity
 *   zero  [dev]  out, same count; may be NULL for SYMMETRIC_RNE_I8 (written
 *                as 0 otherwise).  AES_Q_PER_ROW_INLINE: both ignored, the
 *                constants are written into the rows of Xq
 *   workspace [dev] aes_quantize_workspace_bytes() bytes, 4-byte aligned; may
 *                be NULL when that is 0
 */
int aes_quantize_features(int64_t n, int32_t F, const float *X, int64_t ldx,
                          int32_t scheme, int32_t granularity,
                          int8_t *Xq, int64_t ldq, float *scale, float *zero,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * Sec. 2.3 Eq. 2 as a stand-alone pass, where the paper places it (after the
 * 8-bit features have been loaded, before the SpMM): X[i, c] = q*scale_g +
 * zero_g (AFFINE_FLOOR_U8) or q*scale_g (SYMMETRIC_RNE_I8); multiply, then add,
 * in binary32, so the result is bit-reproducible.  aes_spmm_q8 makes this pass
 * unnecessary; it exists to measure what the fusion saves.
 *
 *   Xq [dev] n x F bytes (ldq); scale, zero [dev] as written by
 *   aes_quantize_features (zero may be NULL for SYMMETRIC_RNE_I8; both
 *   ignored for AES_Q_PER_ROW_INLINE); X [dev] out, n x F float32 (ldx)
 */
int aes_dequantize_features(int64_t n, int32_t F, const int8_t *Xq, int64_t ldq,
                            int32_t scheme, int32_t granularity,
                            const float *scale, const float *zero,
                            float *X, int64_t ldx, void *stream);

/* ------------------------------------------------------------------------- */
/* Multiply stage with the dequantisation of Eq. 2 fused into the gather       */

/*
 * Y[r, c] = sum_k s_val[k] * x_hat[s_col[k], c], where
 * x_hat = q*scale_g + zero_g (AFFINE_FLOOR_U8) or q*scale_g (SYMMETRIC_RNE_I8)
 * and g is the group of element (s_col[k], c).  The group constants are
 * factored out of the inner loop (per column: applied once per output; per
 * row: folded into the edge value), so the result equals the dequantise-then-
 * multiply definition up to float32 rounding, not bit for bit.
 *
 *   Xq    [dev]  n_cols x F bytes, leading dimension ldq
 *   scale, zero [dev]  as written by aes_quantize_features; zero may be NULL
 *                for SYMMETRIC_RNE_I8 (for AES_Q_PER_ROW_FOLDED see
 *                aes_plan_fold_row_constants; ignored for
 *                AES_Q_PER_ROW_INLINE, which reads them from the rows of Xq)
 * Other arguments as aes_spmm_f32, including the treatment of F % 4 columns;
 * Xq and ldq need no particular alignment.
 */
int aes_spmm_q8(int64_t n_rows, int64_t n_cols, int32_t W,
                const int64_t *s_rowptr, const int32_t *s_col, const float *s_val,
                const int32_t *row_perm,
                const int8_t *Xq, int64_t ldq, int32_t F,
                int32_t scheme, int32_t granularity,
                const float *scale, const float *zero,
                float *Y, int64_t ldy, void *stream);

/*
 * Folds per-node (AES_Q_PER_ROW) dequantisation constants into a plan, for a
 * plan that multiplies the same quantised feature matrix more than once.  With
 * per-node scales aes_spmm_q8 gathers scale[s_col[k]] for every slot, and that
 * 4-byte gather costs a whole 128-byte memory line, as much as a 128-feature
 * row of codes.  After
 *     s_val_folded[k] = s_val[k] * scale[s_col[k]]
 *     row_bias[r]     = sum over the slots k of row r of s_val[k] * zero[s_col[k]]
 * (the second only for AES_Q_AFFINE_FLOOR_U8), calling aes_spmm_q8 with
 * s_val = s_val_folded, granularity = AES_Q_PER_ROW_FOLDED, scale ignored (may be
 * NULL) and zero = row_bias (NULL for the symmetric scheme) computes the same
 * Y = sum_k s_val[k] * (q * scale + zero) without touching scale or zero again.
 *
 *   s_rowptr/s_col/s_val [dev]  the plan; n_rows rows
 *   scale, zero [dev]           per-node constants (n_cols entries); zero may be
 *                               NULL for AES_Q_SYMMETRIC_RNE_I8
 *   s_val_folded [dev]          out, as many floats as the plan has slots; may
 *                               alias s_val
 *   row_bias     [dev]          out, n_rows floats; required for the affine
 *                               scheme, ignored (may be NULL) otherwise
 */
int aes_plan_fold_row_constants(int64_t n_rows,
                                const int64_t *s_rowptr, const int32_t *s_col, const float *s_val,
                                int32_t scheme, const float *scale, const float *zero,
                                float *s_val_folded, float *row_bias, void *stream);

/* ------------------------------------------------------------------------- */
/* Algorithm 1 as one kernel: sample each row on the fly, then multiply        */

/*
 * Same result as aes_sample_build followed by aes_spmm_f32 / aes_spmm_q8 (bit
 * for bit: same slots, same summation order), without materialising the plan:
 * each lane group evaluates Table 1 and Eq. 3 for its row and stages the
 * sampled (col, val) pairs straight from the CSR arrays into LDS - the single
 * kernel shape of Sec. 3.2.  Saves the plan's write and read when a plan would
 * be used once.  Arguments as in the calls named above.
 */
int aes_spmm_fused_f32(int64_t n_rows, int64_t n_cols,
                       const int64_t *rowptr, const int32_t *colidx, const float *val,
                       int32_t W, uint64_t seed, int32_t strategy,
                       const float *X, int64_t ldx, int32_t F,
                       float *Y, int64_t ldy, void *stream);

int aes_spmm_fused_q8(int64_t n_rows, int64_t n_cols,
                      const int64_t *rowptr, const int32_t *colidx, const float *val,
                      int32_t W, uint64_t seed, int32_t strategy,
                      const int8_t *Xq, int64_t ldq, int32_t F,
                      int32_t scheme, int32_t granularity,
                      const float *scale, const float *zero,
                      float *Y, int64_t ldy, void *stream);

/* ------------------------------------------------------------------------- */
/* One GNN layer: aggregation (Sec. 3.2) and combination (Sec. 2.1) fused      */

/*
 * H = (A_s X) Theta: the sampled aggregation of aes_spmm_f32 followed by the
 * layer's dense weight matrix, in one kernel.  A workgroup aggregates 32 rows of
 * A_s X into LDS (float32, same summation order as aes_spmm_f32) and multiplies
 * them by Theta on the matrix cores (float32 MFMA, float32 accumulate); the
 * aggregated features are never written to memory.  No bias, no activation.
 *
 *   plan, W         as for aes_spmm_f32, including the treatment of rows above
 *                   2048 slots when W == 0 or W > 2048 (shared by the
 *                   workgroup, float64 partial sums in a fixed order)
 *   X     [dev]     n_cols x F float32 (ldx); any F in 1 .. 2^24-1, no alignment
 *                   needed beyond a float's.  F <= 256 with F % 4 == 0 (and a W
 *                   that rules out long rows) runs a specialised kernel that
 *                   holds whole aggregated rows in LDS; any other shape walks
 *                   the features in chunks of 256 and keeps the MFMA
 *                   accumulators in registers across the chunks
 *   Theta [dev]     F x Fo float32, row-major, leading dimension ldt; output
 *                   columns beyond 512 take one more launch per 512 (each
 *                   aggregates again)
 *   H     [dev]     out, n_rows x Fo float32 (ldh); must not overlap the inputs
 */
int aes_gcn_layer_f32(int64_t n_rows, int64_t n_cols, int32_t W,
                      const int64_t *s_rowptr, const int32_t *s_col, const float *s_val,
                      const float *X, int64_t ldx, int32_t F,
                      const float *Theta, int64_t ldt, int32_t Fo,
                      float *H, int64_t ldh, void *stream);

/*
 * The same layer on 8-bit features: H = (A_s x_hat) Theta with the dequantisation of Sec. 2.3
 * Eq. 2 fused into the gather exactly as in aes_spmm_q8 (same scheme / granularity / scale /
 * zero arguments, AES_Q_PER_ROW_FOLDED and AES_Q_PER_ROW_INLINE included), the aggregated tile multiplied by Theta on
 * the matrix cores.  Any F, as for aes_gcn_layer_f32; Xq and ldq need no particular alignment.
 */
int aes_gcn_layer_q8(int64_t n_rows, int64_t n_cols, int32_t W,
                     const int64_t *s_rowptr, const int32_t *s_col, const float *s_val,
                     const int8_t *Xq, int64_t ldq, int32_t F,
                     int32_t scheme, int32_t granularity, const float *scale, const float *zero,
                     const float *Theta, int64_t ldt, int32_t Fo,
                     float *H, int64_t ldh, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* AES_SPMM_H */
