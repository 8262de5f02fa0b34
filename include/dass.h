/*
 * libdass -- the data-parallel hot path of DaSS pruning for GLU-variant MLPs
 * (Guo et al., "Dependency-aware Semi-structured Sparsity of GLU Variants in
 * Large Language Models", arXiv 2405.01943) on AMD gfx950.
 *
 * C ABI: plain pointers and sizes only.
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or synchronises.  Work is enqueued on
 *     `hip_stream` (a hipStream_t passed as void*; NULL = the default stream)
 *     and calls are ordered by that stream.
 *   - Matrices are row-major in the paper's transposed layout (Sec. 3):
 *     Gate-Proj and Up-Proj are [d_int, d_hidden], Down-Proj is
 *     [d_hidden, d_int]; `ld*` is the row stride in elements.
 *   - Data pointers must be 16-byte aligned and row strides a multiple of
 *     8 elements (bf16) or 4 elements (f32); otherwise DASS_ERR_ALIGN.
 *   - All argument checks happen on the host before the first HIP call, so a
 *     rejected call has touched nothing.
 *   - Inputs must be finite.  The result for NaN or Inf inputs is undefined.
 *   - Thread safe; the only library state is a thread-local error string
 *     (and, for dass_score_mask_unstructured_static, one device array).
 *     Calls enqueued on different streams may run at the same time as long
 *     as no buffer one of them writes (its matrix, outputs, workspace) is
 *     used by another; a call's several launches are ordered by its stream.
 */
#ifndef DASS_H
#define DASS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The enumerations below are plain C enums.  A C++ translation unit gives them the fixed
 * underlying type int (what a C caller passes): a value outside the list, which every entry point
 * must answer with an error code, is then an ordinary value there and not undefined behaviour. */
#ifdef __cplusplus
#define DASS_ENUM(name) enum name : int
#else
#define DASS_ENUM(name) enum name
#endif

typedef DASS_ENUM(dass_status) {
    DASS_OK = 0,
    DASS_ERR_NULL = 1,      /* a required pointer is NULL                        */
    DASS_ERR_SHAPE = 2,     /* non-positive size, ld < width, ragged group axis  */
    DASS_ERR_DTYPE = 3,     /* dtype or activation enum out of range             */
    DASS_ERR_ARG = 4,       /* bad (n_keep, m), alpha, n_prune                   */
    DASS_ERR_ALIGN = 5,     /* pointer or stride alignment                       */
    DASS_ERR_WORKSPACE = 6, /* workspace missing or too small                    */
    DASS_ERR_HIP = 7        /* a HIP launch failed; see dass_last_error_string() */
} dass_status;

typedef DASS_ENUM(dass_dtype) { DASS_F32 = 0, DASS_BF16 = 1 } dass_dtype;

/* sigma(.) of Sec. 2.2 Eq. 2: Swish (beta = 1) for SwiGLU, GeLU (tanh or erf
 * form) for GeGLU, ReLU for ReGLU. */
typedef DASS_ENUM(dass_act) {
    DASS_ACT_SILU = 0,
    DASS_ACT_GELU_TANH = 1,
    DASS_ACT_GELU_ERF = 2,
    DASS_ACT_RELU = 3
} dass_act;

/* A dimension of a row-major matrix W[rows, cols]. */
typedef DASS_ENUM(dass_axis) { DASS_AXIS_ROWS = 0, DASS_AXIS_COLS = 1 } dass_axis;

/*
 * Stage 1 -- calibration statistics (Sec. 2.2 Eq. 2 and Sec. 3 "Incorporating
 * Dependency into Weight Importance": the group-importance indicator is the L2
 * norm of the intermediate activation y, taken over all calibration tokens).
 *
 *   for every intermediate neuron i:
 *     sumsq[i] (+)= sum over t of ( act(X[t,:] . Wgate[i,:]) * (X[t,:] . Wup[i,:]) )^2
 *     norms_out[i] = sqrt(sumsq[i])                          (if norms_out != NULL)
 *
 * The products X Wgate^T and X Wup^T are accumulated in f32 and y is never
 * written to memory.
 *
 *   X      [T, d]      row stride ldx, read only, dtype dt
 *   Wgate  [d_int, d]  row stride ldw, read only, dtype dt
 *   Wup    [d_int, d]  row stride ldw, read only, dtype dt
 *   sumsq  [d_int] f32, in/out: the only carried state.  accumulate = 0
 *          overwrites it, accumulate = 1 adds this call's tokens to it, so a
 *          calibration set can be streamed in chunks (or resumed from a saved
 *          copy of sumsq).
 *   norms_out [d_int] f32 or NULL.
 *   workspace  device scratch of at least dass_calib_workspace_bytes() bytes
 *          (may be NULL when that is 0).
 *
 * d must be a multiple of 8 (bf16) or 4 (f32).  T, d_int are arbitrary positive.
 * The accumulation over tokens uses f32 atomics, so results can differ in the
 * last bits from run to run.
 */
size_t dass_calib_workspace_bytes(int64_t T, int64_t d, int64_t d_int, dass_dtype dt);

dass_status dass_calib_norms(const void *X, int64_t T, int64_t ldx,
                             const void *Wgate, const void *Wup, int64_t ldw,
                             int64_t d, int64_t d_int, dass_dtype dt, dass_act act,
                             float *sumsq, int accumulate, float *norms_out,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Stage 2 -- DaSS scoring with N:M selection (Sec. 3 Eq. 4, Eq. 5 and
 * "Extension to N:M Sparsity").
 *
 *   score[r, c] = |W[r, c]| * f[k],  f = norms^alpha,
 *                 k = r if norm_axis = ROWS, c if norm_axis = COLS
 *
 * In every group of m consecutive positions along group_axis (groups start at
 * index 0) the n_keep positions of highest score are left untouched and the
 * other m - n_keep are overwritten with +0, IN PLACE.  Equal scores: the lower
 * index along the group is kept.  Scores are compared exactly (as the real
 * product of the stored weight and the f32 factor), never after rounding.
 *
 * DaSS uses  Gate/Up: norm_axis = group_axis = ROWS, alpha = 0.5  (Eq. 4,
 *                     input-balanced groups: m consecutive neurons per input)
 *            Down:    norm_axis = group_axis = COLS, alpha = 1    (Eq. 5,
 *                     output-balanced groups).
 *
 *   W      [rows, cols] row stride ld, dtype dt, modified in place
 *   norms  f32, length rows (norm_axis = ROWS) or cols (COLS), read only
 *   alpha  finite, >= 0.  f = 1 for alpha = 0 (also where the norm is 0),
 *          norms for alpha = 1, the correctly rounded f32 square root for 0.5,
 *          otherwise pow() evaluated in f64 and rounded to f32.
 *   m in {2, 4, 8, 16}, 0 < n_keep < m; the length of group_axis must be a
 *          multiple of m (else DASS_ERR_SHAPE); cols must be a multiple of 8.
 *   mask_out NULL, or rows * (cols / 8) bytes: bit (c & 7) of byte c / 8 of
 *          row r is 1 iff W[r, c] was kept.
 *   workspace  device scratch of at least dass_nm_workspace_bytes() bytes,
 *          16-byte aligned; it receives the factor vector f.  Calls that run
 *          concurrently on different streams need separate workspaces.
 */
size_t dass_nm_workspace_bytes(int64_t rows, int64_t cols, dass_axis norm_axis);

dass_status dass_score_mask_nm(void *W, int64_t rows, int64_t cols, int64_t ld, dass_dtype dt,
                               const float *norms, dass_axis norm_axis, dass_axis group_axis,
                               double alpha, int n_keep, int m, uint8_t *mask_out,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Stage 2 for many matrices at once: the N:M masks of all MLP matrices of a
 * model (Sec. 4.5 times the pruning of a whole model; its layers are
 * independent, Sec. 3).  Every task is what one dass_score_mask_nm() call
 * would do, with n_keep:m and dt common to all tasks; the result is the same
 * bit for bit.  Tasks of equal shape, axes and exponent that take the one-pass
 * path (2 n_keep = m <= 8, alpha in {0, 0.5, 1}) share kernel launches, up to
 * 96 matrices per launch, so no launch gap separates their ~30 us of work;
 * any other task is run as a call of its own, in the order given.
 *
 *   tasks      HOST array of n_tasks descriptors (read before the call
 *              returns); W, norms, mask_out are DEVICE pointers as in
 *              dass_score_mask_nm().  The matrices must not overlap.
 *   workspace  device scratch of at least dass_nm_batched_workspace_bytes()
 *              bytes (the largest single-task need), 16-byte aligned.
 *   On an invalid task nothing is launched and the error names its index.
 */
typedef struct {
    void *W;
    int64_t rows, cols, ld;
    const float *norms;
    dass_axis norm_axis, group_axis;
    double alpha;
    uint8_t *mask_out; /* NULL or rows * (cols / 8) bytes */
} dass_nm_task;

size_t dass_nm_batched_workspace_bytes(const dass_nm_task *tasks, int64_t n_tasks);

dass_status dass_score_mask_nm_batched(const dass_nm_task *tasks, int64_t n_tasks, dass_dtype dt,
                                       int n_keep, int m, void *workspace,
                                       size_t workspace_bytes, void *hip_stream);

/*
 * The input-feature norms of the Wanda metric (Sec. 2.1 Eq. 1): for every
 * input feature j the L2 norm of X[:, j] over all tokens,
 *
 *   sumsq[j] (+)= sum_t X[t, j]^2,      norms_out[j] = sqrt(sumsq[j]).
 *
 * With these norms, dass_score_mask_nm(W, ..., norm_axis = group_axis = COLS,
 * alpha = 1) on a [d_out, d_in] matrix is the paper's comparison system
 * (output-balanced |W| * ||X_j||, Eq. 1), and Eq. 5 is the same call on
 * Down-Proj with the stage-1 norms.
 *
 *   X      [T, d] row stride ldx, dtype dt, read only; d a multiple of 8
 *   sumsq  f32[d]; overwritten, or added to when accumulate != 0 (token chunks)
 *   norms_out  NULL or f32[d]
 *   workspace  device scratch of at least dass_input_norms_workspace_bytes()
 *          bytes, 16-byte aligned (per-row-block partial sums; the result does
 *          not depend on scheduling)
 * Squares and block sums are f32, the sum over blocks f64.
 */
size_t dass_input_norms_workspace_bytes(int64_t T, int64_t d);

dass_status dass_input_norms(const void *X, int64_t T, int64_t ldx, int64_t d, dass_dtype dt,
                             float *sumsq, int accumulate, float *norms_out, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/*
 * Stage 2 -- DaSS scoring with per-line unstructured selection (Sec. 3
 * "Pruning Granularity": weights are compared for each input individually for
 * Gate/Up, for each output individually for Down, and the lowest scores of
 * each comparison group are pruned).
 *
 * Every full line along group_axis (a column of W when group_axis = ROWS, a
 * row when group_axis = COLS) is one comparison group.  Its n_prune positions
 * of lowest score are overwritten with +0 in place; among equal scores the
 * higher index is pruned first.  Scores, factor, mask_out as above; the caller
 * converts a sparsity ratio s to n_prune = floor(s * line length).
 *
 *   workspace  device scratch of at least dass_unstructured_workspace_bytes()
 *              bytes, 16-byte aligned.  It holds f; for column lines
 *              (group_axis = ROWS) of a large matrix also the counts and short
 *              lists of the passes that select them tile by tile (a few tens
 *              of MB for a 7B-sized matrix), or, where those passes do not
 *              apply and a line has more than 16384 bf16 / 8192 f32 weights,
 *              a transposed copy of W (rows * cols elements) on which such
 *              lines are selected.  Its contents after the call are unspecified.
 */
size_t dass_unstructured_workspace_bytes(int64_t rows, int64_t cols, dass_dtype dt,
                                         dass_axis norm_axis, dass_axis group_axis);

dass_status dass_score_mask_unstructured(void *W, int64_t rows, int64_t cols, int64_t ld,
                                         dass_dtype dt, const float *norms,
                                         dass_axis norm_axis, dass_axis group_axis,
                                         double alpha, int64_t n_prune, uint8_t *mask_out,
                                         void *workspace, size_t workspace_bytes,
                                         void *hip_stream);

/*
 * dass_score_mask_unstructured for callers that cannot allocate device memory
 * and so have no workspace to pass: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments (without
 * the workspace), same result bit for bit.  The factor vector f lives in a
 * device array of the library's own, 65536 floats (256 KB) on every GPU the
 * library is used on, held until the process ends; its address is looked up
 * on the first call on a device (hipGetSymbolAddress).  Nothing is allocated
 * or freed, by this call or by anything it calls.
 *
 *   - The norm axis may be at most 65536 long; beyond that DASS_ERR_WORKSPACE
 *     (use dass_score_mask_unstructured with a workspace).
 *   - Column lines of more than 16384 bf16 / 8192 f32 weights are selected
 *     by the multi-pass kernels (no room for the transposed copy): correct,
 *     slower.
 *   - All calls on one GPU share the one array: calls that may overlap there
 *     (different streams, different threads) race on it; calls in stream
 *     order on one stream do not.  Every call rewrites the part it reads, so
 *     nothing needs clearing between calls.
 */
dass_status dass_score_mask_unstructured_static(void *W, int64_t rows, int64_t cols, int64_t ld,
                                                dass_dtype dt, const float *norms,
                                                dass_axis norm_axis, dass_axis group_axis,
                                                double alpha, int64_t n_prune,
                                                uint8_t *mask_out, void *hip_stream);

/*
 * The output of the MLP block (Sec. 2.2 Eq. 2 followed by Eq. 3):
 *
 *   y[t, i]   = act(x_t . Wgate_i) * (x_t . Wup_i)
 *   out[t, j] = sum_i y[t, i] * Wdown[j, i]
 *
 * With pruned weights this is the input the next block is calibrated on when
 * blocks are pruned one after the other.
 *
 *   X      [T, d] row stride ldx;  Wgate, Wup [d_int, d] row stride ldw;
 *   Wdown  [d, d_int] row stride ldd;  all device, read only
 *   out    [T, d] row stride ldo, device, overwritten
 *   workspace  device scratch of at least dass_mlp_forward_workspace_bytes()
 *          bytes, 16-byte aligned: y, [T, d_int] in dtype dt (callers short of
 *          memory split the tokens: rows are independent)
 * dt: DASS_BF16 only (DASS_ERR_DTYPE otherwise).  Products accumulate in f32;
 * y is rounded to bf16 once (round to nearest even), out once.  d and d_int
 * must be multiples of 64 (DASS_ERR_SHAPE), pointers 16-byte aligned and
 * leading dimensions multiples of 8 (DASS_ERR_ALIGN).  Two launches on
 * hip_stream; nothing is allocated.
 * Wdown may be NULL: then only Eq. 2 runs and y is left in the workspace as
 * [T, d_int] row-major (out, ldd and ldo are not looked at) - the input of
 * dass_down_proj_sparse24 below.
 */
size_t dass_mlp_forward_workspace_bytes(int64_t T, int64_t d, int64_t d_int, dass_dtype dt);

dass_status dass_mlp_forward(const void *X, int64_t T, int64_t ldx, const void *Wgate,
                             const void *Wup, int64_t ldw, const void *Wdown, int64_t ldd,
                             int64_t d, int64_t d_int, dass_dtype dt, dass_act act, void *out,
                             int64_t ldo, void *workspace, size_t workspace_bytes,
                             void *hip_stream);

/*
 * The 2:4 pattern (Sec. 2.2 "N:M sparsity" with N = 2, M = 4) in compressed
 * form: per group of 4 consecutive positions along group_axis, two values
 * and their two 2-bit positions, which is what sparse matrix units read.
 *
 * A group's stored positions are the first two entries of (positions holding
 * a nonzero, ascending) followed by (positions holding a zero, ascending),
 * in ascending order p0 < p1; its code is the nibble p0 | p1 << 2.  A matrix
 * with at most two nonzeros per group is represented exactly (-0 counts as
 * zero).
 *
 *   W      [rows, cols] row stride ld, dtype dt, device, read only
 *   group_axis = DASS_AXIS_COLS: values_out [rows, cols / 2] row stride ldv:
 *          group g of row r fills values[r, 2 g] and [r, 2 g + 1];
 *          meta_out [rows, cols / 8] bytes, row stride ldm: the code of group
 *          g is nibble (g & 1) of byte g / 2 of row r.  cols % 8 == 0; ldv a
 *          multiple of 4 elements, ldm any.
 *   group_axis = DASS_AXIS_ROWS: values_out [rows / 2, cols]: group g of
 *          column c fills values[2 g, c] and [2 g + 1, c]; meta_out
 *          [rows / 4, cols / 2] bytes: the code of group g of column c is
 *          nibble (c & 1) of byte c / 2 of row g.  rows % 4 == 0, cols % 8 == 0;
 *          ldv a multiple of 8 (bf16) / 4 (f32) elements, meta_out 4-byte
 *          aligned and ldm a multiple of 4.
 *   values_out  dtype dt, device, 16-byte aligned; must not overlap W
 *   meta_out    device
 *   surplus_out NULL, or one device int64 to which the number of groups that
 *          held more than two nonzeros is ADDED (their surplus is dropped)
 */
dass_status dass_compress_24(const void *W, int64_t rows, int64_t cols, int64_t ld, dass_dtype dt,
                             dass_axis group_axis, void *values_out, int64_t ldv,
                             uint8_t *meta_out, int64_t ldm, long long *surplus_out,
                             void *hip_stream);

/*
 * Eq. 3 (Sec. 2.2) from the compressed Down-Proj: out = Y Wdown^T, Wdown given
 * as dass_compress_24(..., group_axis = DASS_AXIS_COLS) wrote it, evaluated
 * on the sparse matrix cores - the hardware use of 2:4 sparsity that Sec. 2.2
 * names.
 *
 *   Y       [T, d_int] row stride ldy (the y of Eq. 2), device, read only
 *   values  [d, d_int / 2] row stride ldv;  meta [d, d_int / 8] bytes, row
 *           stride ldm: the compressed form, device, read only
 *   out     [T, d] row stride ldo, device, overwritten
 * dt: DASS_BF16 only.  Products accumulate in f32, out is rounded to bf16 once.
 * d_int a multiple of 64, d of 8 (DASS_ERR_SHAPE); Y, values, out 16-byte
 * aligned with leading dimensions multiples of 8, meta 4-byte aligned with
 * ldm a multiple of 4 (DASS_ERR_ALIGN).  One launch on hip_stream.
 */
dass_status dass_down_proj_sparse24(const void *Y, int64_t T, int64_t ldy, const void *values,
                                    int64_t ldv, const uint8_t *meta, int64_t ldm, int64_t d,
                                    int64_t d_int, dass_dtype dt, void *out, int64_t ldo,
                                    void *hip_stream);

/* Name of a status code; never NULL. */
const char *dass_status_string(dass_status s);
/* Detail of the calling thread's most recent failed call ("" if none). */
const char *dass_last_error_string(void);
/* Library version, major * 10000 + minor * 100 + patch. */
int dass_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DASS_H */
