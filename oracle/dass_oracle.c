/*
 * DaSS reference oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, float64 CPU statement of what the DaSS pruning hot path
 * computes (Guo et al., "Dependency-aware Semi-structured Sparsity of GLU
 * Variants in Large Language Models", arXiv 2405.01943).  It exists to check
 * the GPU library; it shares no code, header, table or helper with it, and
 * nothing in the product path may call it.  Only the tests, the smoke check
 * and the benchmark's CPU-baseline leg load this file.
 *
 * Every function is the paper's definition written out:
 *   - oracle_sumsq / oracle_norms : Sec. 2.2 Eq. 2 (GLU product) and Sec. 3
 *     "Incorporating Dependency into Weight Importance" (the L2 norm of the
 *     intermediate activation, taken over all calibration tokens as Sec. 2.1
 *     defines the norm of a feature).
 *   - oracle_factor               : the power of the norm in Sec. 3 Eq. 4
 *     (exponent alpha, 0.5 in the paper) and Eq. 5 (exponent 1).
 *   - oracle_mask_nm              : Sec. 3 "Extension to N:M Sparsity" on the
 *     scores of Eq. 4 / Eq. 5.
 *   - oracle_mask_unstructured    : Sec. 3 "Pruning Granularity".
 *   - oracle_input_sumsq          : Sec. 2.1 Eq. 1, the input-feature norms of the Wanda metric.
 *   - oracle_mlp_forward          : Sec. 2.2 Eq. 2 followed by Eq. 3, the output of the MLP
 *     block (with pruned weights: the next block's calibration input).
 *   - oracle_compress_24          : the 2:4 pattern of Sec. 2.2 "N:M sparsity" stored as kept
 *     values plus 2-bit positions (the form sparse matrix units consume).
 *   - oracle_down_sparse24        : Eq. 3 evaluated from that stored form.
 *
 * Inputs are float arrays holding exactly the values the GPU sees (a bf16
 * value widens to float without rounding); all arithmetic is double.  The
 * score |w| * f of a float weight and a float factor needs at most 48
 * significand bits, so the double product is the exact real number and every
 * comparison below is a comparison of real numbers.
 *
 * Ties (the paper gives no rule): of two equal scores the one at the lower
 * index along the group is kept.
 *
 * Pins: tests/test_oracle_*.py (brute force over all subsets, group-count
 * invariants, alpha = 0 magnitude pruning, the Wanda reduction of Eq. 5,
 * scale invariance, Gram-matrix closed forms for the norms, activation spot
 * values, chunk additivity; sums of squares of integers and a hand-worked Wanda selection for
 * the input norms; one-hot closed forms, a library matrix product and the identity with
 * oracle_sumsq for the MLP output; a hand-worked example and the round trip for the compressed
 * form; a library product with the decoded matrix and a hand-worked row for Eq. 3 from it).  No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ACT_SILU = 0, ACT_GELU_TANH = 1, ACT_GELU_ERF = 2, ACT_RELU = 3 };
enum { AXIS_ROWS = 0, AXIS_COLS = 1 };

/* sigma(.) of Eq. 2: Swish with beta = 1 (SwiGLU), GeLU in its tanh or erf
 * form (GeGLU), ReLU (ReGLU). */
double oracle_act(double g, int act)
{
    switch (act) {
    case ACT_SILU:
        return g / (1.0 + exp(-g));
    case ACT_GELU_TANH: {
        const double c = sqrt(2.0 / M_PI);
        return 0.5 * g * (1.0 + tanh(c * (g + 0.044715 * g * g * g)));
    }
    case ACT_GELU_ERF:
        return 0.5 * g * (1.0 + erf(g / sqrt(2.0)));
    case ACT_RELU:
        return g > 0.0 ? g : 0.0;
    default:
        return NAN;
    }
}

/*
 * Eq. 2 followed by the squared sum over tokens.
 *   X  : [T, d]     row-major, row stride ldx
 *   Wg : [d_int, d] row-major, row stride ldw  (Gate-Proj, transposed as in Sec. 3)
 *   Wu : [d_int, d] row-major, row stride ldw  (Up-Proj)
 *   neurons : n_sel row indices into Wg/Wu, or NULL for all d_int rows
 *   sumsq   : n_sel (or d_int) doubles, ADDED to -- so successive calls on
 *             successive token chunks accumulate the norm over all tokens.
 * For neuron i and token t:  y = sigma(x_t . Wg_i) * (x_t . Wu_i);
 *                            sumsq[i] += y^2.
 * Dot products run over j in natural order, in double.
 */
void oracle_sumsq(const float *X, int64_t T, int64_t ldx,
                  const float *Wg, const float *Wu, int64_t ldw,
                  int64_t d, int64_t d_int, int act,
                  const int64_t *neurons, int64_t n_sel, double *sumsq)
{
    const int64_t n = neurons ? n_sel : d_int;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t k = 0; k < n; ++k) {
        const int64_t i = neurons ? neurons[k] : k;
        const float *wg = Wg + i * ldw;
        const float *wu = Wu + i * ldw;
        double acc = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            const float *x = X + t * ldx;
            double g = 0.0, u = 0.0;
            for (int64_t j = 0; j < d; ++j) {
                g += (double)x[j] * (double)wg[j];
                u += (double)x[j] * (double)wu[j];
            }
            const double y = oracle_act(g, act) * u;
            acc += y * y;
        }
        sumsq[k] += acc;
    }
}

/*
 * Eq. 1 (the Wanda metric, which the Down-Proj score of Eq. 5 has the form of): the L2 norm of
 * every input feature over all tokens, ||X_j||_2.  Here its square:
 *   X : [T, d] row-major, row stride ldx;  sumsq : d doubles, ADDED to (token chunks accumulate)
 *   sumsq[j] += sum over t of X[t, j]^2, tokens in natural order, in double.
 */
void oracle_input_sumsq(const float *X, int64_t T, int64_t ldx, int64_t d, double *sumsq)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d; ++j) {
        double acc = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            const double x = (double)X[t * ldx + j];
            acc += x * x;
        }
        sumsq[j] += acc;
    }
}

/* ||y_i||_2 = sqrt(sum over all tokens of y_i^2). */
void oracle_norms(const double *sumsq, int64_t n, double *norms)
{
    for (int64_t i = 0; i < n; ++i)
        norms[i] = sqrt(sumsq[i]);
}

/*
 * The group-importance factor of Eq. 4 / Eq. 5: f = norm^alpha, computed in
 * double from the float norm both sides are handed and rounded once to float.
 * alpha = 0 gives 1 for every norm (also for a zero norm), alpha = 1 returns
 * the norm itself, alpha = 0.5 is the correctly rounded square root.
 */
void oracle_factor(const float *norms, int64_t n, double alpha, float *f)
{
    for (int64_t i = 0; i < n; ++i) {
        const double x = (double)norms[i];
        double v;
        if (alpha == 0.0)
            v = 1.0;
        else if (alpha == 1.0)
            v = x;
        else if (alpha == 0.5)
            v = sqrt(x);
        else
            v = pow(x, alpha);
        f[i] = (float)v;
    }
}

static inline double score_at(const float *W, int64_t ld, const float *f,
                              int norm_axis, int64_t r, int64_t c)
{
    const double w = fabs((double)W[r * ld + c]);
    const double g = (double)f[norm_axis == AXIS_ROWS ? r : c];
    return w * g; /* exact: at most 48 significand bits */
}

static inline void mask_set(uint8_t *mask, int64_t mask_ld, int64_t r, int64_t c, int keep)
{
    if (!mask)
        return;
    uint8_t *b = mask + r * mask_ld + (c >> 3);
    const uint8_t bit = (uint8_t)(1u << (c & 7));
    if (keep)
        *b |= bit;
    else
        *b &= (uint8_t)~bit;
}

/*
 * N:M selection.  W is [rows, cols] row-major with row stride ld and is
 * modified in place.  f holds one factor per row (norm_axis = rows) or per
 * column (norm_axis = cols).  Groups are m consecutive positions along
 * group_axis, aligned to multiples of m.  In each group the n_keep positions
 * of highest score survive; the others become +0.  A position's rank is the
 * number of group-mates that beat it, where b beats a if its score is larger,
 * or equal with b at the lower index.
 * mask (optional): packed bits, row stride ceil(cols / 8) bytes,
 * bit (c & 7) of byte c / 8 of row r is 1 iff W[r, c] was kept.
 * Returns 0, or -1 if the group axis length is not a multiple of m.
 */
int oracle_mask_nm(float *W, int64_t rows, int64_t cols, int64_t ld,
                   const float *f, int norm_axis, int group_axis,
                   int n_keep, int m, uint8_t *mask)
{
    const int64_t len = group_axis == AXIS_ROWS ? rows : cols;
    const int64_t lines = group_axis == AXIS_ROWS ? cols : rows;
    const int64_t mask_ld = (cols + 7) / 8;
    if (m <= 0 || m > 64 || len % m != 0 || n_keep < 0 || n_keep > m)
        return -1;
    /* chunks of 8 lines: when lines are columns, 8 of them share a mask byte */
#pragma omp parallel for schedule(static, 8)
    for (int64_t line = 0; line < lines; ++line) {
        double s[64];
        for (int64_t g0 = 0; g0 < len; g0 += m) {
            for (int a = 0; a < m; ++a) {
                const int64_t r = group_axis == AXIS_ROWS ? g0 + a : line;
                const int64_t c = group_axis == AXIS_ROWS ? line : g0 + a;
                s[a] = score_at(W, ld, f, norm_axis, r, c);
            }
            for (int a = 0; a < m; ++a) {
                int rank = 0;
                for (int b = 0; b < m; ++b)
                    if (s[b] > s[a] || (s[b] == s[a] && b < a))
                        ++rank;
                const int keep = rank < n_keep;
                const int64_t r = group_axis == AXIS_ROWS ? g0 + a : line;
                const int64_t c = group_axis == AXIS_ROWS ? line : g0 + a;
                if (!keep)
                    W[r * ld + c] = 0.0f;
                mask_set(mask, mask_ld, r, c, keep);
            }
        }
    }
    return 0;
}

typedef struct {
    double s;
    int64_t idx;
} scored_t;

/* Order: higher score first; equal scores, lower index first. */
static int scored_cmp(const void *pa, const void *pb)
{
    const scored_t *a = (const scored_t *)pa, *b = (const scored_t *)pb;
    if (a->s > b->s) return -1;
    if (a->s < b->s) return 1;
    if (a->idx < b->idx) return -1;
    if (a->idx > b->idx) return 1;
    return 0;
}

/*
 * Unstructured selection.  Each full line along group_axis (a column when
 * group_axis = rows, a row when group_axis = cols) is one comparison group:
 * its positions are sorted by (score descending, index ascending), the last
 * n_prune become +0 and the others are left untouched.
 * Returns 0, or -1 if n_prune is outside [0, line length].
 */
int oracle_mask_unstructured(float *W, int64_t rows, int64_t cols, int64_t ld,
                             const float *f, int norm_axis, int group_axis,
                             int64_t n_prune, uint8_t *mask)
{
    const int64_t len = group_axis == AXIS_ROWS ? rows : cols;
    const int64_t lines = group_axis == AXIS_ROWS ? cols : rows;
    const int64_t mask_ld = (cols + 7) / 8;
    if (n_prune < 0 || n_prune > len)
        return -1;
    const int64_t n_keep = len - n_prune;
#pragma omp parallel
    {
        scored_t *v = (scored_t *)malloc((size_t)(len > 0 ? len : 1) * sizeof(scored_t));
#pragma omp for schedule(dynamic, 8) /* 8 columns share a mask byte */
        for (int64_t line = 0; line < lines; ++line) {
            for (int64_t a = 0; a < len; ++a) {
                const int64_t r = group_axis == AXIS_ROWS ? a : line;
                const int64_t c = group_axis == AXIS_ROWS ? line : a;
                v[a].s = score_at(W, ld, f, norm_axis, r, c);
                v[a].idx = a;
            }
            qsort(v, (size_t)len, sizeof(scored_t), scored_cmp);
            for (int64_t k = 0; k < len; ++k) {
                const int64_t a = v[k].idx;
                const int keep = k < n_keep;
                const int64_t r = group_axis == AXIS_ROWS ? a : line;
                const int64_t c = group_axis == AXIS_ROWS ? line : a;
                if (!keep)
                    W[r * ld + c] = 0.0f;
                mask_set(mask, mask_ld, r, c, keep);
            }
        }
        free(v);
    }
    return 0;
}

/*
 * Eq. 2 then Eq. 3 for selected tokens:  y_i = sigma(x . Wg_i) * (x . Wu_i),
 * out_j = sum over i of y_i * Wd[j, i].
 *   X  : [T, d] row-major, row stride ldx;  Wg, Wu : [d_int, d], row stride ldw;
 *   Wd : [d, d_int] row-major, row stride ldd (Down-Proj, transposed as in Sec. 3)
 *   tokens : n_sel row indices into X, or NULL for all T rows
 *   out    : [n_sel, d] doubles, overwritten
 *   absout : NULL, or [n_sel, d] doubles receiving sum_i |y_i * Wd[j, i]| (the scale against
 *            which a lower-precision evaluation of the same sum is judged)
 * All sums in double, i and j in natural order.
 */
void oracle_mlp_forward(const float *X, int64_t T, int64_t ldx,
                        const float *Wg, const float *Wu, int64_t ldw,
                        const float *Wd, int64_t ldd, int64_t d, int64_t d_int, int act,
                        const int64_t *tokens, int64_t n_sel, double *out, double *absout)
{
    const int64_t n = tokens ? n_sel : T;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t k = 0; k < n; ++k) {
        const float *x = X + (tokens ? tokens[k] : k) * ldx;
        double *y = (double *)malloc((size_t)d_int * sizeof(double));
        for (int64_t i = 0; i < d_int; ++i) {
            const float *wg = Wg + i * ldw, *wu = Wu + i * ldw;
            double g = 0.0, u = 0.0;
            for (int64_t j = 0; j < d; ++j) {
                g += (double)x[j] * (double)wg[j];
                u += (double)x[j] * (double)wu[j];
            }
            y[i] = oracle_act(g, act) * u;
        }
        for (int64_t j = 0; j < d; ++j) {
            const float *wd = Wd + j * ldd;
            double acc = 0.0, aacc = 0.0;
            for (int64_t i = 0; i < d_int; ++i) {
                const double term = y[i] * (double)wd[i];
                acc += term;
                aacc += fabs(term);
            }
            out[k * d + j] = acc;
            if (absout)
                absout[k * d + j] = aacc;
        }
        free(y);
    }
}

/*
 * 2:4 compressed form.  W is [rows, cols] row-major with row stride ld; groups are 4 consecutive
 * positions along group_axis, aligned to multiples of 4.  A group's two stored positions are the
 * first two entries of the list (positions holding a nonzero, ascending) followed by (positions
 * holding a zero, ascending), put in ascending order p0 < p1; so a group with at most two
 * nonzeros is represented exactly.  Its code is the nibble p0 | p1 << 2.
 *   group_axis = cols: values [rows, cols / 2], row stride ldv: group g of row r fills
 *                      values[r, 2 g] and values[r, 2 g + 1]; meta [rows, cols / 8] bytes, row
 *                      stride ldm: the code of group g is nibble (g & 1) of byte g / 2 of row r.
 *   group_axis = rows: values [rows / 2, cols]: group g of column c fills values[2 g, c] and
 *                      values[2 g + 1, c]; meta [rows / 4, (cols + 1) / 2] bytes: the code of
 *                      group g of column c is nibble (c & 1) of byte c / 2 of row g.
 * Returns the number of groups that held more than two nonzeros (their surplus is dropped), or
 * -1 for a bad shape.
 */
int64_t oracle_compress_24(const float *W, int64_t rows, int64_t cols, int64_t ld, int group_axis,
                           float *values, int64_t ldv, uint8_t *meta, int64_t ldm)
{
    const int64_t len = group_axis == AXIS_ROWS ? rows : cols;
    const int64_t lines = group_axis == AXIS_ROWS ? cols : rows;
    if (rows <= 0 || cols <= 0 || len % 4 != 0 || (group_axis == AXIS_COLS && cols % 8 != 0))
        return -1;
    int64_t surplus = 0;
    for (int64_t line = 0; line < lines; ++line) {
        for (int64_t g = 0; g < len / 4; ++g) {
            float w[4];
            int order[4], n = 0, nz = 0;
            for (int a = 0; a < 4; ++a)
                w[a] = group_axis == AXIS_ROWS ? W[(4 * g + a) * ld + line] : W[line * ld + 4 * g + a];
            for (int a = 0; a < 4; ++a)
                if (w[a] != 0.0f)
                    order[n++] = a, ++nz;
            for (int a = 0; a < 4; ++a)
                if (w[a] == 0.0f)
                    order[n++] = a;
            if (nz > 2)
                ++surplus;
            const int p0 = order[0] < order[1] ? order[0] : order[1];
            const int p1 = order[0] < order[1] ? order[1] : order[0];
            const uint8_t code = (uint8_t)(p0 | (p1 << 2));
            if (group_axis == AXIS_ROWS) {
                values[(2 * g) * ldv + line] = w[p0];
                values[(2 * g + 1) * ldv + line] = w[p1];
                uint8_t *b = meta + g * ldm + (line >> 1);
                *b = (line & 1) ? (uint8_t)((*b & 0x0f) | (code << 4)) : (uint8_t)((*b & 0xf0) | code);
            } else {
                values[line * ldv + 2 * g] = w[p0];
                values[line * ldv + 2 * g + 1] = w[p1];
                uint8_t *b = meta + line * ldm + (g >> 1);
                *b = (g & 1) ? (uint8_t)((*b & 0x0f) | (code << 4)) : (uint8_t)((*b & 0xf0) | code);
            }
        }
    }
    return surplus;
}

/*
 * Eq. 3 with Down-Proj given in the 2:4 compressed form above (groups along the columns):
 *   out[t, j] = sum over groups g and stored values s of  values[j, 2 g + s] * Y[t, 4 g + p_s],
 * p_0 = code & 3, p_1 = code >> 2, code = nibble (g & 1) of meta[j, g / 2] -- i.e. Y times the
 * transpose of the matrix the compressed form stands for, summed in double, g ascending.
 *   Y      : [T, d_int] row-major, row stride ldy
 *   values : [d, d_int / 2], row stride ldv;  meta : [d, d_int / 8] bytes, row stride ldm
 *   tokens : n_sel row indices into Y, or NULL for all T rows
 *   out, absout : [n_sel, d] doubles (absout may be NULL): the sum and the sum of magnitudes
 */
void oracle_down_sparse24(const float *Y, int64_t T, int64_t ldy, const float *values, int64_t ldv,
                          const uint8_t *meta, int64_t ldm, int64_t d, int64_t d_int,
                          const int64_t *tokens, int64_t n_sel, double *out, double *absout)
{
    const int64_t n = tokens ? n_sel : T;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t k = 0; k < n; ++k) {
        const float *y = Y + (tokens ? tokens[k] : k) * ldy;
        for (int64_t j = 0; j < d; ++j) {
            double acc = 0.0, aacc = 0.0;
            for (int64_t g = 0; g < d_int / 4; ++g) {
                const int code = (meta[j * ldm + (g >> 1)] >> (4 * (g & 1))) & 15;
                const double t0 = (double)values[j * ldv + 2 * g] * (double)y[4 * g + (code & 3)];
                const double t1 = (double)values[j * ldv + 2 * g + 1] * (double)y[4 * g + (code >> 2)];
                acc += t0;
                acc += t1;
                aacc += fabs(t0) + fabs(t1);
            }
            out[k * d + j] = acc;
            if (absout)
                absout[k * d + j] = aacc;
        }
    }
}

/* Number of OpenMP threads the loops above will use (for the baseline report). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
