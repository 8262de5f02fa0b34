/*
 * Runs every function of oracle/dass_oracle.c on small ragged inputs held in heap blocks of exactly
 * the size the function may touch.  Built with -fsanitize=address,undefined by
 * tests/test_sanitizers.py: an access outside a block, a misaligned or overflowing operation ends
 * the program with a report.  It also prints a checksum per function, which the test compares with
 * the same calls made through the ordinary build.
 */
#include <inttypes.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double oracle_act(double g, int act);
void oracle_sumsq(const float *X, int64_t T, int64_t ldx, const float *Wg, const float *Wu, int64_t ldw, int64_t d,
                  int64_t d_int, int act, const int64_t *neurons, int64_t n_sel, double *sumsq);
void oracle_input_sumsq(const float *X, int64_t T, int64_t ldx, int64_t d, double *sumsq);
void oracle_norms(const double *sumsq, int64_t n, double *norms);
void oracle_factor(const float *norms, int64_t n, double alpha, float *f);
int oracle_mask_nm(float *W, int64_t rows, int64_t cols, int64_t ld, const float *f, int norm_axis, int group_axis,
                   int n_keep, int m, uint8_t *mask);
int oracle_mask_unstructured(float *W, int64_t rows, int64_t cols, int64_t ld, const float *f, int norm_axis,
                             int group_axis, int64_t n_prune, uint8_t *mask);
void oracle_mlp_forward(const float *X, int64_t T, int64_t ldx, const float *Wg, const float *Wu, int64_t ldw,
                        const float *Wd, int64_t ldd, int64_t d, int64_t d_int, int act, const int64_t *tokens,
                        int64_t n_sel, double *out, double *absout);
int64_t oracle_compress_24(const float *W, int64_t rows, int64_t cols, int64_t ld, int group_axis, float *values,
                           int64_t ldv, uint8_t *meta, int64_t ldm);
void oracle_down_sparse24(const float *Y, int64_t T, int64_t ldy, const float *values, int64_t ldv,
                          const uint8_t *meta, int64_t ldm, int64_t d, int64_t d_int, const int64_t *tokens,
                          int64_t n_sel, double *out, double *absout);

/* the generator tests/test_sanitizers.py repeats: x <- x * 6364136223846793005 + 1442695040888963407 (mod 2^64),
 * value = ((x >> 40) - 2^23) / 2^20, an exact float in [-8, 8) */
static uint64_t lcg_state;
static float next_value(void)
{
    lcg_state = lcg_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (float)((double)((int64_t)(lcg_state >> 40) - (1 << 23)) / 1048576.0);
}

/* [rows, cols] with row stride ld in a block of exactly (rows - 1) * ld + cols floats */
static float *matrix(int64_t rows, int64_t cols, int64_t ld)
{
    const size_t n = (size_t)((rows - 1) * ld + cols);
    float *p = malloc(n * sizeof(float));
    for (size_t i = 0; i < n; ++i)
        p[i] = next_value();
    return p;
}

static void report(const char *name, const void *data, size_t bytes)
{
    uint64_t h = 1469598103934665603ULL; /* FNV-1a over the result's bytes */
    const unsigned char *b = data;
    for (size_t i = 0; i < bytes; ++i)
        h = (h ^ b[i]) * 1099511628211ULL;
    printf("%s %016" PRIx64 "\n", name, h);
}

int main(void)
{
    lcg_state = 2405;
    const int64_t T = 5, d = 12, I = 7, ldx = 13, ldw = 16, ldd = 9;
    float *X = matrix(T, d, ldx), *Wg = matrix(I, d, ldw), *Wu = matrix(I, d, ldw), *Wd = matrix(d, I, ldd);

    for (int act = 0; act < 4; ++act) {
        double *s = calloc((size_t)I, sizeof(double)), *n = malloc((size_t)I * sizeof(double));
        oracle_sumsq(X, T, ldx, Wg, Wu, ldw, d, I, act, NULL, 0, s);
        oracle_norms(s, I, n);
        report("norms", n, (size_t)I * sizeof(double));
        const int64_t sel[3] = {6, 0, 3};
        double *s3 = calloc(3, sizeof(double));
        oracle_sumsq(X, T, ldx, Wg, Wu, ldw, d, I, act, sel, 3, s3);
        report("norms_selected", s3, 3 * sizeof(double));
        double *o = malloc((size_t)(T * d) * sizeof(double)), *ab = malloc((size_t)(T * d) * sizeof(double));
        oracle_mlp_forward(X, T, ldx, Wg, Wu, ldw, Wd, ldd, d, I, act, NULL, 0, o, ab);
        report("forward", o, (size_t)(T * d) * sizeof(double));
        report("forward_abs", ab, (size_t)(T * d) * sizeof(double));
        const int64_t tok[2] = {4, 1};
        oracle_mlp_forward(X, T, ldx, Wg, Wu, ldw, Wd, ldd, d, I, act, tok, 2, o, NULL);
        report("forward_selected", o, (size_t)(2 * d) * sizeof(double));
        free(s); free(n); free(s3); free(o); free(ab);
    }
    {
        double *s = calloc((size_t)d, sizeof(double));
        oracle_input_sumsq(X, T, ldx, d, s);
        report("input_sumsq", s, (size_t)d * sizeof(double));
        free(s);
    }
    const double alphas[4] = {0.0, 0.5, 1.0, 0.3};
    for (int a = 0; a < 4; ++a) {
        /* N:M and unstructured on a [8, 16] matrix with row stride 19, every axis pair, packed mask */
        for (int na = 0; na < 2; ++na)
            for (int ga = 0; ga < 2; ++ga) {
                const int64_t rows = 8, cols = 16, ld = 19;
                float *nrm = malloc((size_t)(na == 0 ? rows : cols) * sizeof(float));
                for (int64_t i = 0; i < (na == 0 ? rows : cols); ++i)
                    nrm[i] = next_value() * next_value();
                nrm[1] = 0.0f;
                float *f = malloc((size_t)(na == 0 ? rows : cols) * sizeof(float));
                for (int64_t i = 0; i < (na == 0 ? rows : cols); ++i)
                    nrm[i] = nrm[i] < 0 ? -nrm[i] : nrm[i];
                oracle_factor(nrm, na == 0 ? rows : cols, alphas[a], f);
                const int nm[4][2] = {{2, 4}, {4, 8}, {1, 2}, {3, 4}};
                for (int k = 0; k < 4; ++k) {
                    float *W = matrix(rows, cols, ld);
                    W[3] = 0.0f; W[ld + 2] = -0.0f; W[2 * ld] = W[2 * ld + 1];   /* zeros and a tie */
                    uint8_t *mask = malloc((size_t)(rows * ((cols + 7) / 8)));
                    if (oracle_mask_nm(W, rows, cols, ld, f, na, ga, nm[k][0], nm[k][1], mask) != 0)
                        return 2;
                    report("mask_nm", W, (size_t)((rows - 1) * ld + cols) * sizeof(float));
                    report("mask_nm_bits", mask, (size_t)(rows * ((cols + 7) / 8)));
                    free(W); free(mask);
                }
                const int64_t len = ga == 0 ? rows : cols;
                const int64_t quotas[4] = {0, 1, len / 2, len};
                for (int k = 0; k < 4; ++k) {
                    float *W = matrix(rows, cols, ld);
                    W[5] = W[6];
                    uint8_t *mask = malloc((size_t)(rows * ((cols + 7) / 8)));
                    if (oracle_mask_unstructured(W, rows, cols, ld, f, na, ga, quotas[k], mask) != 0)
                        return 3;
                    report("mask_unstructured", W, (size_t)((rows - 1) * ld + cols) * sizeof(float));
                    report("mask_unstructured_bits", mask, (size_t)(rows * ((cols + 7) / 8)));
                    free(W); free(mask);
                }
                free(nrm); free(f);
            }
    }
    /* the compressed 2:4 form and Eq. 3 from it: prune Wd to 2:4 along its rows' groups first */
    {
        const int64_t dd = 12, di = 16, ldv = 10, ldm = 3, ldy = 17, Tn = 3;
        float *Wp = matrix(dd, di, di), *one = malloc((size_t)di * sizeof(float));
        for (int64_t i = 0; i < di; ++i)
            one[i] = 1.0f;
        if (oracle_mask_nm(Wp, dd, di, di, one, 1, 1, 2, 4, NULL) != 0)
            return 4;
        float *vals = malloc((size_t)((dd - 1) * ldv + di / 2) * sizeof(float));
        uint8_t *meta = malloc((size_t)((dd - 1) * ldm + di / 8));
        const int64_t surplus = oracle_compress_24(Wp, dd, di, di, 1, vals, ldv, meta, ldm);
        printf("surplus_cols %" PRId64 "\n", surplus);
        float *Y = matrix(Tn, di, ldy);
        double *o = malloc((size_t)(Tn * dd) * sizeof(double)), *ab = malloc((size_t)(Tn * dd) * sizeof(double));
        oracle_down_sparse24(Y, Tn, ldy, vals, ldv, meta, ldm, dd, di, NULL, 0, o, ab);
        report("down_sparse24", o, (size_t)(Tn * dd) * sizeof(double));
        /* groups along the rows, on a dense matrix: every group has surplus */
        float *v2 = malloc((size_t)((dd / 2 - 1) * di + di) * sizeof(float));
        uint8_t *m2 = malloc((size_t)((dd / 4 - 1) * (di / 2) + di / 2));
        float *Wdense = matrix(dd, di, di);
        printf("surplus_rows %" PRId64 "\n", oracle_compress_24(Wdense, dd, di, di, 0, v2, di, m2, di / 2));
        report("compress_rows_values", v2, (size_t)((dd / 2) * di) * sizeof(float));
        free(Wp); free(one); free(vals); free(meta); free(Y); free(o); free(ab); free(v2); free(m2); free(Wdense);
    }
    free(X); free(Wg); free(Wu); free(Wd);
    printf("all ok\n");
    return 0;
}
