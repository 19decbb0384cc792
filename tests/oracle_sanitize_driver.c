/* Host-side sanitizer run of the CPU oracle: built by tests/test_oracle_sanitizers.py with
 * -fsanitize=address,undefined and executed once; any out-of-bounds access, overflow or leak
 * in the oracle aborts it.  Random CSR rows of every Table 1 band, all widths, all modes. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void orc_sample_rowptr(int64_t, const int64_t *, int64_t, int, int64_t *);
void orc_sample_build(int64_t, const int64_t *, const int32_t *, const float *, int64_t, uint64_t, int,
                      const int64_t *, int32_t *, float *, int64_t *);
void orc_spmm_plan(int64_t, const int64_t *, const int64_t *, const int32_t *, const float *, const float *, int64_t,
                   int64_t, double *, double *, int64_t);
int orc_aes_spmm(int64_t, const int64_t *, const int64_t *, const int32_t *, const float *, int64_t, uint64_t, int,
                 const float *, int64_t, int64_t, double *, double *, int64_t);
int orc_quantize(int64_t, int64_t, const float *, int64_t, int, int, int8_t *, int64_t, float *, float *);
int orc_dequantize(int64_t, int64_t, const int8_t *, int64_t, int, int, const float *, const float *, float *, int64_t);
void orc_combine(int64_t, int64_t, int64_t, const double *, int64_t, const float *, int64_t, double *, int64_t);

static uint64_t state = 88172645463325252ull;
static uint64_t rnd(void) { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return state; }

int main(void)
{
    const int64_t n = 300, n_cols = 257, F = 19, Fo = 7;
    const int64_t widths[] = {0, 1, 3, 4, 16, 48, 64};
    int64_t *rowptr = malloc((n + 1) * sizeof *rowptr);
    rowptr[0] = 0;
    for (int64_t r = 0; r < n; ++r) {
        int64_t deg = (int64_t)(rnd() % 200);
        if (r % 37 == 0) deg = 0;
        if (r % 41 == 0) deg = 64 * 55 + 3;          /* the R > 54 band at W = 64 */
        rowptr[r + 1] = rowptr[r] + deg;
    }
    const int64_t nnz = rowptr[n];
    int32_t *col = malloc((nnz + 1) * sizeof *col);
    float *val = malloc((nnz + 1) * sizeof *val);
    for (int64_t e = 0; e < nnz; ++e) { col[e] = (int32_t)(rnd() % n_cols); val[e] = (float)(rnd() % 1000) / 500.0f - 1.0f; }
    float *X = malloc(n_cols * F * sizeof *X);
    for (int64_t i = 0; i < n_cols * F; ++i) X[i] = (float)(rnd() % 2000) / 1000.0f - 1.0f;
    float *Theta = malloc(F * Fo * sizeof *Theta);
    for (int64_t i = 0; i < F * Fo; ++i) Theta[i] = (float)(rnd() % 2000) / 1000.0f - 1.0f;
    double *Y = malloc(n * F * sizeof *Y), *Yabs = malloc(n * F * sizeof *Yabs), *H = malloc(n * Fo * sizeof *H);
    int64_t *s_rowptr = malloc((n + 1) * sizeof *s_rowptr);
    double check = 0.0;
    for (size_t wi = 0; wi < sizeof widths / sizeof widths[0]; ++wi)
        for (int mode = 0; mode < 3; ++mode)
            for (uint64_t seed = 0; seed < 2; ++seed) {
                const int64_t W = widths[wi];
                orc_sample_rowptr(n, rowptr, W, mode, s_rowptr);
                const int64_t S = s_rowptr[n];
                int32_t *s_col = malloc((S + 1) * sizeof *s_col);
                float *s_val = malloc((S + 1) * sizeof *s_val);
                int64_t *s_eid = malloc((S + 1) * sizeof *s_eid);
                orc_sample_build(n, rowptr, col, val, W, seed * 12345, mode, s_rowptr, s_col, s_val, s_eid);
                orc_spmm_plan(n, NULL, s_rowptr, s_col, s_val, X, F, F, Y, Yabs, F);
                check += Y[(rnd() % n) * F];
                if (orc_aes_spmm(n, NULL, rowptr, col, val, W, seed * 12345, mode, X, F, F, Y, NULL, F)) return 2;
                orc_combine(n, F, Fo, Y, F, Theta, Fo, H, Fo);
                check += H[(rnd() % n) * Fo];
                free(s_col); free(s_val); free(s_eid);
            }
    int8_t *Xq = malloc(n_cols * F);
    float *Xhat = malloc(n_cols * F * sizeof *Xhat);
    float *scale = malloc(n_cols * sizeof *scale), *zero = malloc(n_cols * sizeof *zero);
    for (int scheme = 0; scheme < 2; ++scheme)
        for (int gran = 0; gran < 3; ++gran) {
            if (orc_quantize(n_cols, F, X, F, scheme, gran, Xq, F, scale, zero)) return 3;
            if (orc_dequantize(n_cols, F, Xq, F, scheme, gran, scale, zero, Xhat, F)) return 4;
            check += Xhat[rnd() % (n_cols * F)];
        }
    if (orc_quantize(0, F, X, F, 1, 1, Xq, F, scale, zero)) return 5;
    printf("oracle sanitizer run ok (%g)\n", check);
    free(rowptr); free(col); free(val); free(X); free(Theta); free(Y); free(Yabs); free(H); free(s_rowptr);
    free(Xq); free(Xhat); free(scale); free(zero);
    return 0;
}
