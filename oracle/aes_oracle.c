/*
 * CPU oracle for the adaptive-edge-sampling SpMM (AES-SpMM).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  Nothing in the product path may call it,
 * link it or fall back to it; it shares no code, header, table or constant
 * with the HIP sources.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg load it.
 *
 * What it follows (paper sections):
 *   - CSR input format ........................ Sec. 2.2
 *   - feature quantisation / dequantisation ... Sec. 2.3, Eq. 1 and Eq. 2
 *   - the kernel's steps ...................... Sec. 3.2, Algorithm 1
 *   - combination phase (dense weights) ....... Sec. 2.1
 *   - strategy selector ....................... Sec. 3.3, Table 1
 *   - start-index hash ........................ Sec. 3.3, Eq. 3
 *
 * AES-SpMM is an approximation defined by its procedure, so the oracle takes
 * the procedure's steps in the paper's order (selector, hash, sampling into the
 * row's slots, accumulation over the slots) and the paper's names for its
 * quantities (row_nnz, N, sample_cnt), each step written from what it computes.
 * It is exact SpMM only on rows with row_nnz <= W.  Accumulation is in double,
 * in slot order.
 *
 * Readings of points the paper leaves open (each also listed in the design
 * document of this repository):
 *   - R = row_nnz / W is a real ratio; the bands of Table 1 are evaluated by
 *     integer cross-multiplication (row_nnz <= k*W), never by division.
 *   - current_ind of Eq. 3 is the sample index i that Algorithm 1 passes to
 *     hash(); so sample 0 always starts at element 0 when seed == 0.
 *   - Samples may overlap; nothing removes duplicates, each slot is added.
 *   - A row owns N*sample_cnt slots.  When W is not a multiple of the band's
 *     sample count this is fewer than W; no slot beyond N*sample_cnt exists.
 *   - The paper has no seed.  seed is an extension: a per-row offset s_r is
 *     added to current_ind; seed == 0 gives s_r == 0, i.e. exactly Eq. 3.
 *   - An empty row has no slots and a zero output row.
 *   - Two quantisation schemes: the paper's affine floor mapping to 0..255
 *     (Eq. 1/2), and a symmetric round-to-nearest mapping to -127..127 that
 *     the benchmark configurations ask for.  All quantiser arithmetic is
 *     IEEE binary32, one rounding per written operation (compile this file
 *     with -ffp-contract=off and without fast-math).
 *
 * Pins (tests/test_oracle_*.py): hand-worked start indices and slot layouts
 * from Table 1 + Eq. 3, band edges, brute-force dense products on tiny
 * graphs, equality with exact CSR SpMM whenever row_nnz <= W, slot-count and
 * range invariants, closed forms and error bounds of both quantisers.
 * Parity unpinned: the paper's only worked example (the W = 4 walk-through
 * of its overview figure) contradicts Eq. 3 and Table 1 and its row contents
 * are only in the figure, so no printed value of the paper pins the sampler.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_Q_PER_TENSOR = 0, ORC_Q_PER_COLUMN = 1, ORC_Q_PER_ROW = 2 };
enum { ORC_Q_AFFINE_FLOOR_U8 = 0, ORC_Q_SYMMETRIC_RNE_I8 = 1 };

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------------ */
/* Sec. 3.3, Table 1: (N, sample_cnt) from row_nnz and the width sh_width.   */
/* Last sentence of the paragraph before Table 1: N >= 1, sample_cnt <= W.   */
void orc_strategy(int64_t row_nnz, int64_t sh_width, int64_t *N, int64_t *sample_cnt)
{
    if (row_nnz <= sh_width) {          /* R <= 1: the whole row, one sample */
        *N = row_nnz;
        *sample_cnt = 1;
        return;
    }
    int64_t c;
    if (row_nnz <= 2 * sh_width)        /* 1 < R <= 2  */
        c = 4;
    else if (row_nnz <= 36 * sh_width)  /* 2 < R <= 36 */
        c = 8;
    else if (row_nnz <= 54 * sh_width)  /* 36 < R <= 54 */
        c = 16;
    else                                /* R > 54 */
        c = 32;
    int64_t n = sh_width / c;           /* N = W / sample_cnt (integer) */
    if (n < 1) n = 1;
    if (c > sh_width) c = sh_width;
    *N = n;
    *sample_cnt = c;
}

/*
 * Sec. 3.3, paragraph before Table 1: the two fixed granularities the paper
 * compares against.  mode 0: Table 1 (the method).  mode 1, "AFS": N = 1 and
 * sample_cnt = W.  mode 2, "SFS": N = W and one sample.  Rows that fit are
 * kept whole in every mode.  (These follow the paper's description of the
 * strategies; the other system's own code is not available.)
 */
void orc_strategy_mode(int64_t row_nnz, int64_t sh_width, int mode, int64_t *N, int64_t *sample_cnt)
{
    if (mode == 0 || row_nnz <= sh_width) {
        orc_strategy(row_nnz, sh_width, N, sample_cnt);
    } else if (mode == 1) {
        *N = 1;
        *sample_cnt = sh_width;
    } else {
        *N = sh_width;
        *sample_cnt = 1;
    }
}

/* Per-row offset added to current_ind.  Not in the paper; zero at seed 0. */
uint32_t orc_row_offset(uint64_t seed, int64_t rid)
{
    uint64_t t = seed * (2u * (uint64_t)rid + 1u) * 2654435761u;
    return (uint32_t)t;
}

/* Sec. 3.3, Eq. 3: start_ind = (current_ind * prime_num) mod (row_nnz-N+1). */
int64_t orc_hash(uint64_t current_ind, int64_t row_nnz, int64_t N)
{
    const uint64_t prime_num = 1429u;
    uint64_t m = (uint64_t)(row_nnz - N + 1);
    return (int64_t)((current_ind * prime_num) % m);
}

/* Number of slots row `rid` owns. */
int64_t orc_row_slots(int64_t row_nnz, int64_t sh_width, int mode)
{
    int64_t N, sample_cnt;
    orc_strategy_mode(row_nnz, sh_width, mode, &N, &sample_cnt);
    return N * sample_cnt;
}

/*
 * Sampling stage of Sec. 3.2 Algorithm 1 for one row, written from what it produces:
 * a sampled row is made of sample_cnt runs, run number `run` being the N consecutive
 * elements of the row that begin at element hash(run) (Eq. 3), and the runs are
 * interleaved in the row's slot array - element `pos` of run `run` sits in slot
 * pos * sample_cnt + run, so slots 0 .. sample_cnt-1 hold the first element of every
 * run, the next sample_cnt slots the second, and so on.  A row that fits
 * (row_nnz <= width) is the single run of all its elements.
 * Fills slot_col / slot_val (and slot_src, the index into col_ind / val each slot was
 * read from) and returns the number of slots.  width <= 0: no sampling.
 */
static int64_t sample_row(int64_t rid, const int64_t *row_ptr, const int32_t *col_ind,
                          const float *val, int64_t width, uint64_t seed, int mode,
                          int32_t *slot_col, float *slot_val, int64_t *slot_src)
{
    const int64_t first_of_row = row_ptr[rid];
    const int64_t row_nnz = row_ptr[rid + 1] - first_of_row;
    int64_t N, sample_cnt;
    orc_strategy_mode(row_nnz, width <= 0 ? row_nnz : width, mode, &N, &sample_cnt);
    const uint64_t shift = orc_row_offset(seed, rid);          /* 0 at seed 0 */
    for (int64_t run = 0; run < sample_cnt; ++run) {
        const int64_t first = first_of_row + orc_hash((uint64_t)run + shift, row_nnz, N);
        for (int64_t pos = 0; pos < N; ++pos) {
            const int64_t slot = pos * sample_cnt + run;
            slot_col[slot] = col_ind[first + pos];
            slot_val[slot] = val[first + pos];
            if (slot_src) slot_src[slot] = first + pos;
        }
    }
    return N * sample_cnt;
}

/* s_rowptr[r] = number of slots of all rows before r (n_rows + 1 entries). */
void orc_sample_rowptr(int64_t n_rows, const int64_t *row_ptr, int64_t sh_width, int mode,
                       int64_t *s_rowptr)
{
    int64_t acc = 0;
    for (int64_t r = 0; r < n_rows; ++r) {
        s_rowptr[r] = acc;
        int64_t row_nnz = row_ptr[r + 1] - row_ptr[r];
        acc += orc_row_slots(row_nnz, sh_width <= 0 ? row_nnz : sh_width, mode);
    }
    s_rowptr[n_rows] = acc;
}

/*
 * The materialised sampled matrix: row r's slots at s_rowptr[r] + k.
 * s_rowptr must have been filled by orc_sample_rowptr.  s_eid may be NULL.
 */
void orc_sample_build(int64_t n_rows, const int64_t *row_ptr, const int32_t *col_ind,
                      const float *val, int64_t sh_width, uint64_t seed, int mode,
                      const int64_t *s_rowptr, int32_t *s_col, float *s_val, int64_t *s_eid)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t r = 0; r < n_rows; ++r) {
        int64_t o = s_rowptr[r];
        sample_row(r, row_ptr, col_ind, val, sh_width, seed, mode, s_col + o, s_val + o,
                   s_eid ? s_eid + o : NULL);
    }
}

/*
 * Algorithm 1, multiply stage, on a materialised plan:
 *   Y[r, c] = sum_k s_val[k] * X[s_col[k], c], k in slot order, in double.
 * Yabs (may be NULL) receives sum_k |s_val[k] * X[s_col[k], c]|, the scale
 * against which a rounding error of the sum is measured.
 * rows == NULL: all n_rows rows, Y row index = r.
 * rows != NULL: only the n_rows listed rows, Y row index = position in list.
 */
void orc_spmm_plan(int64_t n_rows, const int64_t *rows, const int64_t *s_rowptr,
                   const int32_t *s_col, const float *s_val, const float *X, int64_t ldx,
                   int64_t F, double *Y, double *Yabs, int64_t ldy)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t t = 0; t < n_rows; ++t) {
        int64_t r = rows ? rows[t] : t;
        double *y = Y + t * ldy;
        double *ya = Yabs ? Yabs + t * ldy : NULL;
        for (int64_t c = 0; c < F; ++c) y[c] = 0.0;
        if (ya) for (int64_t c = 0; c < F; ++c) ya[c] = 0.0;
        for (int64_t k = s_rowptr[r]; k < s_rowptr[r + 1]; ++k) {
            double a = (double)s_val[k];
            const float *x = X + (int64_t)s_col[k] * ldx;
            for (int64_t c = 0; c < F; ++c) {
                double p = a * (double)x[c];
                y[c] += p;
                if (ya) ya[c] += fabs(p);
            }
        }
    }
}

/*
 * Algorithm 1 as one pass (sample a row into sh_col/sh_val, then multiply),
 * straight from the CSR, no materialised plan.  Same row-list convention.
 * Returns 0, or -1 if scratch memory could not be obtained.
 */
int orc_aes_spmm(int64_t n_rows, const int64_t *rows, const int64_t *row_ptr,
                 const int32_t *col_ind, const float *val, int64_t sh_width, uint64_t seed, int mode,
                 const float *X, int64_t ldx, int64_t F, double *Y, double *Yabs, int64_t ldy)
{
    int failed = 0;
#pragma omp parallel
    {
        int64_t cap = 0;
        int32_t *sh_col = NULL;
        float *sh_val = NULL;
#pragma omp for schedule(dynamic, 64)
        for (int64_t t = 0; t < n_rows; ++t) {
            int64_t r = rows ? rows[t] : t;
            int64_t row_nnz = row_ptr[r + 1] - row_ptr[r];
            int64_t need = sh_width <= 0 ? row_nnz : (row_nnz < sh_width ? row_nnz : sh_width);
            if (need > cap) {
                free(sh_col);
                free(sh_val);
                cap = need + 64;
                sh_col = (int32_t *)malloc((size_t)cap * sizeof(int32_t));
                sh_val = (float *)malloc((size_t)cap * sizeof(float));
                if (!sh_col || !sh_val) { cap = 0; failed = 1; continue; }
            }
            /* the row's slots, then one output element at a time: the sum over the slots, in slot order */
            const int64_t n_slots = sample_row(r, row_ptr, col_ind, val, sh_width, seed, mode, sh_col, sh_val, NULL);
            double *y = Y + t * ldy;
            double *ya = Yabs ? Yabs + t * ldy : NULL;
            for (int64_t c = 0; c < F; ++c) {
                double sum = 0.0, mag = 0.0;
                for (int64_t k = 0; k < n_slots; ++k) {
                    const double term = (double)sh_val[k] * (double)X[(int64_t)sh_col[k] * ldx + c];
                    sum += term;
                    mag += fabs(term);
                }
                y[c] = sum;
                if (ya) ya[c] = mag;
            }
        }
        free(sh_col);
        free(sh_val);
    }
    return failed ? -1 : 0;
}

/*
 * Sec. 2.1, combination phase of a layer: H = Y * Theta, the aggregated features
 * times the layer's dense weight matrix (F x Fo, row-major), in double.
 */
void orc_combine(int64_t n, int64_t F, int64_t Fo, const double *Y, int64_t ldy, const float *Theta,
                 int64_t ldt, double *H, int64_t ldh)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t)
        for (int64_t o = 0; o < Fo; ++o) {
            double acc = 0.0;
            for (int64_t c = 0; c < F; ++c) acc += Y[t * ldy + c] * (double)Theta[c * ldt + o];
            H[t * ldh + o] = acc;
        }
}

/* ------------------------------------------------------------------------ */
/* Quantisation (Sec. 2.3).  group index of element (i, c):                  */
/*   per tensor: 0; per column: c; per row: i.                               */
static int64_t n_groups(int64_t n, int64_t F, int granularity)
{
    return granularity == ORC_Q_PER_TENSOR ? 1 : granularity == ORC_Q_PER_COLUMN ? F : n;
}

static int64_t group_of(int64_t i, int64_t c, int granularity)
{
    return granularity == ORC_Q_PER_TENSOR ? 0 : granularity == ORC_Q_PER_COLUMN ? c : i;
}

/*
 * scheme AFFINE_FLOOR_U8 (Eq. 1, b = 8):
 *   q = floor((x - x_min) / (x_max - x_min) * 255), stored as the uint8 bit
 *   pattern in Xq; scale = (x_max - x_min) / 255, zero = x_min.
 *   x_max == x_min: q = 0 (so Eq. 2 returns x_min).
 * scheme SYMMETRIC_RNE_I8:
 *   a = max |x|; scale = a / 127 (1 if a == 0); q = rint(x / scale) clamped
 *   to [-127, 127]; zero (if not NULL) is set to 0.
 * scale / zero have one entry per group.  Returns 0, -1 on bad arguments.
 */
int orc_quantize(int64_t n, int64_t F, const float *X, int64_t ldx, int scheme, int granularity,
                 int8_t *Xq, int64_t ldq, float *scale, float *zero)
{
    if (scheme != ORC_Q_AFFINE_FLOOR_U8 && scheme != ORC_Q_SYMMETRIC_RNE_I8) return -1;
    if (granularity < 0 || granularity > 2) return -1;
    int64_t G = n_groups(n, F, granularity);
    float *lo = (float *)malloc((size_t)(G > 0 ? G : 1) * sizeof(float));
    float *hi = (float *)malloc((size_t)(G > 0 ? G : 1) * sizeof(float));
    if (!lo || !hi) { free(lo); free(hi); return -1; }
    for (int64_t g = 0; g < G; ++g) { lo[g] = INFINITY; hi[g] = -INFINITY; }
    for (int64_t i = 0; i < n; ++i)
        for (int64_t c = 0; c < F; ++c) {
            float x = X[i * ldx + c];
            int64_t g = group_of(i, c, granularity);
            if (scheme == ORC_Q_SYMMETRIC_RNE_I8) x = fabsf(x);
            if (x < lo[g]) lo[g] = x;
            if (x > hi[g]) hi[g] = x;
        }
    for (int64_t g = 0; g < G; ++g) {
        if (n * F == 0) { lo[g] = 0.0f; hi[g] = 0.0f; }
        if (scheme == ORC_Q_AFFINE_FLOOR_U8) {
            float d = hi[g] - lo[g];
            scale[g] = d / 255.0f;
            zero[g] = lo[g];
        } else {
            float a = hi[g];
            scale[g] = (a == 0.0f) ? 1.0f : a / 127.0f;
            if (zero) zero[g] = 0.0f;
        }
    }
    for (int64_t i = 0; i < n; ++i)
        for (int64_t c = 0; c < F; ++c) {
            float x = X[i * ldx + c];
            int64_t g = group_of(i, c, granularity);
            if (scheme == ORC_Q_AFFINE_FLOOR_U8) {
                float d = hi[g] - lo[g];
                int q = 0;
                if (d != 0.0f) {
                    float t = (x - lo[g]) / d;
                    t = t * 255.0f;
                    q = (int)floorf(t);
                    if (q < 0) q = 0;
                    if (q > 255) q = 255;
                }
                ((uint8_t *)Xq)[i * ldq + c] = (uint8_t)q;
            } else {
                float t = x / scale[g];
                int q = (int)rintf(t);
                if (q < -127) q = -127;
                if (q > 127) q = 127;
                Xq[i * ldq + c] = (int8_t)q;
            }
        }
    free(lo);
    free(hi);
    return 0;
}

/*
 * Eq. 2: x_hat = q * scale + zero (affine; q read as uint8), or q * scale
 * (symmetric; q read as int8), in binary32, multiply then add.
 */
int orc_dequantize(int64_t n, int64_t F, const int8_t *Xq, int64_t ldq, int scheme,
                   int granularity, const float *scale, const float *zero, float *Xhat,
                   int64_t ldx)
{
    if (scheme != ORC_Q_AFFINE_FLOOR_U8 && scheme != ORC_Q_SYMMETRIC_RNE_I8) return -1;
    if (granularity < 0 || granularity > 2) return -1;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t c = 0; c < F; ++c) {
            int64_t g = group_of(i, c, granularity);
            if (scheme == ORC_Q_AFFINE_FLOOR_U8) {
                float q = (float)((const uint8_t *)Xq)[i * ldq + c];
                float t = q * scale[g];
                Xhat[i * ldx + c] = t + zero[g];
            } else {
                float q = (float)Xq[i * ldq + c];
                Xhat[i * ldx + c] = q * scale[g];
            }
        }
    return 0;
}
