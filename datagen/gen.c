/*
 * Seeded synthetic input generators (counter-based, thread-count independent).
 *
 * This module only manufactures inputs: feature matrices, labels and the planted
 * model used to draw the labels.  It contains none of the solver's arithmetic
 * (no loss, gradient, Hessian or trust-region code) and is the one piece shared
 * by the CPU oracle's tests and the GPU path's tests/benchmarks, so that both
 * consume byte-identical inputs.
 *
 * Every random number is a pure function of (seed, stream, counter), so a chunk
 * of rows can be regenerated on its own and OpenMP scheduling cannot change a bit.
 */
#define _GNU_SOURCE
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define DG_API __attribute__((visibility("default")))

/* ------------------------------------------------------------------ */
/* counter-based generator                                             */
/* ------------------------------------------------------------------ */
static inline uint64_t dg_mix(uint64_t x)
{
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

static inline uint64_t dg_bits(uint64_t seed, uint64_t stream, uint64_t ctr)
{
    uint64_t k = dg_mix(seed ^ dg_mix(stream * 0xD1342543DE82EF95ull + 0x632BE59BD9B4E019ull));
    return dg_mix(k + ctr * 0x9E3779B97F4A7C15ull) ^ dg_mix(k ^ ctr);
}

/* uniform in the open interval (0,1) */
static inline double dg_u01(uint64_t seed, uint64_t stream, uint64_t ctr)
{
    return ((double)(dg_bits(seed, stream, ctr) >> 11) + 0.5) * (1.0 / 9007199254740992.0);
}

/* standard normal: Box-Muller, one output per counter (cosine branch) */
static inline double dg_n01(uint64_t seed, uint64_t stream, uint64_t ctr)
{
    double u1 = dg_u01(seed, stream, 2 * ctr);
    double u2 = dg_u01(seed, stream, 2 * ctr + 1);
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
}

/* pair of standard normals from one counter (both Box-Muller branches) */
static inline void dg_n01_pair(uint64_t seed, uint64_t stream, uint64_t ctr, double *a, double *b)
{
    double u1 = dg_u01(seed, stream, 2 * ctr);
    double u2 = dg_u01(seed, stream, 2 * ctr + 1);
    double r = sqrt(-2.0 * log(u1));
    double s, c;
    sincos(6.283185307179586476925 * u2, &s, &c);
    *a = r * c;
    *b = r * s;
}

DG_API void dg_fill_bits(uint64_t seed, uint64_t stream, uint64_t start, int64_t count, uint64_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) out[i] = dg_bits(seed, stream, start + (uint64_t)i);
}

DG_API void dg_fill_uniform(uint64_t seed, uint64_t stream, uint64_t start, int64_t count, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) out[i] = dg_u01(seed, stream, start + (uint64_t)i);
}

DG_API void dg_fill_normal(uint64_t seed, uint64_t stream, uint64_t start, int64_t count, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) out[i] = dg_n01(seed, stream, start + (uint64_t)i);
}

/* ------------------------------------------------------------------ */
/* dense two-Gaussian rows                                             */
/* ------------------------------------------------------------------ */
enum { DG_STREAM_DENSE_X = 101, DG_STREAM_DENSE_FLIP = 102 };

/*
 * Rows row0 .. row0+nrows-1 of the dense workload.  Row i belongs to class
 * c_i = +1 (i even) or -1 (i odd) and is drawn as  c_i*mu + N(0, I);  its label is
 * c_i, flipped with probability flip_prob.  Each column j is then mapped to
 * (x - shift[j]) * scale[j]  (pass shift = 0, scale = 1 for raw draws).
 */
DG_API void dg_dense_rows(uint64_t seed, int64_t row0, int64_t nrows, int64_t d, const double *mu,
                          double flip_prob, const double *shift, const double *scale, double *X, double *y)
{
    const int64_t pairs = (d + 1) / 2;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nrows; ++r) {
        const int64_t i = row0 + r;
        const double c = (i & 1) ? -1.0 : 1.0;
        double *xr = X + r * d;
        for (int64_t q = 0; q < pairs; ++q) {
            double a, b;
            dg_n01_pair(seed, DG_STREAM_DENSE_X, (uint64_t)i * (uint64_t)pairs + (uint64_t)q, &a, &b);
            const int64_t j = 2 * q;
            xr[j] = (c * mu[j] + a - shift[j]) * scale[j];
            if (j + 1 < d) xr[j + 1] = (c * mu[j + 1] + b - shift[j + 1]) * scale[j + 1];
        }
        if (y) {
            const double u = dg_u01(seed, DG_STREAM_DENSE_FLIP, (uint64_t)i);
            y[r] = (u < flip_prob) ? -c : c;
        }
    }
}

/* ------------------------------------------------------------------ */
/* sparse rows                                                         */
/* ------------------------------------------------------------------ */
enum {
    DG_STREAM_ROWLEN = 201,
    DG_STREAM_COL = 202,
    DG_STREAM_VAL = 203
};

enum { DG_LEN_CONST = 0, DG_LEN_POISSON = 1, DG_LEN_GEOMETRIC = 2 };
enum { DG_COL_UNIFORM_DISTINCT = 0, DG_COL_ZIPF = 1 };
enum { DG_VAL_LOGNORMAL = 0, DG_VAL_ONE = 1 };

typedef struct {
    int64_t n, d;
    int len_kind;      /* DG_LEN_* */
    double len_param;  /* const k, Poisson lambda, geometric mean */
    int64_t len_cap;   /* upper cap on the number of draws per row (0 = none) */
    int col_kind;      /* DG_COL_* */
    double zipf_s;     /* exponent for DG_COL_ZIPF */
    int val_kind;      /* DG_VAL_* */
    uint64_t seed;
} dg_sparse_spec;

/* number of column draws for row i (before de-duplication) */
static int64_t dg_row_draws(const dg_sparse_spec *sp, const double *pois_cdf, int64_t pois_len, int64_t i)
{
    int64_t m;
    if (sp->len_kind == DG_LEN_CONST) {
        m = (int64_t)sp->len_param;
    } else if (sp->len_kind == DG_LEN_POISSON) {
        const double u = dg_u01(sp->seed, DG_STREAM_ROWLEN, (uint64_t)i);
        int64_t lo = 0, hi = pois_len - 1; /* first k with cdf[k] >= u */
        while (lo < hi) {
            int64_t mid = (lo + hi) >> 1;
            if (pois_cdf[mid] >= u) hi = mid; else lo = mid + 1;
        }
        m = lo;
    } else {
        /* geometric on {1,2,...} with mean len_param: P(k) = p (1-p)^(k-1), p = 1/mean */
        const double u = dg_u01(sp->seed, DG_STREAM_ROWLEN, (uint64_t)i);
        const double p = 1.0 / sp->len_param;
        m = 1 + (int64_t)floor(log(u) / log1p(-p));
    }
    if (m < 1) m = 1;
    if (sp->len_cap > 0 && m > sp->len_cap) m = sp->len_cap;
    if (m > sp->d) m = sp->d;
    return m;
}

static int dg_cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * Draw the column set of row i into buf (capacity >= draws), sorted ascending and
 * distinct; returns the realised count.
 *  - uniform-distinct: keep drawing uniform columns, skipping repeats, until
 *    `draws` distinct ones are held;
 *  - Zipf: draw `draws` ranks from P(k) ~ k^-s by CDF inversion, map each through
 *    the feature permutation, drop repeats (no top-up).
 */
static int64_t dg_row_cols(const dg_sparse_spec *sp, const double *zipf_cdf, const int32_t *perm,
                           int64_t i, int64_t draws, int32_t *buf)
{
    int64_t cnt = 0;
    if (sp->col_kind == DG_COL_UNIFORM_DISTINCT) {
        uint64_t t = 0;
        while (cnt < draws) {
            const uint64_t ctr = (uint64_t)i * 4096ull + t++;
            int32_t c = (int32_t)(dg_u01(sp->seed, DG_STREAM_COL, ctr) * (double)sp->d);
            if (c >= sp->d) c = (int32_t)sp->d - 1;
            int dup = 0;
            for (int64_t q = 0; q < cnt; ++q)
                if (buf[q] == c) { dup = 1; break; }
            if (!dup) buf[cnt++] = c;
        }
        qsort(buf, (size_t)cnt, sizeof(int32_t), dg_cmp_i32);
        return cnt;
    }
    for (int64_t t = 0; t < draws; ++t) {
        const uint64_t ctr = (uint64_t)i * 4096ull + (uint64_t)t;
        const double u = dg_u01(sp->seed, DG_STREAM_COL, ctr);
        int64_t lo = 0, hi = sp->d - 1; /* first rank with cdf >= u */
        while (lo < hi) {
            int64_t mid = (lo + hi) >> 1;
            if (zipf_cdf[mid] >= u) hi = mid; else lo = mid + 1;
        }
        buf[t] = perm ? perm[lo] : (int32_t)lo;
    }
    qsort(buf, (size_t)draws, sizeof(int32_t), dg_cmp_i32);
    for (int64_t t = 0; t < draws; ++t)
        if (cnt == 0 || buf[cnt - 1] != buf[t]) buf[cnt++] = buf[t];
    return cnt;
}

static double *dg_poisson_cdf(double lambda, int64_t *len_out)
{
    int64_t len = (int64_t)(lambda + 20.0 * sqrt(lambda) + 40.0);
    double *cdf = (double *)malloc(sizeof(double) * (size_t)len);
    long double term = expl(-(long double)lambda), acc = 0.0L;
    for (int64_t k = 0; k < len; ++k) {
        acc += term;
        cdf[k] = (double)acc;
        term *= (long double)lambda / (long double)(k + 1);
    }
    cdf[len - 1] = 1.0;
    *len_out = len;
    return cdf;
}

static double *dg_zipf_cdf(int64_t d, double s)
{
    double *cdf = (double *)malloc(sizeof(double) * (size_t)d);
    long double tot = 0.0L;
    for (int64_t k = 0; k < d; ++k) tot += powl((long double)(k + 1), -(long double)s);
    long double acc = 0.0L;
    for (int64_t k = 0; k < d; ++k) {
        acc += powl((long double)(k + 1), -(long double)s);
        cdf[k] = (double)(acc / tot);
    }
    cdf[d - 1] = 1.0;
    return cdf;
}

/*
 * Pass 1: realised nnz of every row -> rowptr[0..n] (prefix sums). Returns total nnz.
 * perm (int32[d], may be NULL) maps Zipf rank -> feature index.
 */
DG_API int64_t dg_sparse_rowptr(const dg_sparse_spec *sp, const int32_t *perm, int64_t *rowptr)
{
    int64_t pois_len = 0;
    double *pois = (sp->len_kind == DG_LEN_POISSON) ? dg_poisson_cdf(sp->len_param, &pois_len) : NULL;
    double *zipf = (sp->col_kind == DG_COL_ZIPF) ? dg_zipf_cdf(sp->d, sp->zipf_s) : NULL;
    const int64_t cap = (sp->len_cap > 0) ? sp->len_cap : (pois ? pois_len : 4096);
#pragma omp parallel
    {
        int32_t *buf = (int32_t *)malloc(sizeof(int32_t) * (size_t)(cap + 8));
#pragma omp for schedule(dynamic, 1024)
        for (int64_t i = 0; i < sp->n; ++i) {
            int64_t m = dg_row_draws(sp, pois, pois_len, i);
            if (m > cap) m = cap;
            rowptr[i + 1] = dg_row_cols(sp, zipf, perm, i, m, buf);
        }
        free(buf);
    }
    rowptr[0] = 0;
    for (int64_t i = 0; i < sp->n; ++i) rowptr[i + 1] += rowptr[i];
    free(pois);
    free(zipf);
    return rowptr[sp->n];
}

/*
 * Pass 2: redraw every row (same counters, hence the same columns) and write the
 * column indices and values.  Values are exp(N(0,1)) keyed by (row, column), or 1.0;
 * each row is then scaled to unit Euclidean length.
 */
DG_API void dg_sparse_fill(const dg_sparse_spec *sp, const int32_t *perm, const int64_t *rowptr,
                           int32_t *col, double *val)
{
    int64_t pois_len = 0;
    double *pois = (sp->len_kind == DG_LEN_POISSON) ? dg_poisson_cdf(sp->len_param, &pois_len) : NULL;
    double *zipf = (sp->col_kind == DG_COL_ZIPF) ? dg_zipf_cdf(sp->d, sp->zipf_s) : NULL;
    const int64_t cap = (sp->len_cap > 0) ? sp->len_cap : (pois ? pois_len : 4096);
#pragma omp parallel
    {
        int32_t *buf = (int32_t *)malloc(sizeof(int32_t) * (size_t)(cap + 8));
#pragma omp for schedule(dynamic, 1024)
        for (int64_t i = 0; i < sp->n; ++i) {
            int64_t m = dg_row_draws(sp, pois, pois_len, i);
            if (m > cap) m = cap;
            const int64_t cnt = dg_row_cols(sp, zipf, perm, i, m, buf);
            const int64_t base = rowptr[i];
            double ss = 0.0;
            for (int64_t q = 0; q < cnt; ++q) {
                double v = 1.0;
                if (sp->val_kind == DG_VAL_LOGNORMAL)
                    v = exp(dg_n01(sp->seed, DG_STREAM_VAL, (uint64_t)i * (uint64_t)sp->d + (uint64_t)buf[q]));
                col[base + q] = buf[q];
                val[base + q] = v;
                ss += v * v;
            }
            const double inv = 1.0 / sqrt(ss);
            for (int64_t q = 0; q < cnt; ++q) val[base + q] *= inv;
        }
        free(buf);
    }
    free(pois);
    free(zipf);
}

/* scores[i] = sum_k val[k] * wstar[col[k]] over row i (used only to draw labels) */
DG_API void dg_csr_scores(int64_t n, const int64_t *rowptr, const int32_t *col, const double *val,
                          const double *wstar, double *scores)
{
#pragma omp parallel for schedule(dynamic, 4096)
    for (int64_t i = 0; i < n; ++i) {
        double acc = 0.0;
        for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k) acc += val[k] * wstar[col[k]];
        scores[i] = acc;
    }
}

DG_API int dg_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
