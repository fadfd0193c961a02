/*
 * Softmax oracle: TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow, long-double CPU implementation of what the Two-Pass and
 * Three-Pass softmax algorithms compute.  The paper's method reaches the
 * softmax itself (it is exact up to rounding, Section 1: the model "must be
 * computed exactly according to the specification"), so the oracle is the
 * definition written out (Section 1, the formula for p_i; Section 3, the
 * shift identity with c = max_i x_i):
 *
 *     mu  = max_i x_i
 *     S   = sum_i exp(x_i - mu)
 *     p_i = exp(x_i - mu) / S
 *
 * All arithmetic is x87 80-bit long double (64-bit significand) with libm's
 * expl.  The shift by mu is used only so that expl never overflows; x_i - mu
 * is exact in long double whenever the two fp32 values are within 2^40 of each
 * other in magnitude, and rounds at 2^-64 otherwise.
 *
 * Only tests, the smoke check and the bench's cpu_baseline leg may call this
 * library.  It shares no code, constants or tables with the HIP path.
 *
 * Threading: rows are independent and are dealt out to threads whole.  When
 * there are fewer rows than threads a row is handled by all threads together:
 * mu first (a maximum has no rounding, so its order is irrelevant), then the
 * sum over i is cut into contiguous index ranges, each added up in index order
 * by one thread, and the partial sums are added in ascending range order.
 * With one thread this is exactly the sequential definition.
 */
#define _GNU_SOURCE
#include <float.h>
#include <math.h>
#include <pthread.h>
#include <sched.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

_Static_assert(LDBL_MANT_DIG >= 64, "the oracle needs a long double with a 64-bit significand");

#define ORACLE_MAX_THREADS 256

/* ------------------------------------------------------------------ */
/* element decoding                                                    */
/* ------------------------------------------------------------------ */

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2 };

/* bfloat16 is the upper half of an IEEE binary32: same sign and exponent, 7
 * explicit significand bits.  Every bf16 value is exactly a binary32 value. */
static long double decode_bf16(uint16_t h)
{
    uint32_t w = (uint32_t)h << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (long double)f;
}

/* IEEE 754 binary16: 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits;
 * exponent field 0 holds the subnormals f * 2^-24, exponent field 31 infinities and NaNs. */
static long double decode_f16(uint16_t h)
{
    const int sign = h >> 15, e = (h >> 10) & 31, f = h & 1023;
    long double v;
    if (e == 0)
        v = ldexpl((long double)f, -24);
    else if (e == 31)
        v = f ? (long double)NAN : (long double)INFINITY;
    else
        v = ldexpl((long double)(1024 + f), e - 25);
    return sign ? -v : v;
}

static long double elem_at(const void *base, int kind, int64_t idx)
{
    if (kind == ORACLE_F32)
        return (long double)((const float *)base)[idx];
    if (kind == ORACLE_F16)
        return decode_f16(((const uint16_t *)base)[idx]);
    return decode_bf16(((const uint16_t *)base)[idx]);
}

/* Smallest normal number of the output format: below it a result may be flushed to zero. */
static long double min_normal(int kind)
{
    return kind == ORACLE_F16 ? ldexpl(1.0L, -14) : (long double)FLT_MIN;
}

/* Largest finite number of the output format. */
static long double max_finite(int kind)
{
    return kind == ORACLE_F16 ? 65504.0L : (long double)FLT_MAX;
}

static long double out_at(const void *base, int kind, int64_t idx)
{
    return elem_at(base, kind, idx);
}

/* ------------------------------------------------------------------ */
/* thread plumbing                                                     */
/* ------------------------------------------------------------------ */

int oracle_threads_available(void)
{
    cpu_set_t set;
    CPU_ZERO(&set);
    if (sched_getaffinity(0, sizeof set, &set) == 0) {
        int c = CPU_COUNT(&set);
        if (c > 0)
            return c > ORACLE_MAX_THREADS ? ORACLE_MAX_THREADS : c;
    }
    return 1;
}

static int clamp_threads(int threads)
{
    if (threads <= 0)
        threads = oracle_threads_available();
    if (threads > ORACLE_MAX_THREADS)
        threads = ORACLE_MAX_THREADS;
    return threads;
}

typedef void (*range_fn)(void *ctx, int tid, int64_t lo, int64_t hi);

typedef struct {
    range_fn fn;
    void *ctx;
    int tid;
    int64_t lo, hi;
} task_t;

static void *task_main(void *arg)
{
    task_t *t = (task_t *)arg;
    t->fn(t->ctx, t->tid, t->lo, t->hi);
    return NULL;
}

/* Cut [0, count) into `threads` contiguous ranges, run fn on each. */
static void parallel_ranges(int threads, int64_t count, range_fn fn, void *ctx)
{
    if (threads > count)
        threads = count > 0 ? (int)count : 1;
    if (threads <= 1) {
        fn(ctx, 0, 0, count);
        return;
    }
    pthread_t th[ORACLE_MAX_THREADS];
    task_t tasks[ORACLE_MAX_THREADS];
    for (int t = 0; t < threads; ++t) {
        tasks[t].fn = fn;
        tasks[t].ctx = ctx;
        tasks[t].tid = t;
        tasks[t].lo = count * t / threads;
        tasks[t].hi = count * (t + 1) / threads;
    }
    for (int t = 1; t < threads; ++t)
        pthread_create(&th[t], NULL, task_main, &tasks[t]);
    task_main(&tasks[0]);
    for (int t = 1; t < threads; ++t)
        pthread_join(th[t], NULL);
}

/* ------------------------------------------------------------------ */
/* mu and S                                                            */
/* ------------------------------------------------------------------ */

/* One row, one thread: the definition, in index order. */
static void row_stats_seq(const void *x, int kind, int64_t off, int64_t n, long double *mu_out,
                          long double *S_out)
{
    long double mu = elem_at(x, kind, off);
    for (int64_t i = 1; i < n; ++i) {
        long double v = elem_at(x, kind, off + i);
        if (v > mu)
            mu = v;
    }
    long double S = 0.0L;
    for (int64_t i = 0; i < n; ++i)
        S += expl(elem_at(x, kind, off + i) - mu);
    *mu_out = mu;
    *S_out = S;
}

typedef struct {
    const void *x;
    int kind;
    int64_t off;
    long double mu;
    long double part[ORACLE_MAX_THREADS];
} rowpar_t;

static void rowpar_max(void *c, int tid, int64_t lo, int64_t hi)
{
    rowpar_t *r = (rowpar_t *)c;
    long double m = elem_at(r->x, r->kind, r->off + lo);
    for (int64_t i = lo + 1; i < hi; ++i) {
        long double v = elem_at(r->x, r->kind, r->off + i);
        if (v > m)
            m = v;
    }
    r->part[tid] = m;
}

static void rowpar_sum(void *c, int tid, int64_t lo, int64_t hi)
{
    rowpar_t *r = (rowpar_t *)c;
    long double s = 0.0L;
    for (int64_t i = lo; i < hi; ++i)
        s += expl(elem_at(r->x, r->kind, r->off + i) - r->mu);
    r->part[tid] = s;
}

/* One row, all threads: global max, then contiguous partial sums in order. */
static void row_stats_par(const void *x, int kind, int64_t off, int64_t n, int threads,
                          long double *mu_out, long double *S_out)
{
    if (threads > n)
        threads = (int)n;
    if (threads <= 1) {
        row_stats_seq(x, kind, off, n, mu_out, S_out);
        return;
    }
    rowpar_t r;
    r.x = x;
    r.kind = kind;
    r.off = off;
    parallel_ranges(threads, n, rowpar_max, &r);
    long double mu = r.part[0];
    for (int t = 1; t < threads; ++t)
        if (r.part[t] > mu)
            mu = r.part[t];
    r.mu = mu;
    parallel_ranges(threads, n, rowpar_sum, &r);
    long double S = 0.0L;
    for (int t = 0; t < threads; ++t)
        S += r.part[t];
    *mu_out = mu;
    *S_out = S;
}

typedef struct {
    const void *x;
    int kind;
    int64_t n;
    long double *mu, *S;
} stats_ctx_t;

static void stats_rows(void *c, int tid, int64_t lo, int64_t hi)
{
    (void)tid;
    stats_ctx_t *s = (stats_ctx_t *)c;
    for (int64_t r = lo; r < hi; ++r)
        row_stats_seq(s->x, s->kind, r * s->n, s->n, &s->mu[r], &s->S[r]);
}

static void stats_any(const void *x, int kind, int64_t rows, int64_t n, long double *mu,
                      long double *S, int threads)
{
    if (rows <= 0 || n <= 0)
        return;
    threads = clamp_threads(threads);
    if (rows >= threads || threads == 1) {
        stats_ctx_t c = {x, kind, n, mu, S};
        parallel_ranges(threads, rows, stats_rows, &c);
    } else {
        for (int64_t r = 0; r < rows; ++r)
            row_stats_par(x, kind, r * n, n, threads, &mu[r], &S[r]);
    }
}

/* Per-row mu = max_i x_i and S = sum_i exp(x_i - mu)  (Section 3). */
void oracle_stats_f32(const float *x, int64_t rows, int64_t n, long double *mu, long double *S,
                      int threads)
{
    stats_any(x, ORACLE_F32, rows, n, mu, S, threads);
}

void oracle_stats_bf16(const uint16_t *x, int64_t rows, int64_t n, long double *mu, long double *S,
                       int threads)
{
    stats_any(x, ORACLE_BF16, rows, n, mu, S, threads);
}

/* ------------------------------------------------------------------ */
/* full probability vectors                                            */
/* ------------------------------------------------------------------ */

typedef struct {
    const void *x;
    int kind;
    int64_t n;
    const long double *mu, *S;
    long double *p;
} prob_ctx_t;

static void prob_elems(void *c, int tid, int64_t lo, int64_t hi)
{
    (void)tid;
    prob_ctx_t *q = (prob_ctx_t *)c;
    for (int64_t k = lo; k < hi; ++k) {
        int64_t r = k / q->n;
        q->p[k] = expl(elem_at(q->x, q->kind, k) - q->mu[r]) / q->S[r];
    }
}

static void softmax_any(const void *x, int kind, int64_t rows, int64_t n, long double *p,
                        int threads)
{
    if (rows <= 0 || n <= 0)
        return;
    threads = clamp_threads(threads);
    long double *mu = (long double *)malloc(sizeof(long double) * (size_t)rows);
    long double *S = (long double *)malloc(sizeof(long double) * (size_t)rows);
    stats_any(x, kind, rows, n, mu, S, threads);
    prob_ctx_t c = {x, kind, n, mu, S, p};
    parallel_ranges(threads, rows * n, prob_elems, &c);
    free(mu);
    free(S);
}

/* p[r*n + i] = exp(x[r,i] - mu_r) / S_r as long double (Section 1). */
void oracle_softmax_f32(const float *x, int64_t rows, int64_t n, long double *p, int threads)
{
    softmax_any(x, ORACLE_F32, rows, n, p, threads);
}

void oracle_softmax_bf16(const uint16_t *x, int64_t rows, int64_t n, long double *p, int threads)
{
    softmax_any(x, ORACLE_BF16, rows, n, p, threads);
}

/* ------------------------------------------------------------------ */
/* streaming comparator                                                */
/* ------------------------------------------------------------------ */

/*
 * Compares a candidate output y against p without storing p.
 *
 *   p_i >= TINY : rel_i = |y_i - p_i| / p_i, violation if rel_i > tol + slope * |x_i - mu|
 *                 (slope is 0 unless the caller asks otherwise.  The Three-Pass algorithms
 *                  evaluate Exp on fl32(x_i - mu); that subtraction alone is off by up to half an
 *                  ulp of the difference, a relative error of 2^-24 |x_i - mu| in the result that
 *                  no evaluator, however exact, can remove (Section 6.3 bounds the error of Exp,
 *                  not of its argument).  Their fp32 outputs are therefore held to
 *                  4e-6 + 2^-24 |x_i - mu| per element: slope = 2^-24.)
 *   p_i <  TINY : abs_i = |y_i - p_i|, violation if abs_i > TINY
 *                 (the paper allows subnormal results to be flushed to
 *                  zero, Section 6.3, so either 0 or the denormal passes)
 *   TINY is the smallest normal number of the storage format of y: FLT_MIN for
 *   fp32 and bf16 (same exponent range), 2^-14 for fp16.
 *   any y_i that is NaN, infinite or negative is counted separately.
 *   row sums of y are accumulated in long double.
 */
typedef struct {
    double max_rel_err;     /* over elements with p_i >= FLT_MIN            */
    int64_t worst_index;    /* flat index where max_rel_err occurred, or -1 */
    double worst_expected;  /* p at worst_index                             */
    double worst_got;       /* y at worst_index                             */
    double max_sub_abs_err; /* over elements with p_i < FLT_MIN             */
    double max_row_sum_dev; /* max_r |sum_i y[r,i] - 1|                     */
    int64_t n_rel_viol;     /* normal-range elements beyond tol             */
    int64_t n_sub_viol;     /* subnormal-range elements beyond FLT_MIN      */
    int64_t n_nonfinite;    /* y_i NaN or Inf                               */
    int64_t n_negative;     /* y_i < 0                                      */
    int64_t n_normal;       /* elements with p_i >= FLT_MIN                 */
    int64_t n_total;
    double max_bound_ratio; /* max of rel_i / (tol + slope |x_i - mu|) over those elements */
} oracle_cmp_t;

typedef struct {
    const void *x, *y;
    int kind;
    int64_t n;
    const long double *mu, *S;
    double tol, slope;
    int64_t row; /* used in single-row mode */
    oracle_cmp_t part[ORACLE_MAX_THREADS];
    long double rowsum_part[ORACLE_MAX_THREADS];
} cmp_ctx_t;

static void cmp_init(oracle_cmp_t *c)
{
    memset(c, 0, sizeof *c);
    c->worst_index = -1;
}

/* tol is the bound for this element (the caller has added slope |x_i - mu| to it). */
static void cmp_elem(oracle_cmp_t *acc, long double p, long double y, double tol, int64_t flat,
                     int kind)
{
    const long double tiny = min_normal(kind);
    acc->n_total++;
    if (!(y == y) || y > max_finite(kind) || y < -max_finite(kind)) {
        acc->n_nonfinite++;
        return;
    }
    if (y < 0.0L)
        acc->n_negative++;
    long double d = fabsl(y - p);
    if (p >= tiny) {
        acc->n_normal++;
        double rel = (double)(d / p);
        if (rel > acc->max_rel_err) {
            acc->max_rel_err = rel;
            acc->worst_index = flat;
            acc->worst_expected = (double)p;
            acc->worst_got = (double)y;
        }
        if (rel > tol)
            acc->n_rel_viol++;
        if (rel / tol > acc->max_bound_ratio)
            acc->max_bound_ratio = rel / tol;
    } else {
        if ((double)d > acc->max_sub_abs_err)
            acc->max_sub_abs_err = (double)d;
        if (d > tiny)
            acc->n_sub_viol++;
    }
}

static void cmp_merge(oracle_cmp_t *into, const oracle_cmp_t *from)
{
    if (from->max_rel_err > into->max_rel_err) {
        into->max_rel_err = from->max_rel_err;
        into->worst_index = from->worst_index;
        into->worst_expected = from->worst_expected;
        into->worst_got = from->worst_got;
    }
    if (from->max_bound_ratio > into->max_bound_ratio)
        into->max_bound_ratio = from->max_bound_ratio;
    if (from->max_sub_abs_err > into->max_sub_abs_err)
        into->max_sub_abs_err = from->max_sub_abs_err;
    if (from->max_row_sum_dev > into->max_row_sum_dev)
        into->max_row_sum_dev = from->max_row_sum_dev;
    into->n_rel_viol += from->n_rel_viol;
    into->n_sub_viol += from->n_sub_viol;
    into->n_nonfinite += from->n_nonfinite;
    into->n_negative += from->n_negative;
    into->n_normal += from->n_normal;
    into->n_total += from->n_total;
}

static void cmp_rows(void *c, int tid, int64_t lo, int64_t hi)
{
    cmp_ctx_t *q = (cmp_ctx_t *)c;
    oracle_cmp_t *acc = &q->part[tid];
    cmp_init(acc);
    for (int64_t r = lo; r < hi; ++r) {
        long double rowsum = 0.0L;
        for (int64_t i = 0; i < q->n; ++i) {
            int64_t k = r * q->n + i;
            long double d = elem_at(q->x, q->kind, k) - q->mu[r];
            long double p = expl(d) / q->S[r];
            long double y = out_at(q->y, q->kind, k);
            cmp_elem(acc, p, y, q->tol + q->slope * (double)fabsl(d), k, q->kind);
            if (y == y)
                rowsum += y;
        }
        double dev = (double)fabsl(rowsum - 1.0L);
        if (dev > acc->max_row_sum_dev)
            acc->max_row_sum_dev = dev;
    }
}

static void cmp_one_row_range(void *c, int tid, int64_t lo, int64_t hi)
{
    cmp_ctx_t *q = (cmp_ctx_t *)c;
    oracle_cmp_t *acc = &q->part[tid];
    cmp_init(acc);
    int64_t r = q->row;
    long double rowsum = 0.0L;
    for (int64_t i = lo; i < hi; ++i) {
        int64_t k = r * q->n + i;
        long double d = elem_at(q->x, q->kind, k) - q->mu[r];
        long double p = expl(d) / q->S[r];
        long double y = out_at(q->y, q->kind, k);
        cmp_elem(acc, p, y, q->tol + q->slope * (double)fabsl(d), k, q->kind);
        if (y == y)
            rowsum += y;
    }
    q->rowsum_part[tid] = rowsum;
}

static void compare_any(const void *x, const void *y, int kind, int64_t rows, int64_t n,
                        double tol, double slope, oracle_cmp_t *out, int threads)
{
    cmp_init(out);
    if (rows <= 0 || n <= 0)
        return;
    threads = clamp_threads(threads);
    long double *mu = (long double *)malloc(sizeof(long double) * (size_t)rows);
    long double *S = (long double *)malloc(sizeof(long double) * (size_t)rows);
    stats_any(x, kind, rows, n, mu, S, threads);
    cmp_ctx_t *q = (cmp_ctx_t *)calloc(1, sizeof *q);
    q->x = x;
    q->y = y;
    q->kind = kind;
    q->n = n;
    q->mu = mu;
    q->S = S;
    q->tol = tol;
    q->slope = slope;
    if (rows >= threads || threads == 1) {
        int used = threads > rows ? (int)rows : threads;
        parallel_ranges(threads, rows, cmp_rows, q);
        for (int t = 0; t < used; ++t)
            cmp_merge(out, &q->part[t]);
    } else {
        for (int64_t r = 0; r < rows; ++r) {
            int used = threads > n ? (int)n : threads;
            q->row = r;
            parallel_ranges(threads, n, cmp_one_row_range, q);
            long double rowsum = 0.0L;
            for (int t = 0; t < used; ++t) {
                cmp_merge(out, &q->part[t]);
                rowsum += q->rowsum_part[t];
            }
            double dev = (double)fabsl(rowsum - 1.0L);
            if (dev > out->max_row_sum_dev)
                out->max_row_sum_dev = dev;
        }
    }
    free(q);
    free(mu);
    free(S);
}

void oracle_compare_f32(const float *x, const float *y, int64_t rows, int64_t n, double tol,
                        oracle_cmp_t *out, int threads)
{
    compare_any(x, y, ORACLE_F32, rows, n, tol, 0.0, out, threads);
}

/* The same with the per-element bound tol + slope |x_i - mu| (see the comparator's header). */
void oracle_compare_sloped_f32(const float *x, const float *y, int64_t rows, int64_t n, double tol,
                               double slope, oracle_cmp_t *out, int threads)
{
    compare_any(x, y, ORACLE_F32, rows, n, tol, slope, out, threads);
}

/* x and y are both bf16 bit patterns; y is compared with the unrounded p. */
void oracle_compare_bf16(const uint16_t *x, const uint16_t *y, int64_t rows, int64_t n, double tol,
                         oracle_cmp_t *out, int threads)
{
    compare_any(x, y, ORACLE_BF16, rows, n, tol, 0.0, out, threads);
}

/* x and y are both IEEE binary16 bit patterns; y is compared with the unrounded p. */
void oracle_compare_f16(const uint16_t *x, const uint16_t *y, int64_t rows, int64_t n, double tol,
                        oracle_cmp_t *out, int threads)
{
    compare_any(x, y, ORACLE_F16, rows, n, tol, 0.0, out, threads);
}

void oracle_stats_f16(const uint16_t *x, int64_t rows, int64_t n, long double *mu, long double *S,
                      int threads)
{
    stats_any(x, ORACLE_F16, rows, n, mu, S, threads);
}

void oracle_softmax_f16(const uint16_t *x, int64_t rows, int64_t n, long double *p, int threads)
{
    softmax_any(x, ORACLE_F16, rows, n, p, threads);
}

/* ------------------------------------------------------------------ */
/* scalar exponential, for checking an (m, n) pair evaluator           */
/* ------------------------------------------------------------------ */

/*
 * For each x_k and candidate pair (m_k, n_k) (Section 4: e^x = m * 2^n with
 * m = e^t in [sqrt(2)/2, sqrt(2)], n an integer), returns
 * rel_k = |m_k * 2^(n_k) / e^(x_k) - 1| computed as
 * |m_k / exp(x_k - n_k*ln2) - 1| so nothing overflows, plus the largest value.
 */
double oracle_pair_rel_err_f32(const float *x, const float *m, const float *n, int64_t count,
                               double *rel_out)
{
    const long double ln2 = 0.693147180559945309417232121458176568L;
    double worst = 0.0;
    for (int64_t k = 0; k < count; ++k) {
        long double t = (long double)x[k] - (long double)n[k] * ln2;
        long double ref = expl(t);
        double rel = (double)fabsl((long double)m[k] / ref - 1.0L);
        if (!(rel == rel))
            rel = INFINITY;
        if (rel_out)
            rel_out[k] = rel;
        if (rel > worst)
            worst = rel;
    }
    return worst;
}

/* log-sum-exp of one row: mu + ln S, as long double (for pass-1 checks). */
long double oracle_logsumexp_f32(const float *x, int64_t n, int threads)
{
    long double mu, S;
    stats_any(x, ORACLE_F32, 1, n, &mu, &S, threads);
    return mu + logl(S);
}
