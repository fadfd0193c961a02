/*
 * Host sweep of the fp32 ExtExp arithmetic (csrc/extexp.h compiled by gcc with
 * fmaf/rintf) against libm's 80-bit expl.  Walks every `stride`-th fp32 value in
 * [lo, hi] on `threads` threads and reports, over results that are normal fp32
 * numbers:
 *   max error of m * 2^n in units in the last place of e^x,
 *   min and max of m, max |t| implied, count of non-integer n.
 * Output: one line "count max_ulp min_m max_m bad_n max_ulp_x".
 *
 * A sixth argument 1 sweeps tp_extexp_bits instead (the evaluator of the 16-bit formats): n
 * is read from the bit pattern of z, must equal z - 1.5 * 2^23 and rintf(x log2 e) (bad_n counts
 * the exceptions, exact ties aside), and the error is measured against what that evaluator
 * approximates by design, e^(x - n fl(ln 2)) * 2^n (its reduction uses one constant; the factor
 * e^(n (ln 2 - fl(ln 2))) cancels between numerator and denominator of a softmax).  A seventh
 * number is then printed: the largest deviation from e^x itself, in ULPs.
 */
#define _GNU_SOURCE
#include <float.h>
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../paper_2001_04438_amd/csrc/extexp.h"

typedef struct {
    uint32_t lo_key, hi_key, stride, offset;
    int tid, threads, mode;
    double max_ulp, min_m, max_m, max_ulp_true;
    float max_ulp_x;
    uint64_t count, bad_n;
} job_t;

/* order-preserving map between floats and unsigned keys */
static uint32_t key_of(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
static float float_of(uint32_t k)
{
    uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static void *run(void *arg)
{
    job_t *j = (job_t *)arg;
    j->max_ulp = 0;
    j->min_m = 10;
    j->max_m = 0;
    j->count = 0;
    j->bad_n = 0;
    j->max_ulp_x = 0;
    j->max_ulp_true = 0;
    uint64_t span = (uint64_t)j->hi_key - j->lo_key + 1;
    uint64_t steps = (span + j->stride - 1) / j->stride;
    for (uint64_t s = j->tid; s < steps; s += j->threads) {
        uint64_t k = (uint64_t)j->lo_key + s * j->stride + j->offset;
        if (k > j->hi_key)
            break;
        float x = float_of((uint32_t)k);
        float m, n;
        long double ref = expl((long double)x);
        long double ref_true = ref;
        if (j->mode == 1) {
            float z;
            tp_extexp_bits(x, &m, &z);
            n = z - TP_MAGIC;
            float prod = x * TP_LOG2E;
            int tie = fabsf(prod - truncf(prod)) == 0.5f;   /* the fused rounding may differ there */
            if (tp_float_bits(z) - TP_MAGIC_BITS != (int)n || (n != rintf(prod) && !tie) ||
                fabsf(n - prod) > 0.5f + 1e-6f * fabsf(prod))
                j->bad_n++;
            ref = expl((long double)x - (long double)n * (long double)TP_LN2_HI) * ldexpl(1.0L, (int)n);
        } else {
            tp_extexp(x, &m, &n);
        }
        if (n != rintf(n))
            j->bad_n++;
        if (m < j->min_m) j->min_m = m;
        if (m > j->max_m) j->max_m = m;
        if (ref_true < (long double)FLT_MIN || ref_true > (long double)FLT_MAX)
            continue;
        {
            int et;
            frexpl(ref_true, &et);
            double err_true = (double)(fabsl(ldexpl((long double)m, (int)n) - ref_true) / ldexpl(1.0L, et - 24));
            if (err_true > j->max_ulp_true) j->max_ulp_true = err_true;
        }
        int e;
        frexpl(ref, &e);                         /* ref = f * 2^e, f in [0.5, 1) */
        long double ulp = ldexpl(1.0L, e - 24);   /* spacing of fp32 at ref */
        long double got = ldexpl((long double)m, (int)n);
        double err = (double)(fabsl(got - ref) / ulp);
        if (err > j->max_ulp) {
            j->max_ulp = err;
            j->max_ulp_x = x;
        }
        j->count++;
    }
    return NULL;
}

int main(int argc, char **argv)
{
    float lo = argc > 1 ? strtof(argv[1], NULL) : -104.0f;
    float hi = argc > 2 ? strtof(argv[2], NULL) : 89.0f;
    uint32_t stride = argc > 3 ? (uint32_t)strtoul(argv[3], NULL, 10) : 1;
    int threads = argc > 4 ? atoi(argv[4]) : 8;
    uint32_t offset = argc > 5 ? (uint32_t)strtoul(argv[5], NULL, 10) : 0;
    int mode = argc > 6 ? atoi(argv[6]) : 0;
    if (threads > 64) threads = 64;
    pthread_t th[64];
    job_t jobs[64];
    for (int t = 0; t < threads; ++t) {
        jobs[t].lo_key = key_of(lo);
        jobs[t].hi_key = key_of(hi);
        jobs[t].stride = stride;
        jobs[t].offset = offset % stride;
        jobs[t].tid = t;
        jobs[t].threads = threads;
        jobs[t].mode = mode;
        pthread_create(&th[t], NULL, run, &jobs[t]);
    }
    double max_ulp = 0, min_m = 10, max_m = 0, max_true = 0;
    float max_x = 0;
    uint64_t count = 0, bad = 0;
    for (int t = 0; t < threads; ++t) {
        pthread_join(th[t], NULL);
        if (jobs[t].max_ulp > max_ulp) { max_ulp = jobs[t].max_ulp; max_x = jobs[t].max_ulp_x; }
        if (jobs[t].max_ulp_true > max_true) max_true = jobs[t].max_ulp_true;
        if (jobs[t].min_m < min_m) min_m = jobs[t].min_m;
        if (jobs[t].max_m > max_m) max_m = jobs[t].max_m;
        count += jobs[t].count;
        bad += jobs[t].bad_n;
    }
    printf("%llu %.6f %.9f %.9f %llu %.9g %.6f\n", (unsigned long long)count, max_ulp, min_m, max_m,
           (unsigned long long)bad, (double)max_x, max_true);
    return 0;
}
