/*
 * Scalar model of the Two-Pass softmax: TEST INFRASTRUCTURE, not the product.
 *
 * Follows Algorithm 3 (Section 4) step by step in double precision: ExtExp
 * gives e^x as a pair (m, n) with n = round(x * log2 e), t = x - n * ln 2,
 * m = e^t; pass 1 keeps a running pair (m_sum, n_sum) and rescales both terms
 * to the larger exponent before adding; pass 2 recomputes each pair and forms
 * Y_i = m_i * lambda * 2^(n_i - n_sum) with lambda = 1 / m_sum.
 *
 * e^t comes from libm (a library primitive as one step); there is no
 * polynomial here and no blocking or reordering.  The model exists to show
 * that the pair algebra reproduces the definition that softmax_oracle.c writes
 * out, and to give the expected (m_sum, n_sum) of pass 1.  It shares nothing
 * with the HIP path.
 */
#include <math.h>
#include <stdint.h>

/* ExtExp (Section 4; Algorithm 4 of Section 6.3 without its reconstruction). */
void model_extexp(double x, double *m, double *n)
{
    const double log2e = 1.44269504088896340736;
    const double ln2 = 0.693147180559945309417;
    double nn = nearbyint(x * log2e); /* round to nearest integer */
    double t = fma(-nn, ln2, x);
    *m = exp(t);
    *n = nn;
}

/* Addition in the (m, n) representation (Algorithm 3, loop body of pass 1). */
void model_pair_add(double ma, double na, double mb, double nb, double *m, double *n)
{
    double n_max = na > nb ? na : nb;
    /* both differences are <= 0: values are only ever scaled down */
    *m = ma * exp2(na - n_max) + mb * exp2(nb - n_max);
    *n = n_max;
}

/* Pass 1 of Algorithm 3 over one vector: returns the final (m_sum, n_sum). */
void model_twopass_pass1(const double *x, int64_t N, double *m_sum_out, double *n_sum_out)
{
    double m_sum = 0.0;
    double n_sum = -INFINITY;
    for (int64_t i = 0; i < N; ++i) {
        double m_i, n_i;
        model_extexp(x[i], &m_i, &n_i);
        double n_max = n_i > n_sum ? n_i : n_sum;
        m_sum = m_i * exp2(n_i - n_max) + m_sum * exp2(n_sum - n_max);
        n_sum = n_max;
    }
    *m_sum_out = m_sum;
    *n_sum_out = n_sum;
}

/* Algorithm 3 in full. */
void model_twopass(const double *x, double *y, int64_t N)
{
    double m_sum, n_sum;
    model_twopass_pass1(x, N, &m_sum, &n_sum);
    double lambda_sum = 1.0 / m_sum;
    for (int64_t i = 0; i < N; ++i) {
        double m_i, n_i;
        model_extexp(x[i], &m_i, &n_i);
        y[i] = m_i * lambda_sum * exp2(n_i - n_sum);
    }
}

/* Algorithm 1 (Section 3): max, sum of exp(x - mu), scaled exp(x - mu). */
void model_threepass_recompute(const double *x, double *y, int64_t N)
{
    double mu = x[0];
    for (int64_t i = 1; i < N; ++i)
        if (x[i] > mu)
            mu = x[i];
    double sigma = 0.0;
    for (int64_t i = 0; i < N; ++i)
        sigma += exp(x[i] - mu);
    double lambda = 1.0 / sigma;
    for (int64_t i = 0; i < N; ++i)
        y[i] = lambda * exp(x[i] - mu);
}

/* Algorithm 2 (Section 3): as Algorithm 1 but exp stored in Y then rescaled. */
void model_threepass_reload(const double *x, double *y, int64_t N)
{
    double mu = x[0];
    for (int64_t i = 1; i < N; ++i)
        if (x[i] > mu)
            mu = x[i];
    double sigma = 0.0;
    for (int64_t i = 0; i < N; ++i) {
        y[i] = exp(x[i] - mu);
        sigma += y[i];
    }
    double lambda = 1.0 / sigma;
    for (int64_t i = 0; i < N; ++i)
        y[i] = lambda * y[i];
}
