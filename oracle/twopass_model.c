/*
 * Scalar model of the (m, n) pair algebra behind the Two-Pass softmax: TEST
 * INFRASTRUCTURE, not the product.
 *
 * Section 4 represents e^x as a pair (m, n) with e^x = m * 2^n and defines how two
 * such pairs are added.  The model states exactly that, in double precision:
 * model_extexp makes a pair (n = round(x log2 e), m = e^(x - n ln 2) from libm),
 * model_pair_add adds two pairs, and everything else is built from those two: the
 * row's sum is a fold of model_pair_add over the pairs starting from the identity
 * (0, -inf), an output is the quotient of an element's pair by the sum's pair.  The
 * tests fold in index order and in random tree orders, and check
 * ln m_sum + n_sum ln 2 against the oracle's log-sum-exp.  There is no polynomial
 * here and nothing is shared with the HIP path.
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

/* The sum of e^(x_i) over one vector as a pair: the fold of pair addition, in index
 * order, over the elements' pairs (what pass 1 of Algorithm 3 produces). */
void model_twopass_pass1(const double *x, int64_t N, double *m_sum_out, double *n_sum_out)
{
    double m_sum = 0.0, n_sum = -INFINITY; /* the additive identity */
    for (int64_t i = 0; i < N; ++i) {
        double m_i, n_i;
        model_extexp(x[i], &m_i, &n_i);
        model_pair_add(m_sum, n_sum, m_i, n_i, &m_sum, &n_sum);
    }
    *m_sum_out = m_sum;
    *n_sum_out = n_sum;
}

/* Softmax through the pair algebra: each output is the element's pair divided by the
 * pair of the sum, (m_i / m_sum) * 2^(n_i - n_sum) (what pass 2 of Algorithm 3 writes). */
void model_twopass(const double *x, double *y, int64_t N)
{
    double m_sum, n_sum;
    model_twopass_pass1(x, N, &m_sum, &n_sum);
    for (int64_t i = 0; i < N; ++i) {
        double m_i, n_i;
        model_extexp(x[i], &m_i, &n_i);
        y[i] = (m_i / m_sum) * exp2(n_i - n_sum);
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
