/*
 * CPU oracle for the two steps that sit next to the sample layer in the paper's algorithms
 * (arxiv 2604.04736).  TEST INFRASTRUCTURE, not the product; shares no code with the HIP library.
 *
 * 1. The optimizer-update line that closes the inner loop of Algorithm 1 and Algorithm 2 (Adam is the
 *    paper's example).  The paper gives no hyper-parameters, so they are inputs.  Adam
 *    as published (Kingma and Ba, "Adam: a method for stochastic optimization", ICLR 2015,
 *    Algorithm 1), applied to mu and to sigma with their own moment estimates, at step t >= 1:
 *        g  = grad_scale * grad
 *        m  = beta1 m + (1 - beta1) g           v = beta2 v + (1 - beta2) g^2
 *        mh = m / (1 - beta1^t)                 vh = v / (1 - beta2^t)
 *        theta = theta - lr * mh / (sqrt(vh) + eps)
 *    and afterwards sigma = max(sigma, sigma_min): the paper's q needs sigma > 0 but does not say
 *    how that is kept; sigma_min <= 0 switches the clamp off.
 *
 * 2. Monte Carlo dropout as the paper describes it in weight space (section "Monte Carlo
 *    Dropout": in the variational reading each weight carries a random 0/1 keep factor): for sample s and
 *    weight i, b[s,i] = 1 with probability keep, else 0, and
 *        w[s,i] = mu[i] * b[s,i] / keep                       (forward; 1/keep keeps E[w] = mu)
 *        grad_mu[i] = g * sum_s G[s,i] * b[s,i] / keep        (chain rule; g as in the Gaussian layer)
 *    The Bernoulli variable is a threshold on the raw 32-bit generator word of (s, i), which is an
 *    INPUT here (the integer stage is pinned in eps_oracle.c):  b = (word < threshold),
 *    threshold = floor(keep * 2^32) in [0, 2^32], compared in 64 bits, so that keep = 1 keeps every
 *    word (a Bernoulli variable with probability 1 is identically 1) and P(b = 1) = threshold / 2^32.
 *
 * Pins (tests/test_update_oracle_pins.py): closed forms of Adam's first step and of a constant
 * gradient, torch.optim.Adam as the library routine, invariances; mask frequency, unbiasedness and
 * hand-computed cases for the dropout layer.  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

typedef struct {
    double lr, beta1, beta2, eps, grad_scale, sigma_min;
    int64_t step; /* t >= 1 */
} update_oracle_adam_params;

static void adam_one(double *theta, double *m, double *v, double grad, const update_oracle_adam_params *p)
{
    double g = p->grad_scale * grad;
    *m = p->beta1 * (*m) + (1.0 - p->beta1) * g;
    *v = p->beta2 * (*v) + (1.0 - p->beta2) * g * g;
    double mh = *m / (1.0 - pow(p->beta1, (double)p->step));
    double vh = *v / (1.0 - pow(p->beta2, (double)p->step));
    *theta = *theta - p->lr * mh / (sqrt(vh) + p->eps);
}

/* All arrays fp64 [n], updated in place (the caller converts the fp32 state). */
void update_oracle_adam(int64_t n, const update_oracle_adam_params *p, double *mu, double *sigma,
                        const double *grad_mu, const double *grad_sigma, double *m_mu, double *v_mu,
                        double *m_sigma, double *v_sigma)
{
    for (int64_t i = 0; i < n; ++i) {
        adam_one(&mu[i], &m_mu[i], &v_mu[i], grad_mu[i], p);
        adam_one(&sigma[i], &m_sigma[i], &v_sigma[i], grad_sigma[i], p);
        if (p->sigma_min > 0.0 && sigma[i] < p->sigma_min) sigma[i] = p->sigma_min;
    }
}

uint64_t update_oracle_dropout_threshold(double keep)
{
    double t = floor(keep * 4294967296.0);
    if (t > 4294967296.0) t = 4294967296.0;
    if (t < 0.0) t = 0.0;
    return (uint64_t)t;
}

/* words [S_loc, ld_words] raw generator words; w out [S_loc, n] fp64. */
void update_oracle_dropout_forward(int64_t n, int64_t ld_words, int32_t s_loc, double keep, const float *mu,
                                   const uint32_t *words, double *w)
{
    uint64_t thr = update_oracle_dropout_threshold(keep);
    for (int32_t s = 0; s < s_loc; ++s)
        for (int64_t i = 0; i < n; ++i) {
            double b = (uint64_t)words[(size_t)s * (size_t)ld_words + (size_t)i] < thr ? 1.0 : 0.0;
            w[(size_t)s * (size_t)n + (size_t)i] = (double)mu[i] * b / keep;
        }
}

/* G [S_loc, ld] fp32 upstream gradients; grad_mu out [n] fp64; g = 1/S or 1/S_loc as in bbb_oracle_grad. */
void update_oracle_dropout_backward(int64_t n, int64_t ld, int64_t ld_words, int32_t s_loc, int32_t s_total,
                                    int reduce_mean, double keep, const float *G, const uint32_t *words,
                                    double *grad_mu)
{
    uint64_t thr = update_oracle_dropout_threshold(keep);
    double g = reduce_mean ? 1.0 / (double)s_loc : 1.0 / (double)s_total;
    for (int64_t i = 0; i < n; ++i) {
        double acc = 0.0;
        for (int32_t s = 0; s < s_loc; ++s) {
            double b = (uint64_t)words[(size_t)s * (size_t)ld_words + (size_t)i] < thr ? 1.0 : 0.0;
            acc += (double)G[(size_t)s * (size_t)ld + (size_t)i] * b / keep;
        }
        grad_mu[i] = g * acc;
    }
}
