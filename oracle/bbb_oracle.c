/*
 * CPU oracle for the mean-field Gaussian sample layer of sampling-parallel
 * Bayes-by-Backprop training (arxiv 2604.04736, Algorithm 2, per-GPU inner loop;
 * Algorithm 1 is the same with one GPU).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is the plain definition of
 * what the path computes, written out with nested loops in fp64 on the fp32
 * input values.  Nothing here is blocked, fused, vectorised or reordered, and it
 * shares no code, header, table or helper with the HIP library.  Only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Notation (the paper's): N weights, each with mean mu[i] and standard deviation
 * sigma[i]; S samples in total over all GPUs; this GPU holds S_loc of them;
 * |D| = dataset size.  2-D arrays are row-major [S_loc, ld] with pitch ld >= N;
 * columns N..ld-1 are padding and are neither read nor written.
 *
 * Every function below is pinned by tests that do not call it to produce their
 * expected values (closed forms of the Gaussian KL, quadrature of the KL
 * integral, finite differences of the scalar objective, moment checks, the
 * sharding invariant of Algorithm 2): nothing here is "parity unpinned".
 *
 * Plain C99.  The two loops whose iterations are independent carry an OpenMP
 * pragma so the benchmark can also time the oracle on several host cores; with
 * nthreads = 1 they are ordinary serial loops.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static int clamp_threads(int nthreads)
{
#ifdef _OPENMP
    if (nthreads < 1) nthreads = 1;
    return nthreads;
#else
    (void)nthreads;
    return 1;
#endif
}

/* How many threads a call with this nthreads argument really uses. */
int bbb_oracle_threads(int nthreads)
{
    return clamp_threads(nthreads);
}

/*
 * Reparameterisation, Algorithm 2 line "w_{p,s} <- mu + sigma (.) eps_s"
 * (Algorithm 1 has the same line):  w[s,i] = mu[i] + sigma[i] * eps[s,i].
 * Output is fp64, row-major [S_loc, ld_out].
 */
void bbb_oracle_reparam(int64_t n, int64_t ld, int32_t s_loc,
                        const float *mu, const float *sigma, const float *eps,
                        double *w, int64_t ld_out, int nthreads)
{
    int nt = clamp_threads(nthreads);
    (void)nt;
    for (int32_t s = 0; s < s_loc; ++s) {
#pragma omp parallel for num_threads(nt) schedule(static)
        for (int64_t i = 0; i < n; ++i) {
            double m = (double)mu[i];
            double sd = (double)sigma[i];
            double e = (double)eps[(size_t)s * (size_t)ld + (size_t)i];
            w[(size_t)s * (size_t)ld_out + (size_t)i] = m + sd * e;
        }
    }
}

/*
 * Prior-matching term, Algorithm 2 line
 *   L_KL <- 1/2 sum_i ( sigma_i^2 + mu_i^2 - 1 - log sigma_i^2 ),
 * the closed form of KL( N(mu_i, sigma_i^2) || N(0,1) ) summed over weights.
 * log is the natural logarithm; log sigma^2 is evaluated as 2 log sigma, which is
 * the same number and stays finite when sigma^2 underflows.  Summed serially in
 * index order.  sigma = 0 gives +inf, sigma < 0 gives NaN (IEEE propagation).
 */
double bbb_oracle_kl(int64_t n, const float *mu, const float *sigma)
{
    double acc = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double m = (double)mu[i];
        double sd = (double)sigma[i];
        acc += sd * sd + m * m - 1.0 - 2.0 * log(sd);
    }
    return 0.5 * acc;
}

/*
 * Gradients of the negative scaled ELBO with respect to mu and sigma, local share
 * of one GPU (Algorithm 2: per-sample loss L_{p,s} = L_data,p,s + L_KL/|D|, its
 * gradient, and the 1/S average after the all-reduce).
 *
 * G[s,i] = dL_data,s / dw[s,i] is what back-propagation through the network
 * delivers.  Chain rule through w = mu + sigma*eps: dw/dmu = 1, dw/dsigma = eps.
 * Differentiating the KL line: dKL/dmu_i = mu_i, dKL/dsigma_i = sigma_i - 1/sigma_i.
 *
 *   grad_mu[i]    = g * sum_s G[s,i]            + k * mu[i]
 *   grad_sigma[i] = g * sum_s G[s,i] * eps[s,i] + k * (sigma[i] - 1/sigma[i])
 *
 * reduce_mean == 0 (sum convention): g = 1/S, k = S_loc/(S*|D|).  Adding these
 *   outputs over all GPUs gives exactly Algorithm 2's averaged gradient, and with
 *   S_loc = S it is Algorithm 1's gradient.
 * reduce_mean != 0 (mean convention): g = 1/S_loc, k = 1/|D|.  Averaging these
 *   outputs over GPUs that hold equally many samples gives the same gradient.
 */
void bbb_oracle_grad(int64_t n, int64_t ld, int32_t s_loc, int32_t s_total,
                     double dataset_size, int reduce_mean,
                     const float *mu, const float *sigma, const float *eps,
                     const float *G, double *grad_mu, double *grad_sigma,
                     int nthreads)
{
    int nt = clamp_threads(nthreads);
    (void)nt;
    double g, k;
    if (reduce_mean) {
        g = 1.0 / (double)s_loc;
        k = 1.0 / dataset_size;
    } else {
        g = 1.0 / (double)s_total;
        k = (double)s_loc / ((double)s_total * dataset_size);
    }
#pragma omp parallel for num_threads(nt) schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double sum_g = 0.0;
        double sum_ge = 0.0;
        for (int32_t s = 0; s < s_loc; ++s) {
            size_t at = (size_t)s * (size_t)ld + (size_t)i;
            double gi = (double)G[at];
            double ei = (double)eps[at];
            sum_g += gi;
            sum_ge += gi * ei;
        }
        double m = (double)mu[i];
        double sd = (double)sigma[i];
        grad_mu[i] = g * sum_g + k * m;
        grad_sigma[i] = g * sum_ge + k * (sd - 1.0 / sd);
    }
}
