/*
 * CPU oracle for the predictive statistics of sampling-based Bayesian learning
 * (arxiv 2604.04736): the S predictions of one step are aggregated into their mean (the
 * model's output) and their standard deviation (the uncertainty) -- section "Bayesian
 * Neural Networks and Variational Inference", training description, and section "Monte
 * Carlo Dropout" -- and, with the samples spread over GPUs, the exact variant the paper
 * mentions after Algorithm 2: every GPU contributes two numbers per output, from which mean
 * and standard deviation over ALL samples are recovered without approximation.
 *
 * TEST INFRASTRUCTURE, not the product; shares no code with the HIP library.
 *
 * yhat is row-major [S, ld] fp32: row s holds the M outputs (batch x output dimension,
 * flattened) predicted with weight sample s.  Everything is evaluated in fp64 with the
 * two-pass textbook definitions.
 *
 *   whole    mean_m = (1/S) sum_s y[s,m];  std_m = sqrt( sum_s (y[s,m]-mean_m)^2 / (S-ddof) )
 *   partial  what one GPU sends for its S_loc rows: mean_m and M2_m = sum_s (y[s,m]-mean_m)^2
 *   merge    from the partials (n_p, mean_p, M2_p) of P GPUs (pooled mean and pooled sum of
 *            squares, the pairwise update of Chan, Golub, LeVeque 1979 applied to P groups):
 *              n = sum_p n_p;  mean = sum_p n_p mean_p / n;
 *              M2 = sum_p [ M2_p + n_p (mean_p - mean)^2 ];  std = sqrt(M2 / (n - ddof)).
 * The paper does not say whether the standard deviation is the population (ddof = 0) or the
 * sample (ddof = 1) one, so ddof is an argument.
 *
 * Pins (tests/test_stats_oracle_pins.py): closed forms for constant and arithmetic-progression
 * columns, numpy's mean / std as the library special case, shift and scale laws, and the
 * identity merge(partials of any grouping) == whole.  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

void stats_oracle_whole(int64_t m, int64_t ld, int32_t s, const float *y, int32_t ddof,
                        double *mean, double *std)
{
    for (int64_t j = 0; j < m; ++j) {
        double sum = 0.0;
        for (int32_t r = 0; r < s; ++r) sum += (double)y[(size_t)r * (size_t)ld + (size_t)j];
        double mu = sum / (double)s;
        double ss = 0.0;
        for (int32_t r = 0; r < s; ++r) {
            double d = (double)y[(size_t)r * (size_t)ld + (size_t)j] - mu;
            ss += d * d;
        }
        mean[j] = mu;
        std[j] = sqrt(ss / (double)(s - ddof));
    }
}

void stats_oracle_partial(int64_t m, int64_t ld, int32_t s_loc, const float *y, double *mean, double *m2)
{
    for (int64_t j = 0; j < m; ++j) {
        double sum = 0.0;
        for (int32_t r = 0; r < s_loc; ++r) sum += (double)y[(size_t)r * (size_t)ld + (size_t)j];
        double mu = sum / (double)s_loc;
        double ss = 0.0;
        for (int32_t r = 0; r < s_loc; ++r) {
            double d = (double)y[(size_t)r * (size_t)ld + (size_t)j] - mu;
            ss += d * d;
        }
        mean[j] = mu;
        m2[j] = ss;
    }
}

/* means and m2s are [parts, ld] fp64; counts[p] = number of samples behind partial p. */
void stats_oracle_merge(int32_t parts, int64_t m, int64_t ld, const int32_t *counts, const double *means,
                        const double *m2s, int32_t ddof, double *mean, double *std)
{
    double n = 0.0;
    for (int32_t p = 0; p < parts; ++p) n += (double)counts[p];
    for (int64_t j = 0; j < m; ++j) {
        double wsum = 0.0;
        for (int32_t p = 0; p < parts; ++p) wsum += (double)counts[p] * means[(size_t)p * (size_t)ld + (size_t)j];
        double mu = wsum / n;
        double ss = 0.0;
        for (int32_t p = 0; p < parts; ++p) {
            double d = means[(size_t)p * (size_t)ld + (size_t)j] - mu;
            ss += m2s[(size_t)p * (size_t)ld + (size_t)j] + (double)counts[p] * d * d;
        }
        mean[j] = mu;
        std[j] = sqrt(ss / (n - (double)ddof));
    }
}
