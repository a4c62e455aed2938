/*
 * CPU oracle for one sampled Bayesian linear layer, the first concrete instance of the
 * "ForwardPass(x, w_s)" line of Algorithm 1 / Algorithm 2 (arxiv 2604.04736): every weight
 * and bias of the layer has a mean and a standard deviation, sample s uses
 *   W_s = mu_W + sigma_W (.) eps_s ,  b_s = mu_b + sigma_b (.) eps_s^b      (reparameterisation line)
 *   y_s = x W_s^T + b_s
 * The input is the minibatch x, the same for every sample (Algorithm 2 loads one minibatch per
 * step), or, for a layer further inside the network, the previous layer's output under the same
 * sample: x_s.  x_sample_stride is the distance in floats from x_s to x_{s+1}; 0 means shared.
 *
 * TEST INFRASTRUCTURE, not the product; shares no code with the HIP library.  Plain triple
 * loop in fp64 on the fp32 inputs; eps is an input here (fp64), so the function is the layer's
 * definition and nothing else.
 *
 * Layouts: x [R, ldx] row-major (R rows = batch x tokens) or [S, R, ldx], mu_W / sigma_W [O, K] row-major
 * packed (the layout of a framework's Linear weight), eps_w [S, O, K], mu_b / sigma_b [O]
 * (NULL for a layer without bias), eps_b [S, O], y [S, R, O].
 *
 * Pins (tests/test_linear_oracle_pins.py): numpy's einsum as the library special case,
 * unit-vector inputs that read single sampled weights back, sigma = 0 (an ordinary linear
 * layer), linearity in x and additivity over a split of K; for the backward function central
 * finite differences through the forward function, einsum, and the flat-vector gradient oracle
 * (bbb_oracle.c) fed with the per-sample weight gradients.  Nothing here is "parity unpinned".
 */
#include <stddef.h>
#include <stdint.h>

void linear_oracle_forward(int32_t s_loc, int64_t rows, int64_t in_features, int64_t out_features, int64_t ldx,
                           int64_t x_sample_stride, const float *x, const float *mu_w, const float *sigma_w, const double *eps_w,
                           const float *mu_b, const float *sigma_b, const double *eps_b, double *y)
{
    for (int32_t s = 0; s < s_loc; ++s)
        for (int64_t r = 0; r < rows; ++r)
            for (int64_t o = 0; o < out_features; ++o) {
                double acc = 0.0;
                for (int64_t k = 0; k < in_features; ++k) {
                    size_t wk = (size_t)o * (size_t)in_features + (size_t)k;
                    double w = (double)mu_w[wk] +
                               (double)sigma_w[wk] * eps_w[(size_t)s * (size_t)out_features * (size_t)in_features + wk];
                    acc += (double)x[(size_t)s * (size_t)x_sample_stride + (size_t)r * (size_t)ldx + (size_t)k] * w;
                }
                if (mu_b)
                    acc += (double)mu_b[o] + (double)sigma_b[o] * eps_b[(size_t)s * (size_t)out_features + (size_t)o];
                y[((size_t)s * (size_t)rows + (size_t)r) * (size_t)out_features + (size_t)o] = acc;
            }
}

/*
 * Back-propagation through the same layer (the "Compute gradients" and averaging lines of
 * Algorithm 1 / 2 for a Linear layer).  dy[S, R, O] holds dL_s/dy_s.  With the per-sample weight
 * gradient G_s[o, k] = sum_r dy_s[r, o] x_s[r, k] and bias gradient Gb_s[o] = sum_r dy_s[r, o]
 * (chain rule through y_s = x_s W_s^T + b_s), the reparameterisation gives dW/dmu = 1,
 * dW/dsigma = eps, and the prior-matching term adds k mu and k (sigma - 1/sigma):
 *   grad_mu_w    = g sum_s G_s            + k mu_w
 *   grad_sigma_w = g sum_s G_s (.) eps_s  + k (sigma_w - 1/sigma_w)        (biases likewise)
 *   dx_s[r, k]   = sum_o dy_s[r, o] W_s[o, k]                              (one per sample)
 * g and k are the caller's scaling (see bbb_oracle.c).  dx may be NULL.  All outputs fp64.
 */
void linear_oracle_backward(int32_t s_loc, int64_t rows, int64_t in_features, int64_t out_features, int64_t ldx,
                            int64_t x_sample_stride, double g, double k, const float *x, const float *dy,
                            const float *mu_w, const float *sigma_w, const double *eps_w, const float *mu_b,
                            const float *sigma_b, const double *eps_b, double *grad_mu_w, double *grad_sigma_w,
                            double *grad_mu_b, double *grad_sigma_b, double *dx)
{
    const size_t K = (size_t)in_features, O = (size_t)out_features, R = (size_t)rows;
    for (size_t o = 0; o < O; ++o)
        for (size_t kk = 0; kk < K; ++kk) {
            double sum_g = 0.0, sum_ge = 0.0;
            for (int32_t s = 0; s < s_loc; ++s) {
                double G = 0.0;
                for (size_t r = 0; r < R; ++r)
                    G += (double)dy[((size_t)s * R + r) * O + o] *
                         (double)x[(size_t)s * (size_t)x_sample_stride + r * (size_t)ldx + kk];
                sum_g += G;
                sum_ge += G * eps_w[((size_t)s * O + o) * K + kk];
            }
            const double m = (double)mu_w[o * K + kk], sd = (double)sigma_w[o * K + kk];
            grad_mu_w[o * K + kk] = g * sum_g + k * m;
            grad_sigma_w[o * K + kk] = g * sum_ge + k * (sd - 1.0 / sd);
        }
    if (mu_b)
        for (size_t o = 0; o < O; ++o) {
            double sum_g = 0.0, sum_ge = 0.0;
            for (int32_t s = 0; s < s_loc; ++s) {
                double G = 0.0;
                for (size_t r = 0; r < R; ++r) G += (double)dy[((size_t)s * R + r) * O + o];
                sum_g += G;
                sum_ge += G * eps_b[(size_t)s * O + o];
            }
            const double m = (double)mu_b[o], sd = (double)sigma_b[o];
            grad_mu_b[o] = g * sum_g + k * m;
            grad_sigma_b[o] = g * sum_ge + k * (sd - 1.0 / sd);
        }
    if (dx)
        for (int32_t s = 0; s < s_loc; ++s)
            for (size_t r = 0; r < R; ++r)
                for (size_t kk = 0; kk < K; ++kk) {
                    double acc = 0.0;
                    for (size_t o = 0; o < O; ++o) {
                        const double w = (double)mu_w[o * K + kk] +
                                         (double)sigma_w[o * K + kk] * eps_w[((size_t)s * O + o) * K + kk];
                        acc += (double)dy[((size_t)s * R + r) * O + o] * w;
                    }
                    dx[((size_t)s * R + r) * K + kk] = acc;
                }
}
