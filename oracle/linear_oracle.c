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
 * layer), linearity in x and additivity over a split of K.  Nothing here is "parity unpinned".
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
