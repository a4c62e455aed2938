// Adam's update of one parameter (Kingma and Ba, ICLR 2015) in fp32, and the constants it needs,
// shared by the stand-alone optimizer kernel and by the backward kernel that applies the update
// in its epilogue (arxiv 2604.04736, Algorithm 1 / 2: the optimizer-update line).
#ifndef HOT_ADAM_H
#define HOT_ADAM_H

#include <hip/hip_runtime.h>

#include <cmath>

#include "hot.h"

namespace {

struct AdamConst {
    float lr, beta1, beta2, one_minus_beta1, one_minus_beta2, eps, grad_scale, sigma_min;
    float corr1, corr2;   // 1 / (1 - beta1^t), 1 / (1 - beta2^t)
};

// Moments, bias correction, step.
__device__ __forceinline__ void adam_one(float &theta, float &m, float &v, float grad, const AdamConst &c)
{
    const float g = c.grad_scale * grad;
    m = __builtin_fmaf(c.beta1, m, c.one_minus_beta1 * g);
    v = __builtin_fmaf(c.beta2, v, c.one_minus_beta2 * (g * g));
    const float mh = m * c.corr1, vh = v * c.corr2;
    theta = theta - c.lr * mh / (sqrtf(vh) + c.eps);
}

// The same with the optional floor that keeps a standard deviation positive.
__device__ __forceinline__ void adam_one_sigma(float &sigma, float &m, float &v, float grad, const AdamConst &c)
{
    adam_one(sigma, m, v, grad, c);
    if (c.sigma_min > 0.0f && sigma < c.sigma_min) sigma = c.sigma_min;
}

// Validates the hyper-parameters and rounds them to the fp32 constants of the kernels.
inline bool make_adam_const(const hot_adam *p, AdamConst &c)
{
    if (!p) return false;
    if (!(p->lr >= 0.0) || !(p->beta1 >= 0.0 && p->beta1 < 1.0) || !(p->beta2 >= 0.0 && p->beta2 < 1.0) ||
        !(p->eps >= 0.0) || !std::isfinite(p->grad_scale) || !std::isfinite(p->lr) || p->step < 1)
        return false;
    c.lr = (float)p->lr;
    c.beta1 = (float)p->beta1;
    c.beta2 = (float)p->beta2;
    c.one_minus_beta1 = (float)(1.0 - p->beta1);
    c.one_minus_beta2 = (float)(1.0 - p->beta2);
    c.eps = (float)p->eps;
    c.grad_scale = (float)p->grad_scale;
    c.sigma_min = (float)p->sigma_min;
    c.corr1 = (float)(1.0 / (1.0 - std::pow(p->beta1, (double)p->step)));
    c.corr2 = (float)(1.0 / (1.0 - std::pow(p->beta2, (double)p->step)));
    return true;
}

}  // namespace

#endif  // HOT_ADAM_H
