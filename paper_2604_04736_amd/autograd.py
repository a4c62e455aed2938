"""torch.autograd plumbing around the C ABI: the Gaussian sample layer as a differentiable
function of (mu, sigma), so that a PyTorch training loop can use the HIP path unchanged.

    layer = GaussianSampleLayer(n_weights, s_local, dataset_size)
    w, kl = layer.sample(mu, sigma, step)          # w[s] = mu + sigma * eps_s,  eps drawn in the kernel
    loss = sum(net_loss(w[s]) for s in range(s_local)) / s_local
    loss.backward()                                 # mu.grad, sigma.grad = d(loss + KL/|D|)/d(mu, sigma)

The KL term of the negative scaled ELBO (Algorithm 1 / 2 of arxiv 2604.04736: L = L_data + KL/|D|)
is added to the gradients inside the backward kernel, as a fused regulariser; `kl` is returned
detached for logging.  No arithmetic of the method happens here: the forward is hot_forward_rng,
the backward hot_backward_rng with HOT_REDUCE_NONE (the incoming gradient already carries the
caller's scaling).
"""
from __future__ import annotations

import torch

from . import binding as hot


class _Sample(torch.autograd.Function):
    @staticmethod
    def forward(ctx, mu, sigma, layer, step):
        w = torch.empty(layer.s_local, layer.n_weights, dtype=torch.float32, device=mu.device)
        kl = torch.empty(1, dtype=torch.float64, device=mu.device)
        rng = hot.hot_rng(seed=layer.seed, step=step, first_sample=layer.first_sample)
        hot.hot_forward_rng(layer.plan, rng, mu.detach(), sigma.detach(), w, kl)
        ctx.layer, ctx.rng = layer, rng
        ctx.save_for_backward(mu.detach(), sigma.detach())
        ctx.mark_non_differentiable(kl)
        return w, kl

    @staticmethod
    def backward(ctx, grad_w, _grad_kl):
        mu, sigma = ctx.saved_tensors
        grad_w = grad_w.contiguous()
        gmu, gsig = torch.empty_like(mu), torch.empty_like(sigma)
        hot.hot_backward_rng(ctx.layer.plan, ctx.rng, mu, sigma, grad_w, gmu, gsig)
        return gmu, gsig, None, None


class GaussianSampleLayer:
    """Holds the plan of one flat parameter vector; `first_sample` is the global index of this GPU's
    first sample (rank * s_local under sampling parallelism), so that GPUs sharing a seed draw
    disjoint samples."""

    def __init__(self, n_weights: int, s_local: int, dataset_size: float, device: int = 0, seed: int = 0,
                 first_sample: int = 0):
        self.n_weights, self.s_local, self.seed, self.first_sample = n_weights, s_local, seed, first_sample
        self.plan = hot.hot_create(n_weights, n_weights, s_local, s_local, dataset_size, device, hot.HOT_REDUCE_NONE)

    def sample(self, mu: torch.Tensor, sigma: torch.Tensor, step: int):
        """w[S_loc, N] (differentiable with respect to mu and sigma) and the KL term (detached, fp64)."""
        return _Sample.apply(mu, sigma, self, int(step))
