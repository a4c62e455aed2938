"""torch.autograd plumbing around the C ABI: the Gaussian sample layer as a differentiable
function of (mu, sigma), so that a PyTorch training loop can use the HIP path unchanged, and the
sampled linear layer (BayesianLinear, at the end) whose weights and per-sample weight gradients
never exist in memory.

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


class _Linear(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, mu_w, sigma_w, mu_b, sigma_b, layer, step):
        rng = hot.hot_rng(seed=layer.seed, step=step, first_sample=layer.first_sample)
        xd = x.detach().contiguous()
        y = torch.empty(layer.s_local, xd.shape[-2], layer.out_features, dtype=torch.float32, device=x.device)
        det = [t.detach() if t is not None else None for t in (mu_w, sigma_w, mu_b, sigma_b)]
        hot.hot_linear_forward_rng(rng, xd, det[0], det[1], det[2], det[3], y, layer.weight_offset, layer.bias_offset)
        ctx.layer, ctx.rng, ctx.has_bias = layer, rng, mu_b is not None
        ctx.save_for_backward(xd, *[t for t in det if t is not None])
        return y

    @staticmethod
    def backward(ctx, grad_y):
        layer = ctx.layer
        xd, mu_w, sigma_w = ctx.saved_tensors[:3]
        mu_b, sigma_b = ctx.saved_tensors[3:] if ctx.has_bias else (None, None)
        gmw, gsw = torch.empty_like(mu_w), torch.empty_like(sigma_w)
        gmb = torch.empty_like(mu_b) if ctx.has_bias else None
        gsb = torch.empty_like(sigma_b) if ctx.has_bias else None
        dx = None
        if ctx.needs_input_grad[0]:
            dx = torch.empty(layer.s_local, xd.shape[-2], layer.in_features, dtype=torch.float32, device=xd.device)
        # few weights and many rows: the library spreads the rows over the chip through scratch memory of ours
        ws_bytes = hot.hot_linear_backward_workspace_bytes(xd.shape[-2], layer.in_features, layer.out_features, layer.s_local)
        ws = torch.empty(ws_bytes // 4, dtype=torch.float32, device=xd.device) if ws_bytes > 0 else None
        hot.hot_linear_backward_rng(ctx.rng, xd, grad_y.contiguous(), mu_w, sigma_w, mu_b, sigma_b, gmw, gsw, gmb, gsb, dx,
                                    layer.s_local, layer.dataset_size, hot.HOT_REDUCE_NONE, layer.weight_offset,
                                    layer.bias_offset, workspace=ws)
        if dx is not None and xd.dim() == 2:
            dx = dx.sum(0)          # a shared input collects every sample's share
        return dx, gmw, gsw, gmb, gsb, None, None


class BayesianLinear:
    """One mean-field Gaussian linear layer on the fused kernels.  `weight_offset` places the layer in
    the flat parameter vector of the network (it selects the generator's counters, so two layers must
    not overlap); `next_offset` is where the following layer may start.  forward(x, ...) takes the
    minibatch [R, K] (first layer) or one input per sample [S_loc, R, K] and returns y [S_loc, R, O];
    the gradients it hands to autograd include the KL part divided by dataset_size."""

    def __init__(self, in_features: int, out_features: int, s_local: int, dataset_size: float, bias: bool = True,
                 seed: int = 0, first_sample: int = 0, weight_offset: int = 0):
        if in_features % 4 or weight_offset % 4:
            raise ValueError("in_features and weight_offset must be multiples of 4")
        self.in_features, self.out_features, self.s_local = in_features, out_features, s_local
        self.dataset_size, self.seed, self.first_sample, self.bias = float(dataset_size), seed, first_sample, bias
        self.weight_offset = weight_offset
        self.bias_offset = weight_offset + in_features * out_features        # a multiple of 4 as well
        self.next_offset = (self.bias_offset + (out_features if bias else 0) + 3) // 4 * 4

    def kl(self, mu_w, sigma_w, mu_b=None, sigma_b=None) -> torch.Tensor:
        """The layer's KL term (one float64 on the device, detached; its gradient is added by backward)."""
        if not hasattr(self, "_kl_plans"):
            dev = mu_w.device.index or 0
            sizes = [self.in_features * self.out_features] + ([self.out_features] if self.bias else [])
            self._kl_plans = [hot.hot_create(n, n, 1, 1, self.dataset_size, dev) for n in sizes]
        out = torch.zeros(len(self._kl_plans), dtype=torch.float64, device=mu_w.device)
        hot.hot_kl(self._kl_plans[0], mu_w.detach().reshape(-1), sigma_w.detach().reshape(-1), out[0:1])
        if self.bias:
            hot.hot_kl(self._kl_plans[1], mu_b.detach(), sigma_b.detach(), out[1:2])
        return out.sum()

    def forward(self, x, mu_w, sigma_w, mu_b, sigma_b, step: int):
        if self.bias == (mu_b is None):
            raise ValueError("bias arrays do not match the layer's bias setting")
        return _Linear.apply(x, mu_w, sigma_w, mu_b, sigma_b, self, int(step))


class BayesianModule(torch.nn.Module):
    """Any torch.nn.Module with all of its parameters made mean-field Gaussian: the module's
    parameters are flattened into one vector, `mu` starts at their current values, `sigma` at
    sqrt(kappa / fan_in) per parameter tensor (a constant that shrinks with the layer width, as the
    paper's experiments initialise it), and every forward call draws S_loc weight samples with the
    library, runs the module once per sample on views of the sampled vector, and returns the stacked
    outputs [S_loc, ...] with the KL term (detached; its gradient, divided by dataset_size, reaches
    mu.grad and sigma.grad through the backward kernel)."""

    def __init__(self, module: torch.nn.Module, s_local: int, dataset_size: float, kappa: float = 0.01, seed: int = 0,
                 first_sample: int = 0):
        super().__init__()
        self.module = module
        params = list(module.named_parameters())
        if not params:
            raise ValueError("the module has no parameters")
        device = params[0][1].device
        self._slices, at = [], 0
        for name, p in params:
            self._slices.append((name, at, at + p.numel(), tuple(p.shape)))
            at += p.numel()
        flat = torch.cat([p.detach().reshape(-1).float() for _, p in params])
        spread = torch.cat([torch.full((p.numel(),), (kappa / (p[0].numel() if p.dim() > 1 else p.numel())) ** 0.5)
                            for _, p in params]).to(device)
        self.mu = torch.nn.Parameter(flat.clone())
        self.sigma = torch.nn.Parameter(spread)
        for _, p in params:
            p.requires_grad_(False)             # the module's own tensors are only shape templates from here on
        self.layer = GaussianSampleLayer(at, s_local, dataset_size, device.index or 0, seed, first_sample)

    def forward(self, *inputs, step: int):
        w, kl = self.layer.sample(self.mu, self.sigma, step)
        outs = []
        for s in range(self.layer.s_local):
            sampled = {name: w[s, a:b].view(shape) for name, a, b, shape in self._slices}
            outs.append(torch.func.functional_call(self.module, sampled, inputs))
        return torch.stack(outs), kl
