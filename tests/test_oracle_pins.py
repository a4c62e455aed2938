"""Pins of the CPU oracle against what the paper's formulas and the mathematics fix.

None of the expected values below is produced by the oracle itself: they are closed
forms of the Gaussian KL divergence, quadrature of its defining integral, finite
differences of the scalar objective of Algorithm 2, moment checks of the Gaussian the
reparameterisation must reproduce, and the exactness of sample sharding that the paper
claims for the prior-matching part (arxiv 2604.04736, Algorithm 1, Algorithm 2 and the
paragraphs after Algorithm 2).
"""
import math
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
f32 = np.float32


def _rng(seed):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------------------- KL

def test_kl_closed_form_values(oracle):
    rows = np.loadtxt(os.path.join(GOLDEN, "kl_closed_forms.txt"))
    for mu, sigma, want in rows:
        got = oracle.kl(np.array([mu], f32), np.array([sigma], f32))
        # sigma = e is not an fp32 number: allow its representation error
        assert got == pytest.approx(want, abs=1e-6 if abs(sigma - math.e) < 1e-6 else 1e-12)


def test_kl_mean_only_is_half_sum_of_squares(oracle):
    a = np.array([0.5, -1.25, 3.0, 0.0, 1e-3], f32)
    got = oracle.kl(a, np.ones_like(a))
    assert got == pytest.approx(0.5 * float(np.sum(a.astype(np.float64) ** 2)), rel=1e-14)
    n = 1000
    got = oracle.kl(np.full(n, 0.75, f32), np.ones(n, f32))
    assert got == pytest.approx(n * 0.75 ** 2 / 2, rel=1e-13)


def test_kl_nonnegative_and_zero_only_at_prior(oracle):
    r = _rng(1)
    for _ in range(200):
        mu = r.normal(size=3).astype(f32) * 10 ** r.uniform(-3, 2)
        sigma = (10 ** r.uniform(-6, 3, size=3)).astype(f32)
        assert oracle.kl(mu, sigma) >= 0.0
    assert oracle.kl(np.zeros(7, f32), np.ones(7, f32)) == 0.0
    assert oracle.kl(np.zeros(1, f32), np.array([1.001], f32)) > 0.0
    assert oracle.kl(np.array([1e-3], f32), np.ones(1, f32)) > 0.0


def _kl_by_quadrature(mu, sigma, half_width=14.0, points=400001):
    """Trapezoid rule on the definition  integral q ln(q/p) dx  with p = N(0,1)."""
    x = np.linspace(mu - half_width * sigma, mu + half_width * sigma, points)
    log_q = -0.5 * ((x - mu) / sigma) ** 2 - math.log(sigma) - 0.5 * math.log(2 * math.pi)
    log_p = -0.5 * x ** 2 - 0.5 * math.log(2 * math.pi)
    f = np.exp(log_q) * (log_q - log_p)
    h = x[1] - x[0]
    return float(h * (f.sum() - 0.5 * (f[0] + f[-1])))


def test_kl_matches_definition_by_quadrature(oracle):
    r = _rng(2)
    for _ in range(12):
        mu = float(f32(r.normal() * 2.0))
        sigma = float(f32(10 ** r.uniform(-1.5, 0.8)))
        want = _kl_by_quadrature(mu, sigma)
        got = oracle.kl(np.array([mu], f32), np.array([sigma], f32))
        assert got == pytest.approx(want, rel=1e-9, abs=1e-10)


def test_kl_additive_over_partitions(oracle):
    r = _rng(3)
    n = 1013
    mu = r.normal(size=n).astype(f32)
    sigma = (10 ** r.uniform(-3, 1, size=n)).astype(f32)
    whole = oracle.kl(mu, sigma)
    for cut in (1, 17, 500, 1012):
        parts = oracle.kl(mu[:cut].copy(), sigma[:cut].copy()) + oracle.kl(mu[cut:].copy(), sigma[cut:].copy())
        assert parts == pytest.approx(whole, rel=1e-13)
    perm = r.permutation(n)
    assert oracle.kl(mu[perm], sigma[perm]) == pytest.approx(whole, rel=1e-13)


def test_kl_uses_log_of_sigma_not_of_underflowing_square(oracle):
    # sigma^2 underflows fp32 (and a product formed in fp32 would be 0 -> log = -inf)
    sigma = np.array([1e-20], f32)
    want = 0.5 * (float(sigma[0]) ** 2 - 1.0 - 2.0 * math.log(float(sigma[0])))
    assert oracle.kl(np.zeros(1, f32), sigma) == pytest.approx(want, rel=1e-14)
    assert want == pytest.approx(45.55, abs=0.01)      # -1/2 + 20 ln 10


def test_kl_ieee_propagation(oracle):
    assert oracle.kl(np.zeros(1, f32), np.zeros(1, f32)) == math.inf
    assert math.isnan(oracle.kl(np.zeros(1, f32), np.array([-1.0], f32)))


# ------------------------------------------------------------------------ reparam

def test_reparam_identities(oracle):
    r = _rng(4)
    n, s = 37, 5
    mu = r.normal(size=n).astype(f32)
    sigma = (10 ** r.uniform(-3, 1, size=n)).astype(f32)
    eps = r.normal(size=(s, n)).astype(f32)
    mu64, sg64, e64 = mu.astype(np.float64), sigma.astype(np.float64), eps.astype(np.float64)
    w = oracle.reparam(mu, sigma, eps)
    assert w.shape == (s, n) and w.dtype == np.float64
    # eps = 0 -> w = mu ; sigma = 0 -> w = mu
    assert np.array_equal(oracle.reparam(mu, sigma, np.zeros_like(eps)), np.broadcast_to(mu64, (s, n)))
    assert np.array_equal(oracle.reparam(mu, np.zeros_like(sigma), eps), np.broadcast_to(mu64, (s, n)))
    # antithetic pair: w(eps) - w(-eps) = 2 sigma eps ; w(eps) + w(-eps) = 2 mu
    wm = oracle.reparam(mu, sigma, -eps)
    ulp = 4 * np.finfo(np.float64).eps * (np.abs(mu64) + np.abs(sg64 * e64))
    assert np.all(np.abs((w - wm) - 2 * sg64 * e64) <= ulp)
    assert np.all(np.abs((w + wm) - 2 * mu64) <= ulp)
    # each row uses its own eps row and each column its own (mu, sigma): hand-checked entries
    for (si, i) in [(0, 0), (4, 36), (2, 17), (1, 35)]:
        assert w[si, i] == mu64[i] + sg64[i] * e64[si, i]


def test_reparam_reproduces_the_gaussian_it_samples(oracle):
    # q(w) = N(mu, sigma^2): sample mean and variance over many eps rows, 5 standard errors
    r = _rng(5)
    s, n = 200_000, 4
    mu = np.array([0.3, -2.0, 10.0, 0.0], f32)
    sigma = np.array([0.5, 2.0, 0.01, 1.0], f32)
    eps = r.normal(size=(s, n)).astype(f32)
    w = oracle.reparam(mu, sigma, eps)
    se_mean = sigma / math.sqrt(s)
    assert np.all(np.abs(w.mean(axis=0) - mu) < 5 * se_mean)
    se_var = sigma.astype(np.float64) ** 2 * math.sqrt(2.0 / (s - 1))
    assert np.all(np.abs(w.var(axis=0, ddof=1) - sigma.astype(np.float64) ** 2) < 5 * se_var)


def test_reparam_pitch_and_padding(oracle):
    r = _rng(6)
    n, ld, s = 13, 20, 3
    mu = r.normal(size=n).astype(f32)
    sigma = r.uniform(0.1, 1, size=n).astype(f32)
    eps = np.full((s, ld), np.nan, f32)
    eps[:, :n] = r.normal(size=(s, n)).astype(f32)
    w = oracle.reparam(mu, sigma, eps)
    assert np.all(np.isfinite(w))
    np.testing.assert_array_equal(w, oracle.reparam(mu, sigma, np.ascontiguousarray(eps[:, :n])))


# --------------------------------------------------------------------------- grads

def _objective(oracle, mu, sigma, eps, loss, s_total, dataset_size, reduce_mean):
    """J(mu, sigma) = g * sum_s f_s(mu + sigma*eps_s) + k * KL(mu, sigma), built from the
    oracle's reparameterisation and KL and an analytic data loss."""
    s_loc = eps.shape[0]
    g = 1.0 / s_loc if reduce_mean else 1.0 / s_total
    k = 1.0 / dataset_size if reduce_mean else s_loc / (s_total * dataset_size)
    w = oracle.reparam(mu, sigma, eps)
    return g * sum(loss(s, w[s]) for s in range(s_loc)) + k * oracle.kl(mu, sigma)


def _exact_f32_grid(r, shape, lo, hi, bits=12):
    """fp32 values on a coarse binary grid, so that +-h perturbations stay exact in fp32."""
    return (np.round(r.uniform(lo, hi, size=shape) * 2 ** bits) / 2 ** bits).astype(f32)


@pytest.mark.parametrize("reduce_mean", [False, True])
@pytest.mark.parametrize("kind", ["linear", "quadratic"])
def test_grad_matches_finite_differences_of_objective(oracle, kind, reduce_mean):
    r = _rng(7)
    n, s_loc, s_total, dsize = 9, 3, 12, 50.0
    mu = _exact_f32_grid(r, n, -1, 1)
    sigma = _exact_f32_grid(r, n, 0.25, 2.0)
    eps = r.normal(size=(s_loc, n)).astype(f32)
    c = r.normal(size=(s_loc, n))
    a = r.uniform(0.5, 2.0, size=n)
    t = r.normal(size=n)
    if kind == "linear":
        loss = lambda s, w: float(np.dot(c[s], w))
        G64 = c
    else:
        loss = lambda s, w: float(0.5 * np.sum(a * (w - t) ** 2))
        G64 = a * (oracle.reparam(mu, sigma, eps) - t)
    # the oracle takes G as fp32: round it, and use the rounded values in the linear loss
    G = G64.astype(f32)
    if kind == "linear":
        c = G.astype(np.float64)
    gmu, gsig = oracle.grad(mu, sigma, eps, G, s_total, dsize, reduce_mean)

    h = 2.0 ** -10          # exactly representable step; mu +- h and sigma +- h are exact fp32

    def J(m, sd):
        return _objective(oracle, m, sd, eps, loss, s_total, dsize, reduce_mean)

    for i in range(n):
        d = np.zeros(n, f32)
        d[i] = h
        fd_mu = (J(mu + d, sigma) - J(mu - d, sigma)) / (2 * h)
        fd_sg = (J(mu, sigma + d) - J(mu, sigma - d)) / (2 * h)
        if kind == "quadratic":
            # G was rounded to fp32; the objective's true gradient uses the unrounded one
            tol = 1e-6
        else:
            tol = 1e-6
        # central differences: O(h^2) error from the KL's log term, h^2 ~ 1e-6
        assert gmu[i] == pytest.approx(fd_mu, rel=tol, abs=tol)
        assert gsig[i] == pytest.approx(fd_sg, rel=tol, abs=tol)


def test_grad_linear_loss_exact_closed_form(oracle):
    # Linear loss: J is quadratic-free in the data part, so the gradient has a closed form
    # that can be typed from the chain rule without any limit process.
    n, s_loc, s_total, dsize = 4, 2, 8, 10.0
    mu = np.array([0.5, -1.0, 2.0, 0.0], f32)
    sigma = np.array([2.0, 0.5, 1.0, 4.0], f32)
    eps = np.array([[1.0, -1.0, 0.5, 2.0], [0.0, 3.0, -0.5, 1.0]], f32)
    G = np.array([[1.0, 2.0, -4.0, 0.5], [3.0, -2.0, 8.0, 0.25]], f32)
    gmu, gsig = oracle.grad(mu, sigma, eps, G, s_total, dsize)
    k = 2 / (8 * 10.0)
    want_mu = np.array([4.0, 0.0, 4.0, 0.75]) / 8 + k * np.array([0.5, -1.0, 2.0, 0.0])
    want_sg = np.array([1.0, -8.0, -6.0, 1.25]) / 8 + k * np.array([1.5, -1.5, 0.0, 3.75])
    np.testing.assert_allclose(gmu, want_mu, rtol=1e-15)
    np.testing.assert_allclose(gsig, want_sg, rtol=1e-15)
    # mean convention: g = 1/S_loc, k = 1/|D|
    gmu, gsig = oracle.grad(mu, sigma, eps, G, s_total, dsize, reduce_mean=True)
    np.testing.assert_allclose(gmu, np.array([4.0, 0.0, 4.0, 0.75]) / 2 + np.array([0.5, -1.0, 2.0, 0.0]) / 10, rtol=1e-15)
    np.testing.assert_allclose(gsig, np.array([1.0, -8.0, -6.0, 1.25]) / 2 + np.array([1.5, -1.5, 0.0, 3.75]) / 10, rtol=1e-15)


def test_grad_zero_upstream_leaves_kl_gradient(oracle):
    r = _rng(8)
    n, s_loc, s_total, dsize = 50, 4, 16, 45000.0
    mu = r.normal(size=n).astype(f32)
    sigma = (10 ** r.uniform(-3, 1, size=n)).astype(f32)
    eps = r.normal(size=(s_loc, n)).astype(f32)
    gmu, gsig = oracle.grad(mu, sigma, eps, np.zeros_like(eps), s_total, dsize)
    k = s_loc / (s_total * dsize)
    np.testing.assert_allclose(gmu, k * mu.astype(np.float64), rtol=1e-15)
    np.testing.assert_allclose(gsig, k * (sigma.astype(np.float64) - 1 / sigma.astype(np.float64)), rtol=1e-14)
    # dKL/dsigma: 1.5 at sigma = 2, -1.5 at 1/2, 0 at 1 ; dKL/dmu = mu   (S_loc = S, |D| = 1)
    mu3 = np.array([0.25, -2.0, 7.0], f32)
    sg3 = np.array([2.0, 0.5, 1.0], f32)
    z = np.zeros((1, 3), f32)
    gmu, gsig = oracle.grad(mu3, sg3, z, z, 1, 1.0)
    np.testing.assert_array_equal(gmu, [0.25, -2.0, 7.0])
    np.testing.assert_array_equal(gsig, [1.5, -1.5, 0.0])


def test_grad_expectation_for_quadratic_loss(oracle):
    # f(w) = 1/2 sum a (w - t)^2:  E[(1/S) sum_s G_s] = a (mu - t),  E[(1/S) sum_s G_s eps_s] = a sigma
    r = _rng(9)
    n, s = 16, 100_000
    mu = r.normal(size=n).astype(f32)
    sigma = r.uniform(0.2, 1.5, size=n).astype(f32)
    a = r.uniform(0.5, 2.0, size=n)
    t = r.normal(size=n)
    eps = r.normal(size=(s, n)).astype(f32)
    G = (a * (oracle.reparam(mu, sigma, eps) - t)).astype(f32)
    big_d = 1e30                                   # switches the KL part off
    gmu, gsig = oracle.grad(mu, sigma, eps, G, s, big_d)
    mu64, sg64 = mu.astype(np.float64), sigma.astype(np.float64)
    se_mu = a * sg64 / math.sqrt(s)
    # Var[a (mu - t + sigma e) e] = a^2 ((mu-t)^2 + 2 sigma^2)
    se_sg = a * np.sqrt((mu64 - t) ** 2 + 2 * sg64 ** 2) / math.sqrt(s)
    assert np.all(np.abs(gmu - a * (mu64 - t)) < 5 * se_mu)
    assert np.all(np.abs(gsig - a * sg64) < 5 * se_sg)


@pytest.mark.parametrize("parts", [2, 4, 8, 16])
def test_sharding_samples_over_gpus_is_exact(oracle, parts):
    # Algorithm 2 on P GPUs summed (sum convention) or averaged (mean convention) equals
    # Algorithm 1 on all S samples.
    r = _rng(10)
    n, s, dsize = 33, 16, 123.0
    mu = r.normal(size=n).astype(f32)
    sigma = (10 ** r.uniform(-2, 0.5, size=n)).astype(f32)
    eps = r.normal(size=(s, n)).astype(f32)
    G = (r.normal(size=(s, n)) * 10 ** r.uniform(-3, 3, size=(s, n))).astype(f32)
    whole_mu, whole_sg = oracle.grad(mu, sigma, eps, G, s, dsize)
    per = s // parts
    acc_mu, acc_sg = np.zeros(n), np.zeros(n)
    avg_mu, avg_sg = np.zeros(n), np.zeros(n)
    for p in range(parts):
        e = np.ascontiguousarray(eps[p * per:(p + 1) * per])
        g = np.ascontiguousarray(G[p * per:(p + 1) * per])
        a, b = oracle.grad(mu, sigma, e, g, s, dsize)
        acc_mu += a
        acc_sg += b
        a, b = oracle.grad(mu, sigma, e, g, s, dsize, reduce_mean=True)
        avg_mu += a / parts
        avg_sg += b / parts
    scale_mu = np.abs(G.astype(np.float64)).sum(0) / s + np.abs(mu) / dsize
    scale_sg = np.abs(G.astype(np.float64) * eps).sum(0) / s + (sigma + 1.0 / sigma) / dsize
    assert np.all(np.abs(acc_mu - whole_mu) <= 1e-14 * scale_mu)
    assert np.all(np.abs(acc_sg - whole_sg) <= 1e-14 * scale_sg)
    assert np.all(np.abs(avg_mu - whole_mu) <= 1e-14 * scale_mu)
    assert np.all(np.abs(avg_sg - whole_sg) <= 1e-14 * scale_sg)


def test_grad_permutation_and_padding(oracle):
    r = _rng(11)
    n, ld, s_loc, s_total, dsize = 29, 32, 5, 10, 77.0
    mu = r.normal(size=n).astype(f32)
    sigma = r.uniform(0.05, 3, size=n).astype(f32)
    eps = np.full((s_loc, ld), np.nan, f32)
    G = np.full((s_loc, ld), np.nan, f32)
    eps[:, :n] = r.normal(size=(s_loc, n))
    G[:, :n] = r.normal(size=(s_loc, n))
    gmu, gsig = oracle.grad(mu, sigma, eps, G, s_total, dsize)
    assert np.all(np.isfinite(gmu)) and np.all(np.isfinite(gsig))
    # weights permuted -> outputs permuted the same way
    perm = r.permutation(n)
    e2 = np.ascontiguousarray(eps[:, :n][:, perm])
    g2 = np.ascontiguousarray(G[:, :n][:, perm])
    pmu, psig = oracle.grad(mu[perm], sigma[perm], e2, g2, s_total, dsize)
    np.testing.assert_array_equal(pmu, gmu[perm])
    np.testing.assert_array_equal(psig, gsig[perm])
    # samples permuted -> same up to reassociation
    sp = r.permutation(s_loc)
    qmu, qsig = oracle.grad(mu, sigma, np.ascontiguousarray(eps[sp]), np.ascontiguousarray(G[sp]), s_total, dsize)
    np.testing.assert_allclose(qmu, gmu, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(qsig, gsig, rtol=1e-13, atol=1e-15)


def test_oracle_threads_give_identical_results(oracle):
    r = _rng(12)
    n, s = 10007, 3
    mu = r.normal(size=n).astype(f32)
    sigma = r.uniform(0.05, 3, size=n).astype(f32)
    eps = r.normal(size=(s, n)).astype(f32)
    G = r.normal(size=(s, n)).astype(f32)
    np.testing.assert_array_equal(oracle.reparam(mu, sigma, eps, 1), oracle.reparam(mu, sigma, eps, 4))
    a1, b1 = oracle.grad(mu, sigma, eps, G, 6, 10.0, False, 1)
    a4, b4 = oracle.grad(mu, sigma, eps, G, 6, 10.0, False, 4)
    np.testing.assert_array_equal(a1, a4)
    np.testing.assert_array_equal(b1, b4)


def test_grad_equals_autograd_of_the_bayes_by_backprop_objective(oracle):
    """Algorithm 1 end to end on a tiny Bayesian MLP: automatic differentiation (fp64) of
    J = (1/S) sum_s Loss(Net(x; mu + sigma*eps_s), y) + KL(mu, sigma)/|D| with respect to mu and sigma
    must equal the oracle's gradients fed with the per-sample weight gradients G_s = dLoss_s/dw_s."""
    import torch
    torch.manual_seed(0)
    d_in, d_h, d_out, batch, s, dsize = 5, 7, 3, 11, 6, 50.0
    n = d_in * d_h + d_h + d_h * d_out + d_out
    mu32 = (torch.randn(n) * 0.3).float()
    sigma32 = (torch.rand(n) * 0.2 + 0.05).float()
    eps32 = torch.randn(s, n).float()
    x = torch.randn(batch, d_in, dtype=torch.float64)
    y = torch.randn(batch, d_out, dtype=torch.float64)

    def net_loss(w):
        o = 0
        w1 = w[o:o + d_in * d_h].view(d_h, d_in); o += d_in * d_h
        b1 = w[o:o + d_h]; o += d_h
        w2 = w[o:o + d_h * d_out].view(d_out, d_h); o += d_h * d_out
        b2 = w[o:o + d_out]
        h = torch.tanh(x @ w1.T + b1)
        return ((h @ w2.T + b2 - y) ** 2).mean()

    mu = mu32.double().requires_grad_(True)
    sigma = sigma32.double().requires_grad_(True)
    eps = eps32.double()
    ws = [(mu + sigma * eps[i]) for i in range(s)]
    for w in ws:
        w.retain_grad()
    data = sum(net_loss(w) for w in ws) / s
    kl = 0.5 * (sigma ** 2 + mu ** 2 - 1 - torch.log(sigma ** 2)).sum()
    (data + kl / dsize).backward()
    # autograd's dJ/dw_s carries the 1/S of the average; the path takes G_s = dLoss_s/dw_s
    G = torch.stack([w.grad * s for w in ws]).float().numpy()
    # G was rounded to fp32 for the oracle's interface: tolerance 1e-6 relative to the addends
    gmu, gsig = oracle.grad(mu32.numpy(), sigma32.numpy(), eps32.numpy(), G, s, dsize)
    scale_mu = np.abs(G).sum(0) / s + np.abs(mu32.numpy()) / dsize
    scale_sg = np.abs(G * eps32.numpy()).sum(0) / s + (sigma32.numpy() + 1 / sigma32.numpy()) / dsize
    assert np.all(np.abs(gmu - mu.grad.numpy()) <= 1e-6 * scale_mu)
    assert np.all(np.abs(gsig - sigma.grad.numpy()) <= 1e-6 * scale_sg)
    assert oracle.kl(mu32.numpy(), sigma32.numpy()) == pytest.approx(kl.item(), rel=1e-13)
    w64 = oracle.reparam(mu32.numpy(), sigma32.numpy(), eps32.numpy())
    np.testing.assert_allclose(w64, torch.stack(ws).detach().numpy(), rtol=1e-15)
    # the same with the samples on 3 "GPUs" of 2 samples each (Algorithm 2, sum convention)
    acc_mu, acc_sg = np.zeros(n), np.zeros(n)
    for p in range(3):
        a, b = oracle.grad(mu32.numpy(), sigma32.numpy(), np.ascontiguousarray(eps32.numpy()[2 * p:2 * p + 2]),
                           np.ascontiguousarray(G[2 * p:2 * p + 2]), s, dsize)
        acc_mu += a
        acc_sg += b
    assert np.all(np.abs(acc_mu - mu.grad.numpy()) <= 1e-6 * scale_mu)
    assert np.all(np.abs(acc_sg - sigma.grad.numpy()) <= 1e-6 * scale_sg)
