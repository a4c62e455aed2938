"""Pins of the Adam-step and MC-dropout oracle (oracle/update_oracle.c): closed forms of Adam's
published update, torch.optim.Adam as the library routine, and what a Bernoulli(keep) mask scaled
by 1/keep must satisfy (arxiv 2604.04736: optimizer line of Algorithms 1 / 2; section "Monte Carlo
Dropout")."""
import math

import numpy as np
import pytest
import torch


def _state(n, seed):
    r = np.random.default_rng(seed)
    return dict(mu=r.normal(size=n), sigma=r.uniform(0.05, 1.0, size=n), m_mu=np.zeros(n), v_mu=np.zeros(n),
                m_sigma=np.zeros(n), v_sigma=np.zeros(n))


def test_adam_first_step_closed_form(oracle):
    n = 6
    st = _state(n, 1)
    g_mu = np.array([1.0, -2.0, 1e-3, -5e4, 0.25, 3.0])
    g_sg = np.array([-1.0, 0.5, 2.0, 1e-5, -1e3, 7.0])
    lr, eps = 0.01, 1e-8
    mu, sg, mm, vm, ms, vs = oracle.adam_step(st["mu"], st["sigma"], g_mu, g_sg, st["m_mu"], st["v_mu"], st["m_sigma"],
                                              st["v_sigma"], step=1, lr=lr, eps=eps)
    # t = 1 from zero moments: m_hat = g, v_hat = g^2  ->  step = lr * g / (|g| + eps)
    np.testing.assert_allclose(mu, st["mu"] - lr * g_mu / (np.abs(g_mu) + eps), rtol=1e-14)
    np.testing.assert_allclose(sg, st["sigma"] - lr * g_sg / (np.abs(g_sg) + eps), rtol=1e-14)
    np.testing.assert_allclose(mm, 0.1 * g_mu, rtol=1e-15)
    np.testing.assert_allclose(vm, 0.001 * g_mu ** 2, rtol=1e-12)
    np.testing.assert_allclose(ms, 0.1 * g_sg, rtol=1e-15)
    np.testing.assert_allclose(vs, 0.001 * g_sg ** 2, rtol=1e-12)


def test_adam_constant_gradient_moves_by_lr_every_step(oracle):
    n, lr, eps, steps = 4, 1e-3, 1e-8, 50
    st = _state(n, 2)
    g = np.array([0.3, -4.0, 1e-2, 100.0])
    cur = [st[k] for k in ("mu", "sigma", "m_mu", "v_mu", "m_sigma", "v_sigma")]
    for t in range(1, steps + 1):
        cur = list(oracle.adam_step(cur[0], cur[1], g, -g, cur[2], cur[3], cur[4], cur[5], step=t, lr=lr, eps=eps))
    # bias-corrected moments of a constant gradient are the gradient itself at every step
    np.testing.assert_allclose(cur[0], st["mu"] - steps * lr * g / (np.abs(g) + eps), rtol=1e-12)
    np.testing.assert_allclose(cur[1], st["sigma"] + steps * lr * g / (np.abs(g) + eps), rtol=1e-12)


@pytest.mark.parametrize("betas,eps", [((0.9, 0.999), 1e-8), ((0.8, 0.95), 1e-3)])
def test_adam_equals_torch_optim_adam(oracle, betas, eps):
    n, lr, steps = 40, 3e-3, 12
    st = _state(n, 3)
    r = np.random.default_rng(4)
    p_mu = torch.tensor(st["mu"], dtype=torch.float64, requires_grad=True)
    p_sg = torch.tensor(st["sigma"], dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p_mu, p_sg], lr=lr, betas=betas, eps=eps)
    cur = [st[k] for k in ("mu", "sigma", "m_mu", "v_mu", "m_sigma", "v_sigma")]
    for t in range(1, steps + 1):
        g_mu = r.normal(size=n) * 10 ** r.uniform(-3, 2, size=n)
        g_sg = r.normal(size=n) * 10 ** r.uniform(-3, 2, size=n)
        p_mu.grad = torch.tensor(g_mu)
        p_sg.grad = torch.tensor(g_sg)
        opt.step()
        cur = list(oracle.adam_step(cur[0], cur[1], g_mu, g_sg, cur[2], cur[3], cur[4], cur[5], step=t, lr=lr,
                                    beta1=betas[0], beta2=betas[1], eps=eps))
        np.testing.assert_allclose(cur[0], p_mu.detach().numpy(), rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(cur[1], p_sg.detach().numpy(), rtol=1e-11, atol=1e-13)


def test_adam_grad_scale_zero_gradient_and_sigma_floor(oracle):
    n = 5
    st = _state(n, 5)
    g = np.array([1.0, -1.0, 0.5, 2.0, -3.0])
    a = oracle.adam_step(st["mu"], st["sigma"], 4 * g, 4 * g, st["m_mu"], st["v_mu"], st["m_sigma"], st["v_sigma"],
                         step=1, lr=0.1, grad_scale=0.25)
    b = oracle.adam_step(st["mu"], st["sigma"], g, g, st["m_mu"], st["v_mu"], st["m_sigma"], st["v_sigma"],
                         step=1, lr=0.1)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=1e-15)
    # zero gradient with zero moments: nothing moves
    z = oracle.adam_step(st["mu"], st["sigma"], 0 * g, 0 * g, st["m_mu"], st["v_mu"], st["m_sigma"], st["v_sigma"],
                         step=3, lr=0.1)
    np.testing.assert_array_equal(z[0], st["mu"])
    np.testing.assert_array_equal(z[1], st["sigma"])
    # a large positive gradient would push sigma below zero: the floor holds it, mu is untouched by it
    sg = np.full(n, 0.05)
    c = oracle.adam_step(st["mu"], sg, g, np.full(n, 10.0), st["m_mu"], st["v_mu"], st["m_sigma"], st["v_sigma"],
                         step=1, lr=0.1, sigma_min=1e-3)
    np.testing.assert_array_equal(c[1], np.full(n, 1e-3))
    d = oracle.adam_step(st["mu"], sg, g, np.full(n, 10.0), st["m_mu"], st["v_mu"], st["m_sigma"], st["v_sigma"],
                         step=1, lr=0.1)
    assert np.all(d[1] < 0)
    np.testing.assert_array_equal(c[0], d[0])


def test_dropout_threshold_and_hand_case(oracle):
    assert oracle.dropout_threshold(0.5) == 1 << 31
    assert oracle.dropout_threshold(1.0) == 1 << 32
    assert oracle.dropout_threshold(0.0) == 0
    assert oracle.dropout_threshold(0.75) == 3 << 30
    mu = np.array([2.0, -4.0, 8.0], np.float32)
    words = np.array([[0, (1 << 31) - 1, 1 << 31], [(1 << 32) - 1, 5, 1 << 30]], np.uint32)
    w = oracle.dropout_forward(mu, words, 0.5)
    np.testing.assert_array_equal(w, [[4.0, -8.0, 0.0], [0.0, -8.0, 16.0]])
    G = np.array([[1.0, 2.0, 3.0], [10.0, 20.0, 30.0]], np.float32)
    gm = oracle.dropout_backward(G, words, 0.5, s_total=4)
    np.testing.assert_array_equal(gm, [(1.0 * 2) / 4, (2.0 * 2 + 20.0 * 2) / 4, (30.0 * 2) / 4])
    gm = oracle.dropout_backward(G, words, 0.5, s_total=4, reduce_mean=True)
    np.testing.assert_array_equal(gm, [(1.0 * 2) / 2, (2.0 * 2 + 20.0 * 2) / 2, (30.0 * 2) / 2])


def test_dropout_with_keep_one_keeps_every_weight(oracle):
    """A Bernoulli variable with probability 1 is identically 1 (section "Monte Carlo Dropout"): also the
    largest generator word is kept, forward and backward, and the layer is then the identity in mu."""
    mu = np.array([2.0, -4.0, 8.0, 0.5], np.float32)
    words = np.array([[0, (1 << 32) - 1, 1 << 31, (1 << 32) - 2], [(1 << 32) - 1] * 4], np.uint32)
    np.testing.assert_array_equal(oracle.dropout_forward(mu, words, 1.0), np.broadcast_to(mu.astype(np.float64), (2, 4)))
    G = np.array([[1.0, 2.0, 3.0, 4.0], [10.0, 20.0, 30.0, 40.0]], np.float32)
    np.testing.assert_array_equal(oracle.dropout_backward(G, words, 1.0, s_total=2), [5.5, 11.0, 16.5, 22.0])
    # just below one, the largest word is dropped again: the threshold is floor(keep * 2^32)
    keep = 1.0 - 2.0 ** -32
    assert oracle.dropout_threshold(keep) == (1 << 32) - 1
    w = oracle.dropout_forward(mu, words, keep)
    assert w[0, 1] == 0.0 and np.all(w[1] == 0.0) and w[0, 3] == float(mu[3]) / keep
    # a keep probability below 2^-32 has threshold 0: nothing is kept
    assert oracle.dropout_threshold(2.0 ** -33) == 0
    assert np.all(oracle.dropout_forward(mu, words, 2.0 ** -33) == 0.0)


@pytest.mark.parametrize("keep", [0.5, 0.9, 0.2])
def test_dropout_is_unbiased_and_is_the_gradient_of_its_forward(oracle, keep):
    n, s = 2000, 64
    mu = np.random.default_rng(6).normal(size=n).astype(np.float32)
    mu[[0, 17, 1999]] = [1.25, -0.75, 3.5]          # so that mu +- 0.5 is exact in fp32 below
    words = oracle.eps_bits(n, s, seed=77)
    w = oracle.dropout_forward(mu, words, keep)
    kept = (w != 0) | (mu == 0)
    frac = kept.mean()
    assert abs(frac - keep) < 5 * math.sqrt(keep * (1 - keep) / kept.size)
    # every entry is either 0 or mu / keep
    np.testing.assert_allclose(w[kept], np.broadcast_to(mu.astype(np.float64) / keep, w.shape)[kept], rtol=1e-15)
    # E[w] = mu: mean over samples within 5 standard errors
    se = np.abs(mu) * math.sqrt((1 - keep) / keep / s)
    assert np.mean(np.abs(w.mean(axis=0) - mu) < 5 * se + 1e-12) > 0.999
    # the backward is the derivative of  J = g sum_s <c_s, w_s>  with respect to mu (w is linear in mu)
    c = np.random.default_rng(7).normal(size=(s, n)).astype(np.float32)
    gm = oracle.dropout_backward(c, words, keep, s_total=2 * s)
    J = lambda m: float(np.sum(c.astype(np.float64) * oracle.dropout_forward(m, words, keep))) / (2 * s)
    for i in (0, 17, 1999):
        d = np.zeros(n, np.float32)
        d[i] = 0.5
        assert (J(mu + d) - J(mu - d)) / 1.0 == pytest.approx(gm[i], rel=1e-9, abs=1e-12)
