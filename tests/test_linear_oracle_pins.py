"""Pins of the sampled-linear-layer oracle (oracle/linear_oracle.c): the layer's definition
y_s = x (mu_W + sigma_W * eps_s)^T + (mu_b + sigma_b * eps_s^b) from the reparameterisation and
ForwardPass lines of Algorithm 1 / 2 (arxiv 2604.04736), checked against numpy's einsum, against
inputs that read single sampled weights back, and against the structure of the formula."""
import numpy as np
import pytest

f32 = np.float32


def _case(seed, s=3, r=5, k=12, o=7, ldx=None):
    g = np.random.default_rng(seed)
    ldx = ldx or k
    x = np.full((r, ldx), np.nan, f32)
    x[:, :k] = g.normal(size=(r, k))
    return dict(x=x, mu_w=g.normal(size=(o, k)).astype(f32), sigma_w=g.uniform(0.01, 1, size=(o, k)).astype(f32),
                eps_w=g.normal(size=(s, o, k)), mu_b=g.normal(size=o).astype(f32),
                sigma_b=g.uniform(0.01, 1, size=o).astype(f32), eps_b=g.normal(size=(s, o)))


def test_matches_einsum(oracle):
    for seed, ldx in ((1, None), (2, 16)):
        c = _case(seed, ldx=ldx)
        k = c["mu_w"].shape[1]
        y = oracle.linear_forward(**c)
        w = c["mu_w"].astype(np.float64) + c["sigma_w"].astype(np.float64) * c["eps_w"]
        b = c["mu_b"].astype(np.float64) + c["sigma_b"].astype(np.float64) * c["eps_b"]
        want = np.einsum("rk,sok->sro", c["x"][:, :k].astype(np.float64), w) + b[:, None, :]
        np.testing.assert_allclose(y, want, rtol=1e-13, atol=1e-13)
        assert y.shape == (3, 5, 7)


def test_unit_vectors_read_sampled_weights_back(oracle):
    c = _case(3, r=12, k=12)
    c["x"] = np.eye(12, dtype=f32)
    y = oracle.linear_forward(**c)
    w = c["mu_w"].astype(np.float64) + c["sigma_w"].astype(np.float64) * c["eps_w"]       # [S, O, K]
    b = c["mu_b"].astype(np.float64) + c["sigma_b"].astype(np.float64) * c["eps_b"]
    # row k of the identity picks column k of W_s: y[s, k, o] = W_s[o, k] + b_s[o]
    np.testing.assert_allclose(y, np.transpose(w, (0, 2, 1)) + b[:, None, :], rtol=1e-15, atol=1e-15)


def test_zero_sigma_is_an_ordinary_linear_layer_for_every_sample(oracle):
    c = _case(4)
    c["sigma_w"][:] = 0
    c["sigma_b"][:] = 0
    y = oracle.linear_forward(**c)
    want = c["x"].astype(np.float64) @ c["mu_w"].astype(np.float64).T + c["mu_b"].astype(np.float64)
    for s in range(y.shape[0]):
        np.testing.assert_allclose(y[s], want, rtol=1e-14, atol=1e-14)


def test_without_bias_and_bias_only(oracle):
    c = _case(5)
    with_b = oracle.linear_forward(**c)
    nb = dict(c, mu_b=None, sigma_b=None, eps_b=None)
    without = oracle.linear_forward(**nb)
    b = c["mu_b"].astype(np.float64) + c["sigma_b"].astype(np.float64) * c["eps_b"]
    np.testing.assert_allclose(with_b - without, np.broadcast_to(b[:, None, :], with_b.shape), rtol=1e-12, atol=1e-13)
    c0 = dict(c, x=np.zeros_like(c["x"]))
    np.testing.assert_allclose(oracle.linear_forward(**c0), np.broadcast_to(b[:, None, :], with_b.shape), rtol=1e-15)


def test_linearity_in_x_and_split_of_the_inner_dimension(oracle):
    c = _case(6)
    nb = dict(c, mu_b=None, sigma_b=None, eps_b=None)
    y = oracle.linear_forward(**nb)
    y2 = oracle.linear_forward(**dict(nb, x=(c["x"] * f32(2)).astype(f32)))
    np.testing.assert_allclose(y2, 2 * y, rtol=1e-14, atol=1e-14)
    # K = 12 split into 5 + 7: the two partial layers add up
    a = dict(nb, x=np.ascontiguousarray(c["x"][:, :5]), mu_w=np.ascontiguousarray(c["mu_w"][:, :5]),
             sigma_w=np.ascontiguousarray(c["sigma_w"][:, :5]), eps_w=np.ascontiguousarray(c["eps_w"][:, :, :5]))
    b = dict(nb, x=np.ascontiguousarray(c["x"][:, 5:]), mu_w=np.ascontiguousarray(c["mu_w"][:, 5:]),
             sigma_w=np.ascontiguousarray(c["sigma_w"][:, 5:]), eps_w=np.ascontiguousarray(c["eps_w"][:, :, 5:]))
    np.testing.assert_allclose(oracle.linear_forward(**a) + oracle.linear_forward(**b), y, rtol=1e-13, atol=1e-13)


def test_samples_are_independent_slices(oracle):
    c = _case(7, s=4)
    y = oracle.linear_forward(**c)
    for s in range(4):
        one = dict(c, eps_w=c["eps_w"][s:s + 1], eps_b=c["eps_b"][s:s + 1])
        np.testing.assert_array_equal(oracle.linear_forward(**one)[0], y[s])
    # the output mean over many samples tends to the mean-weight layer (E[eps] = 0)
    g = np.random.default_rng(8)
    big = dict(c, eps_w=g.normal(size=(20000, 7, 12)), eps_b=g.normal(size=(20000, 7)))
    m = oracle.linear_forward(**big).mean(axis=0)
    det = c["x"].astype(np.float64) @ c["mu_w"].astype(np.float64).T + c["mu_b"].astype(np.float64)
    spread = np.sqrt((c["x"].astype(np.float64) ** 2) @ (c["sigma_w"].astype(np.float64) ** 2).T
                     + c["sigma_b"].astype(np.float64) ** 2)
    assert np.all(np.abs(m - det) < 5 * spread / np.sqrt(20000))


def test_per_sample_inputs_equal_one_call_per_sample(oracle):
    """x of shape [S, R, ldx] gives sample s its own input: the result must be what S separate
    calls with a shared input give, and must match einsum; identical blocks reduce to the shared case."""
    c = _case(21, s=4, r=6, k=8, o=5, ldx=12)
    g = np.random.default_rng(22)
    xs = np.full((4, 6, 12), np.nan, f32)
    xs[:, :, :8] = g.normal(size=(4, 6, 8))
    y = oracle.linear_forward(**dict(c, x=xs))
    for s in range(4):
        one = oracle.linear_forward(xs[s], c["mu_w"], c["sigma_w"], c["eps_w"][s:s + 1], c["mu_b"], c["sigma_b"],
                                    c["eps_b"][s:s + 1])
        np.testing.assert_array_equal(y[s], one[0])
    w = c["mu_w"].astype(np.float64) + c["sigma_w"].astype(np.float64) * c["eps_w"]
    b = c["mu_b"].astype(np.float64) + c["sigma_b"].astype(np.float64) * c["eps_b"]
    want = np.einsum("srk,sok->sro", xs[:, :, :8].astype(np.float64), w) + b[:, None, :]
    np.testing.assert_allclose(y, want, rtol=1e-13, atol=1e-13)
    same = np.ascontiguousarray(np.broadcast_to(c["x"], (4,) + c["x"].shape))
    np.testing.assert_array_equal(oracle.linear_forward(**dict(c, x=same)), oracle.linear_forward(**c))
    with pytest.raises(ValueError):
        oracle.linear_forward(**dict(c, x=xs[:3]))


def _loss(oracle, c, coef, x=None):
    """L = sum_s sum_{r,o} coef[s,r,o] * y_s[r,o]: a loss whose dL_s/dy_s is coef[s] exactly."""
    y = oracle.linear_forward(**(c if x is None else dict(c, x=x)))
    return float(np.sum(coef * y))


@pytest.mark.parametrize("per_sample_x", [False, True])
def test_backward_matches_central_differences_of_the_forward_oracle(oracle, per_sample_x):
    """dL/dmu, dL/dsigma (weights and biases) and dL/dx by central differences of the forward
    function; the loss is linear in every one of them, so the differences are exact up to rounding."""
    c = _case(31, s=3, r=4, k=8, o=5)
    g = np.random.default_rng(32)
    if per_sample_x:
        c["x"] = g.normal(size=(3, 4, 8)).astype(f32)
    coef = g.normal(size=(3, 4, 5)).astype(f32)
    gmw, gsw, gmb, gsb, dx = oracle.linear_backward(c["x"], coef, c["mu_w"], c["sigma_w"], c["eps_w"], c["mu_b"],
                                                    c["sigma_b"], c["eps_b"], g=1.0, k=0.0)
    h = 2.0 ** -6                      # exact in fp32 for values of order one
    for name, grad in (("mu_w", gmw), ("sigma_w", gsw), ("mu_b", gmb), ("sigma_b", gsb)):
        for idx in list(np.ndindex(c[name].shape))[::3]:
            up, dn = c[name].copy(), c[name].copy()
            up[idx] += h
            dn[idx] -= h
            fd = (_loss(oracle, dict(c, **{name: up}), coef) - _loss(oracle, dict(c, **{name: dn}), coef)) / \
                 (float(up[idx]) - float(dn[idx]))
            assert abs(fd - grad[idx]) <= 1e-9 * (1 + abs(grad[idx])), (name, idx, fd, grad[idx])
    x = c["x"]
    for idx in list(np.ndindex(x.shape))[::5]:
        up, dn = x.copy(), x.copy()
        up[idx] += h
        dn[idx] -= h
        fd = (_loss(oracle, c, coef, up) - _loss(oracle, c, coef, dn)) / (float(up[idx]) - float(dn[idx]))
        want = dx[idx] if per_sample_x else dx[(slice(None),) + idx].sum()      # a shared x collects every sample's share
        assert abs(fd - want) <= 1e-9 * (1 + abs(want)), (idx, fd, want)


def test_backward_weight_gradients_equal_the_flat_gradient_oracle(oracle):
    """The layer's weight gradients must be what the flat-vector oracle (Algorithm 2's gradient and
    averaging lines) returns for the per-sample weight gradients G_s = dy_s^T x_s formed by einsum,
    including the KL part and the sum convention's scaling."""
    c = _case(41, s=4, r=6, k=8, o=3)
    g = np.random.default_rng(42)
    dy = g.normal(size=(4, 6, 3)).astype(f32)
    s_total, dsize = 16, 450.0
    gg, kk = 1.0 / s_total, 4 / (s_total * dsize)
    gmw, gsw, gmb, gsb, dx = oracle.linear_backward(c["x"], dy, c["mu_w"], c["sigma_w"], c["eps_w"], c["mu_b"],
                                                    c["sigma_b"], c["eps_b"], g=gg, k=kk)
    G = np.einsum("sro,rk->sok", dy.astype(np.float64), c["x"].astype(np.float64))        # [S, O, K]
    # the flat oracle takes fp32 arrays: compare on inputs where G and eps are exactly representable
    G32, e32 = G.astype(f32), c["eps_w"].astype(f32)
    want_m, want_s = oracle.grad(c["mu_w"].ravel(), c["sigma_w"].ravel(), e32.reshape(4, -1), G32.reshape(4, -1), s_total, dsize)
    gmw32, gsw32, _, _, _ = oracle.linear_backward(c["x"], dy, c["mu_w"], c["sigma_w"], e32.astype(np.float64), g=gg, k=kk,
                                                   want_dx=False)
    np.testing.assert_allclose(gmw32.ravel(), want_m, rtol=1e-6, atol=1e-9)          # G32 is G rounded to fp32
    np.testing.assert_allclose(gsw32.ravel(), want_s, rtol=1e-6, atol=1e-9)
    # closed forms: the data part by einsum, the KL part mu and sigma - 1/sigma
    m64, s64 = c["mu_w"].astype(np.float64), c["sigma_w"].astype(np.float64)
    np.testing.assert_allclose(gmw, gg * G.sum(0) + kk * m64, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(gsw, gg * (G * c["eps_w"]).sum(0) + kk * (s64 - 1 / s64), rtol=1e-13, atol=1e-15)
    Gb = dy.astype(np.float64).sum(1)                                                       # [S, O]
    mb, sb = c["mu_b"].astype(np.float64), c["sigma_b"].astype(np.float64)
    np.testing.assert_allclose(gmb, gg * Gb.sum(0) + kk * mb, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(gsb, gg * (Gb * c["eps_b"]).sum(0) + kk * (sb - 1 / sb), rtol=1e-13, atol=1e-15)
    w = m64 + s64 * c["eps_w"]
    np.testing.assert_allclose(dx, np.einsum("sro,sok->srk", dy.astype(np.float64), w), rtol=1e-13, atol=1e-14)


def test_backward_special_cases(oracle):
    c = _case(51, s=2, r=3, k=4, o=2)
    zero = np.zeros((2, 3, 2), f32)
    gmw, gsw, gmb, gsb, dx = oracle.linear_backward(c["x"], zero, c["mu_w"], c["sigma_w"], c["eps_w"], c["mu_b"],
                                                    c["sigma_b"], c["eps_b"], g=0.5, k=0.25)
    np.testing.assert_array_equal(gmw, 0.25 * c["mu_w"].astype(np.float64))             # dy = 0: only the KL part is left
    s64 = c["sigma_b"].astype(np.float64)
    np.testing.assert_allclose(gsb, 0.25 * (s64 - 1 / s64), rtol=1e-15)
    assert not dx.any()
    # no bias, no dx
    out = oracle.linear_backward(c["x"], zero, c["mu_w"], c["sigma_w"], c["eps_w"], want_dx=False)
    assert out[2] is None and out[3] is None and out[4] is None
    with pytest.raises(ValueError):
        oracle.linear_backward(c["x"], zero[:, :2], c["mu_w"], c["sigma_w"], c["eps_w"])
