"""GPU parity of the fused sampled linear layer (hot_linear_forward_rng) against the triple-loop
oracle fed with the eps oracle's draw, and against the materialised path (hot_forward_rng's w).

Tolerance, per output y[s, r, o], with A = sum_k |x_k| (|mu_k| + sigma_k r_k) + |mu_b| + sigma_b r_b
(r the Box-Muller radius of the draw, the natural magnitude of eps):
    |y - y64| <= 1e-5 * A
(the default fp32 tolerance, taken relative to the sum of addend magnitudes).  It covers the fp32
draw (measured 2.6e-7 r), the rounding of w and the fp32 accumulation on the matrix cores, whose
rounding errors grow like sqrt(K) * 2^-24 in practice: the worst error measured over the shapes
below is 2.8e-7 * A at K = 2160."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def hot():
    from paper_2604_04736_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def _layer(seed, rows, k, o, ldx=None):
    g = np.random.default_rng(seed)
    ldx = ldx or k
    x = np.full((rows, ldx), np.nan, np.float32)
    x[:, :k] = g.normal(size=(rows, k))
    return dict(x=x, mu_w=(g.normal(size=(o, k)) * np.sqrt(2.0 / k)).astype(np.float32),
                sigma_w=(np.sqrt(0.01 / k) * np.exp(0.25 * g.normal(size=(o, k)))).astype(np.float32),
                mu_b=(g.normal(size=o) * 0.1).astype(np.float32),
                sigma_b=(0.05 * np.exp(0.25 * g.normal(size=o))).astype(np.float32))


def _run(hot, c, s, rng, w_off, b_off, bias=True):
    xd = torch.from_numpy(c["x"]).to(DEV)
    k, o = c["mu_w"].shape[1], c["mu_w"].shape[0]
    rows = c["x"].shape[-2]
    y = torch.full((s, rows, o), float("nan"), device=DEV)
    t = {n: torch.from_numpy(c[n]).to(DEV) for n in ("mu_w", "sigma_w", "mu_b", "sigma_b")}
    hot.hot_linear_forward_rng(rng, xd[..., :k], t["mu_w"], t["sigma_w"], t["mu_b"] if bias else None,
                               t["sigma_b"] if bias else None, y, w_off, b_off)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def _check(oracle, c, y, s, rng, w_off, b_off, bias=True):
    o, k = c["mu_w"].shape
    ew, rw = oracle.eps_normal(o * k, s, rng.seed, rng.step, rng.first_sample, with_radius=True, col0=w_off)
    ew, rw = ew.reshape(s, o, k), rw.reshape(s, o, k)
    if bias:
        eb, rb = oracle.eps_normal(o, s, rng.seed, rng.step, rng.first_sample, with_radius=True, col0=b_off)
        want = oracle.linear_forward(c["x"], c["mu_w"], c["sigma_w"], ew, c["mu_b"], c["sigma_b"], eb)
    else:
        want = oracle.linear_forward(c["x"], c["mu_w"], c["sigma_w"], ew)
    ax = np.abs(c["x"][..., :k].astype(np.float64))
    mag = np.abs(c["mu_w"].astype(np.float64))[None] + c["sigma_w"].astype(np.float64)[None] * rw      # [S, O, K]
    A = np.einsum("srk,sok->sro" if ax.ndim == 3 else "rk,sok->sro", ax, mag)
    if bias:
        A = A + (np.abs(c["mu_b"].astype(np.float64)) + c["sigma_b"].astype(np.float64) * rb)[:, None, :]
    tol = 1e-5 * A
    err = np.abs(y.astype(np.float64) - want)
    assert np.all(np.isfinite(y))
    assert np.all(err <= tol), f"worst {np.max(err / A):.3e} of the magnitude sum (allowed {np.max(tol / A):.3e})"
    return float(np.max(err / A))


# (rows, in, out, samples): the paper's MLP, ViT and SWIN layer shapes and edge cases
SHAPES = [(64, 96, 128, 4), (64, 128, 24, 4), (65, 192, 576, 4), (256, 192, 10, 4), (1, 540, 2160, 2),
          (8, 540, 2160, 2), (64, 2160, 540, 2), (130, 768, 192, 16), (1, 4, 1, 1), (17, 36, 33, 3), (33, 100, 70, 5),
          (16, 32, 64, 1), (200, 64, 16, 2)]


@pytest.mark.parametrize("rows,k,o,s", SHAPES)
def test_fused_layer_matches_oracle(oracle, hot, rows, k, o, s):
    print("case linear", rows, k, o, s, flush=True)
    c = _layer(rows * 7 + k, rows, k, o, ldx=k + 4 if rows % 2 else k)
    rng = hot.hot_rng(seed=0xABCDEF12345, step=4, first_sample=2 * s)
    w_off, b_off = 4 * 1000, 4 * 1000 + ((o * k + 3) // 4) * 4 + 8
    y = _run(hot, c, s, rng, w_off, b_off)
    worst = _check(oracle, c, y, s, rng, w_off, b_off)
    print("  worst error / magnitude sum: %.2e" % worst, flush=True)


def test_no_bias_and_zero_offsets(oracle, hot):
    c = _layer(3, 20, 64, 48)
    rng = hot.hot_rng(seed=5, step=0, first_sample=0)
    y = _run(hot, c, 3, rng, 0, 0, bias=False)
    _check(oracle, c, y, 3, rng, 0, 0, bias=False)


def test_layer_sees_the_w_of_hot_forward_rng(hot):
    """The fused layer equals x @ w_s^T + b_s with w_s, b_s materialised by hot_forward_rng on the
    flat parameter vector that holds the layer at the given offsets (fp64 matmul of those fp32 w)."""
    rows, k, o, s = 24, 128, 40, 3
    c = _layer(11, rows, k, o)
    w_off = 64
    b_off = w_off + o * k + 12
    n = b_off + o + 5
    mu = torch.zeros(n, device=DEV)
    sigma = torch.ones(n, device=DEV)
    mu[w_off:w_off + o * k] = torch.from_numpy(c["mu_w"]).flatten().to(DEV)
    sigma[w_off:w_off + o * k] = torch.from_numpy(c["sigma_w"]).flatten().to(DEV)
    mu[b_off:b_off + o] = torch.from_numpy(c["mu_b"]).to(DEV)
    sigma[b_off:b_off + o] = torch.from_numpy(c["sigma_b"]).to(DEV)
    rng = hot.hot_rng(seed=99, step=7, first_sample=1)
    plan = hot.hot_create(n, n, s, s, 1.0, 0)
    w = torch.empty(s, n, device=DEV)
    hot.hot_forward_rng(plan, rng, mu, sigma, w)
    torch.cuda.synchronize()
    hot.hot_destroy(plan)
    y = _run(hot, c, s, rng, w_off, b_off)
    w64 = w.cpu().numpy().astype(np.float64)
    x64 = c["x"].astype(np.float64)
    for si in range(s):
        ws = w64[si, w_off:w_off + o * k].reshape(o, k)
        want = x64 @ ws.T + w64[si, b_off:b_off + o]
        A = np.abs(x64) @ np.abs(ws).T + np.abs(w64[si, b_off:b_off + o])
        assert np.all(np.abs(y[si] - want) <= 1e-5 * A)


# (rows, in, out, samples): every row-tile count, sample-chunk size and a ragged everything
PER_SAMPLE = [(1, 8, 3, 2), (16, 128, 128, 4), (17, 36, 33, 5), (33, 100, 70, 3), (64, 128, 24, 16), (70, 64, 40, 2), (256, 192, 10, 1)]


@pytest.mark.parametrize("rows,k,o,s", PER_SAMPLE)
def test_fused_layer_with_one_input_per_sample(oracle, hot, rows, k, o, s):
    print("case linear per-sample x", rows, k, o, s, flush=True)
    c = _layer(rows * 13 + k, rows, k, o, ldx=k + 4 if rows % 2 else k)
    g = np.random.default_rng(rows + s)
    xs = np.full((s,) + c["x"].shape, np.nan, np.float32)
    xs[:, :, :k] = g.normal(size=(s, rows, k))
    c["x"] = xs
    rng = hot.hot_rng(seed=2024, step=4, first_sample=3)
    w_off, b_off = 16, 16 + ((o * k + 3) // 4) * 4 + 8
    y = _run(hot, c, s, rng, w_off, b_off)
    worst = _check(oracle, c, y, s, rng, w_off, b_off)
    print("  worst error / magnitude sum: %.2e" % worst, flush=True)


def test_two_layer_bayesian_mlp_forward(oracle, hot):
    """The paper's use-case-2 MLP shape in miniature: layer 1 on the shared minibatch, ReLU, layer 2
    on each sample's own activations, both with weights drawn in the kernel from one hot_rng over
    the flattened parameter vector; against the oracle run on the oracle's own activations."""
    rows, d_in, d_h, d_out, s = 48, 96, 128, 24, 4
    l1, l2 = _layer(1, rows, d_in, d_h), _layer(2, rows, d_h, d_out)
    off = {"w1": 0, "b1": d_in * d_h, "w2": d_in * d_h + d_h, "b2": d_in * d_h + d_h + d_h * d_out}
    rng = hot.hot_rng(seed=7, step=11, first_sample=0)
    t1 = {n: torch.from_numpy(l1[n]).to(DEV) for n in ("mu_w", "sigma_w", "mu_b", "sigma_b")}
    t2 = {n: torch.from_numpy(l2[n]).to(DEV) for n in ("mu_w", "sigma_w", "mu_b", "sigma_b")}
    x = torch.from_numpy(l1["x"]).to(DEV)
    h = torch.empty(s, rows, d_h, device=DEV)
    y = torch.empty(s, rows, d_out, device=DEV)
    hot.hot_linear_forward_rng(rng, x, t1["mu_w"], t1["sigma_w"], t1["mu_b"], t1["sigma_b"], h, off["w1"], off["b1"])
    a = torch.relu(h)
    hot.hot_linear_forward_rng(rng, a, t2["mu_w"], t2["sigma_w"], t2["mu_b"], t2["sigma_b"], y, off["w2"], off["b2"])
    torch.cuda.synchronize()

    def eps(n, col0, shape):
        return oracle.eps_normal(n, s, rng.seed, rng.step, rng.first_sample, col0=col0).reshape(shape)

    h64 = oracle.linear_forward(l1["x"], l1["mu_w"], l1["sigma_w"], eps(d_in * d_h, off["w1"], (s, d_h, d_in)),
                                l1["mu_b"], l1["sigma_b"], eps(d_h, off["b1"], (s, d_h)))
    a32 = np.maximum(h64, 0.0).astype(np.float32)
    y64 = oracle.linear_forward(a32, l2["mu_w"], l2["sigma_w"], eps(d_h * d_out, off["w2"], (s, d_out, d_h)),
                                l2["mu_b"], l2["sigma_b"], eps(d_out, off["b2"], (s, d_out)))
    # layer 1's error (1e-5 of its magnitude sums) passes through |W2|; bound it by the norms involved
    scale = np.abs(a32).astype(np.float64).sum(-1).max() * np.abs(l2["mu_w"]).max() + 1.0
    assert np.abs(y.cpu().numpy() - y64).max() <= 2e-5 * scale


def test_rejects_what_it_cannot_run(hot):
    x = torch.zeros(4, 8, device=DEV)
    mu = torch.zeros(3, 8, device=DEV)
    y = torch.zeros(2, 4, 3, device=DEV)
    rng = hot.hot_rng(seed=1, step=0, first_sample=0)
    with pytest.raises(hot.HotError):
        hot.hot_linear_forward_rng(rng, x, mu, mu.clone(), None, None, y, weight_offset=2)       # not a multiple of 4
    with pytest.raises(hot.HotError):
        hot.hot_linear_forward_rng(rng, x[:, :6], mu[:, :6].contiguous(), mu[:, :6].contiguous(), None, None, y)   # K % 4
    with pytest.raises(ValueError):
        hot.hot_linear_forward_rng(rng, x, mu, mu.clone(), torch.zeros(3, device=DEV), None, y)
    with pytest.raises(TypeError):
        hot.hot_linear_forward_rng(rng, x, mu, mu.clone(), None, None, y.double())
