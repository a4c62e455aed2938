"""GPU parity of the fused sampled linear layer (hot_linear_forward_rng) against the triple-loop
oracle fed with the eps oracle's draw, and against the materialised path (hot_forward_rng's w).

Tolerance, per output y[s, r, o], with A = sum_k |x_k| (|mu_k| + sigma_k r_k) + |mu_b| + sigma_b r_b
(r the Box-Muller radius of the draw, the natural magnitude of eps):
    |y - y64| <= 1e-5 * A
(the default fp32 tolerance, taken relative to the sum of addend magnitudes).  It covers the fp32
draw (measured 2.6e-7 r), the rounding of w and the fp32 accumulation on the matrix cores, whose
rounding errors grow like sqrt(K) * 2^-24 in practice: the worst error measured over the shapes
below is 2.8e-7 * A at K = 2160.  The kernels with 64 rows per wave multiply bf16 pieces of both factors
(six partial products, what they leave out is below 3 * 2^-24 of a product): the same bound holds, and
test_products_from_bf16_pieces_keep_fp32_accuracy puts values to them that use every piece."""
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
          (16, 32, 64, 1), (200, 64, 16, 2),
          # 256 rows and more on at least 128 workgroups: the kernel whose waves share the draws through LDS
          # (two samples per pass; an odd sample count; one sample with two column tiles; ragged everything)
          (300, 64, 2100, 2), (1030, 36, 2050, 3), (260, 100, 4100, 1), (513, 132, 2049, 5),
          # more than a thousand rows on layers whose tiles of 512 rows do not fill the chip (they stay with the kernel above)
          (1025, 36, 4100, 2), (1540, 20, 4160, 3), (1100, 52, 4097, 1), (2049, 16, 2500, 2)]

# 256 rows and more on layers whose tiles of 256, 512 or 1024 rows fill the chip: the kernel that loads x straight into LDS, one
# layer per launch shape it has (rows, outputs and inputs all ragged: 36, 20 and 16 inputs are 2.25, 1.25 and 1 steps of 16,
# the last block of rows is short, the last tile of outputs partly outside).  (rows, in, out, samples, launch shape as
# hot_linear_launch_shape reports it: 100 x waves + 10 x outputs per workgroup / 32 + samples per pass, + 1000 x outputs / 32
# of the launch for an odd last sample.)
SLAB_SHARED = [(2040, 36, 4090, 2, 1621), (2040, 16, 8180, 3, 1621),      # 1024 rows x 64 outputs, one sample per pass
               (1530, 20, 5400, 2, 822), (1000, 20, 2902, 2, 812),         # two samples per pass on 64 and on 32 outputs
               (1530, 20, 5400, 3, 2822), (1530, 16, 8180, 3, 1812),       # ... followed by the third on its own
               (1530, 20, 10800, 1, 841), (1530, 20, 14000, 1, 821), (7260, 20, 540, 1, 811),
               # 256 rows per workgroup (four waves), for layers that tiles of 512 rows fill badly: two samples per pass, three
               # (the last one on tiles of 32 and of 64 outputs), one
               (300, 20, 3702, 2, 412), (760, 16, 4102, 2, 412), (300, 20, 3702, 3, 1412), (700, 20, 8202, 3, 2412),
               (300, 20, 3702, 1, 411), (700, 20, 8202, 1, 421),
               # ... from 129 rows on where the layer's outputs alone fill the chip with such workgroups (the last waves without rows)
               (200, 36, 8192, 2, 412), (140, 20, 8192, 1, 411),
               # 65 to 128 rows: four waves of 32 rows each (code 2xx): two samples per pass, a third on its own, one
               (100, 20, 8192, 2, 212), (70, 8, 16384, 3, 2212), (120, 12, 16384, 1, 221)]
SLAB_PER_SAMPLE = [(2040, 24, 4090, 2, 1621), (1530, 24, 5300, 2, 841), (1530, 36, 7000, 2, 821),
                   (7260, 20, 540, 2, 811), (300, 20, 1902, 2, 411), (300, 20, 4902, 3, 421), (700, 24, 5102, 2, 421),
                   (150, 20, 8192, 2, 411), (96, 12, 12288, 2, 211), (128, 20, 8192, 2, 221)]
# (rows, in, out, samples, per-sample x, bias, launch shape of the input gradients): dy is the input there, its rows
# are read in quads, and the weight tile is drawn transposed; 38 outputs are no multiple of 4: the other kernel
SLAB_BACKWARD = [(2040, 4092, 36, 2, False, True, 1621), (1530, 5300, 36, 2, False, True, 841), (1530, 7000, 20, 2, True, False, 821),
                 (7260, 540, 20, 2, False, True, 811), (2040, 4092, 38, 2, False, True, 0),
                 (300, 1904, 20, 2, False, True, 411), (300, 4904, 20, 3, True, False, 421), (700, 5104, 24, 2, False, True, 421),
                 (180, 8192, 24, 2, False, True, 411), (100, 8192, 24, 2, False, True, 221)]


@pytest.mark.parametrize("rows,k,o,s,shape", SLAB_SHARED)
def test_fused_layer_on_the_512_row_kernel(oracle, hot, rows, k, o, s, shape):
    print("case linear, 512-row kernel", rows, k, o, s, shape, flush=True)
    ldx = k + 4 if rows % 2 else k
    assert hot.hot_linear_launch_shape(rows, k, o, s, 0, ldx=ldx) == shape
    c = _layer(rows * 7 + k, rows, k, o, ldx=ldx)
    rng = hot.hot_rng(seed=0xABCDEF12345, step=4, first_sample=2 * s)
    w_off, b_off = 4 * 1000, 4 * 1000 + ((o * k + 3) // 4) * 4 + 8
    y = _run(hot, c, s, rng, w_off, b_off)
    worst = _check(oracle, c, y, s, rng, w_off, b_off)
    print("  worst error / magnitude sum: %.2e" % worst, flush=True)


@pytest.mark.parametrize("rows,k,o,s,shape", [(1530, 20, 5400, 2, 822), (2040, 36, 4090, 2, 1621), (300, 20, 3702, 2, 412)])
def test_products_from_bf16_pieces_keep_fp32_accuracy(oracle, hot, rows, k, o, s, shape):
    """The kernels with 64 rows per wave form every product x w from three bf16 pieces of either factor (six of the
    nine partial products).  Values that put the pieces to the test: small integers (one piece each: the result must
    be the exact integer), full 24-bit mantissas (all three pieces of both factors carry bits), and magnitudes spread
    over twelve decades within one row."""
    assert hot.hot_linear_launch_shape(rows, k, o, s, 0) == shape
    g = np.random.default_rng(rows + o)
    rng = hot.hot_rng(seed=99, step=1, first_sample=0)
    zero = np.zeros((o, k), np.float32)
    # exact integers
    c = dict(x=g.integers(-64, 65, size=(rows, k)).astype(np.float32), mu_w=g.integers(-8, 9, size=(o, k)).astype(np.float32),
             sigma_w=zero, mu_b=np.zeros(o, np.float32), sigma_b=np.zeros(o, np.float32))
    y = _run(hot, c, s, rng, 0, o * k)
    want = c["x"].astype(np.int64) @ c["mu_w"].astype(np.int64).T
    assert all(np.array_equal(y[i].astype(np.int64), want) and np.array_equal(y[i], np.rint(y[i])) for i in range(s))
    # full mantissas: (2^24 - odd) * 2^e on both sides, sigma = 0: against the fp64 products
    def full(shape_, lo, hi):
        m = (2 ** 24 - 1 - 2 * g.integers(0, 2 ** 20, size=shape_)).astype(np.float64)
        return (m * 2.0 ** g.integers(lo, hi, size=shape_) * g.choice([-1.0, 1.0], size=shape_)).astype(np.float32)
    c = dict(x=full((rows, k), -30, -20), mu_w=full((o, k), -28, -22), sigma_w=zero, mu_b=np.zeros(o, np.float32), sigma_b=np.zeros(o, np.float32))
    y = _run(hot, c, s, rng, 0, o * k)
    want = c["x"].astype(np.float64) @ c["mu_w"].astype(np.float64).T
    A = np.abs(c["x"].astype(np.float64)) @ np.abs(c["mu_w"].astype(np.float64)).T
    worst = max(float(np.max(np.abs(y[i] - want) / A)) for i in range(s))
    print("  full mantissas: worst error / magnitude sum %.2e" % worst, flush=True)
    assert worst <= 1e-6        # (the six products leave out 3 * 2^-24; fp32 accumulation adds its own)
    # twelve decades in a row, drawn weights: the oracle's tolerance
    c = _layer(7, rows, k, o)
    c["x"] = (c["x"] * 10.0 ** g.uniform(-6, 6, size=c["x"].shape)).astype(np.float32)
    c["mu_w"] = (c["mu_w"] * 10.0 ** g.uniform(-3, 3, size=c["mu_w"].shape)).astype(np.float32)
    y = _run(hot, c, s, rng, 8, 8 + ((o * k + 3) // 4) * 4)
    print("  twelve decades: worst error / magnitude sum %.2e" % _check(oracle, c, y, s, rng, 8, 8 + ((o * k + 3) // 4) * 4), flush=True)


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
PER_SAMPLE = [(1, 8, 3, 2), (16, 128, 128, 4), (17, 36, 33, 5), (33, 100, 70, 3), (64, 128, 24, 16), (70, 64, 40, 2), (256, 192, 10, 1),
              (257, 68, 2064, 2), (400, 40, 2100, 3),      # the 256-row kernel with one input per sample
              # more rows: the 512-row kernel from a lower fill on than with a shared x (shapes 821, 841, 811)
              (700, 40, 2100, 3), (1030, 24, 4100, 2), (1537, 36, 3100, 3)]


@pytest.mark.parametrize("rows,k,o,s,shape", [c + (None,) for c in PER_SAMPLE] + SLAB_PER_SAMPLE)
def test_fused_layer_with_one_input_per_sample(oracle, hot, rows, k, o, s, shape):
    print("case linear per-sample x", rows, k, o, s, shape, flush=True)
    ldx = k + 4 if rows % 2 else k
    if shape is not None:
        assert hot.hot_linear_launch_shape(rows, k, o, s, 0, per_sample_x=True, ldx=ldx) == shape
    c = _layer(rows * 13 + k, rows, k, o, ldx=ldx)
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


# (rows, in, out, samples, per-sample x, bias, dx)
BACKWARD = [(1, 4, 1, 1, False, True, True), (16, 64, 16, 2, False, True, True), (17, 36, 33, 3, True, True, True),
            (33, 100, 70, 5, False, False, True), (64, 128, 24, 4, True, True, True), (64, 96, 128, 16, False, True, False),
            (70, 68, 40, 2, True, True, True), (8, 540, 2160, 2, False, True, True), (130, 192, 48, 3, True, False, True),
            (5, 2160, 540, 2, True, True, True), (1030, 64, 32, 4, False, True, True), (300, 260, 20, 16, True, True, True),
            # many rows and many tiles: a wave owns two output groups, operands prefetched; rows split over four
            # waves, and one tile per wave
            (600, 516, 1840, 2, False, True, False), (515, 1028, 3900, 1, False, True, False),
            # many rows: the input-gradient kernel whose waves share the draws (odd O: dy rows only dword-aligned,
            # a last partial step of outputs; O a multiple of the step)
            (520, 516, 33, 8, False, True, True), (1100, 1028, 48, 2, True, False, True),
            # up to 64 rows on thousands of tiles, a tile per wave (one to four 16-row blocks, the last one ragged; 2052
            # inputs are 32 tiles and 4 columns, 4100 outputs 256 groups and 4; one x per sample; no bias)
            (16, 2052, 4100, 2, False, True, False), (20, 4100, 2052, 3, True, False, False), (40, 2052, 4100, 1, False, True, False),
            (50, 2052, 4100, 2, False, True, True), (64, 516, 2100, 4, True, True, False)]


@pytest.mark.parametrize("rows,k,o,s,xs,bias,want_dx,shape", [c + (None,) for c in BACKWARD] + [c[:6] + (True, c[6]) for c in SLAB_BACKWARD])
def test_fused_layer_backward_matches_oracle(oracle, hot, rows, k, o, s, xs, bias, want_dx, shape):
    """Weight, bias and input gradients of the fused layer against the fp64 oracle, each within 1e-5
    of the sum of the magnitudes of its addends (eps taken at its Box-Muller radius, which also
    covers the 2e-6 r error of the fp32 draw)."""
    print("case linear backward", rows, k, o, s, xs, bias, want_dx, shape, flush=True)
    if shape is not None:
        assert hot.hot_linear_launch_shape(rows, k, o, s, 1, per_sample_x=xs) == shape
    c = _layer(rows * 17 + k + o, rows, k, o)
    g = np.random.default_rng(rows + 3 * s)
    if xs:
        c["x"] = g.normal(size=(s, rows, k)).astype(np.float32)
    dy = (g.normal(size=(s, rows, o)) * 10 ** g.uniform(-2, 1, size=(s, 1, o))).astype(np.float32)
    rng = hot.hot_rng(seed=77, step=5, first_sample=2)
    w_off, b_off = 32, 32 + ((o * k + 3) // 4) * 4 + 4
    s_total, dsize = 4 * s, 500.0
    t = {n: torch.from_numpy(c[n]).to(DEV) for n in ("x", "mu_w", "sigma_w", "mu_b", "sigma_b")}
    out = {"gmw": torch.full((o, k), float("nan"), device=DEV), "gsw": torch.full((o, k), float("nan"), device=DEV),
           "gmb": torch.full((o,), float("nan"), device=DEV), "gsb": torch.full((o,), float("nan"), device=DEV),
           "dx": torch.full((s, rows, k), float("nan"), device=DEV)}
    hot.hot_linear_backward_rng(rng, t["x"], torch.from_numpy(dy).to(DEV), t["mu_w"], t["sigma_w"],
                                t["mu_b"] if bias else None, t["sigma_b"] if bias else None, out["gmw"], out["gsw"],
                                out["gmb"] if bias else None, out["gsb"] if bias else None, out["dx"] if want_dx else None,
                                s_total, dsize, hot.HOT_REDUCE_SUM, w_off, b_off)
    torch.cuda.synchronize()
    got = {n: v.cpu().numpy().astype(np.float64) for n, v in out.items()}

    ew, rw = oracle.eps_normal(o * k, s, rng.seed, rng.step, rng.first_sample, with_radius=True, col0=w_off)
    ew, rw = ew.reshape(s, o, k), rw.reshape(s, o, k)
    eb, rb = oracle.eps_normal(o, s, rng.seed, rng.step, rng.first_sample, with_radius=True, col0=b_off)
    gg, kk = 1.0 / s_total, s / (s_total * dsize)
    want = oracle.linear_backward(c["x"], dy, c["mu_w"], c["sigma_w"], ew, c["mu_b"] if bias else None,
                                  c["sigma_b"] if bias else None, eb if bias else None, g=gg, k=kk, want_dx=want_dx)
    ax, ady = np.abs(c["x"].astype(np.float64)), np.abs(dy.astype(np.float64))
    Gabs = np.matmul(ady.transpose(0, 2, 1), ax)                                              # [S, O, K]
    m64, s64 = np.abs(c["mu_w"].astype(np.float64)), c["sigma_w"].astype(np.float64)
    checks = [("gmw", want[0], gg * Gabs.sum(0) + kk * m64), ("gsw", want[1], gg * (Gabs * rw).sum(0) + kk * (s64 + 1 / s64))]
    if bias:
        Gb = ady.sum(1)
        mb, sb = np.abs(c["mu_b"].astype(np.float64)), c["sigma_b"].astype(np.float64)
        checks += [("gmb", want[2], gg * Gb.sum(0) + kk * mb), ("gsb", want[3], gg * (Gb * rb).sum(0) + kk * (sb + 1 / sb))]
    else:
        assert np.isnan(got["gmb"]).all() and np.isnan(got["gsb"]).all()
    if want_dx:
        checks.append(("dx", want[4], np.einsum("sro,sok->srk", ady, m64[None] + s64[None] * rw)))
    else:
        assert np.isnan(got["dx"]).all()
    for name, w64, A in checks:
        err = np.abs(got[name] - w64)
        assert np.all(np.isfinite(got[name])), name
        assert np.all(err <= 1e-5 * A), f"{name}: worst {np.max(err / A):.3e} of the magnitude sum"
        print("  %s worst error / magnitude sum: %.2e" % (name, np.max(err / A)), flush=True)


# (rows, in, out, samples, per-sample x, bias, dx, fraction of the wanted workspace, expected use of it)
WITH_WORKSPACE = [(4200, 64, 48, 2, False, True, False, 1.0, True), (17000, 36, 20, 3, True, True, False, 1.0, True),
                  (17000, 36, 20, 2, False, False, False, 0.3, True), (17000, 36, 20, 2, False, True, False, 0.01, False),
                  (2100, 516, 1840, 1, False, True, False, 1.0, True), (300, 64, 48, 2, False, True, False, 1.0, False),
                  # rows enough for wide tiles through parts: all of the workspace, a part of it, too little for any part
                  (8200, 256, 512, 1, False, True, False, 1.0, True), (8200, 256, 512, 1, False, True, False, 0.3, True),
                  (8200, 256, 512, 1, False, True, False, 0.05, False),
                  # input gradients on too few 256-row workgroups: the outputs cut into parts (ragged last part; a
                  # workspace for fewer parts; none)
                  (1030, 132, 700, 2, False, True, True, 1.0, True), (300, 36, 333, 3, True, False, True, 1.0, True),
                  (1030, 132, 700, 2, False, True, True, 0.6, True), (1030, 132, 700, 2, False, True, True, 0.1, False),
                  # ... from 129 rows on (one 256-row workgroup per 64 inputs, its last waves without rows)
                  (200, 132, 700, 2, False, True, True, 1.0, True),
                  # the shape on which one accumulator register was once read before the matrix pipeline had written it
                  # (a partial last row block in a tile without biases; the kernels now wait explicitly)
                  (19549, 84, 1744, 1, False, True, False, 1.0, True)]


@pytest.mark.parametrize("rows,k,o,s,xs,bias,want_dx,fraction,used", WITH_WORKSPACE)
def test_backward_with_a_workspace_matches_oracle(oracle, hot, rows, k, o, s, xs, bias, want_dx, fraction, used):
    """hot_linear_backward_rng_ws.  Weight gradients of few tiles and many rows: the rows cut into parts over
    workgroups, partial sums in the caller's workspace, added in part order by a second kernel.  Input gradients
    on too few workgroups: the outputs cut into parts the same way.  Everything against the oracle to the same
    bound as without a workspace; a workspace smaller than asked for (fewer parts, or none) and a shape that
    wants none give the same; the workspace is the only memory written besides the outputs."""
    _backward_with_a_workspace(oracle, hot, rows, k, o, s, xs, bias, want_dx, fraction, used)


# (rows, in, out, samples, per-sample x, bias, fraction of the wanted workspace, expected use of it, shape code)
# every instantiation of the two kernels (a wave draws whole tiles: 16-row blocks x samples held 12, 14, 18, 22, 24; the
# waves split the rows: 112, 122); inputs that are not a multiple of 64 and outputs that are not a multiple of 16; a
# last row block with one row, a wave without rows; half the workspace (fewer parts); too little for two parts (the
# separate kernels run); 200 strips of inputs (one part, no workspace needed)
ONE_PASS = [(16, 2052, 4100, 2, False, True, 1.0, True, 12), (5, 2160, 540, 1, True, True, 1.0, True, 12),
            (13, 132, 1000, 3, False, True, 1.0, True, 14), (9, 132, 1000, 7, True, False, 1.0, True, 18),
            (17, 36, 330, 2, False, True, 1.0, True, 22), (20, 4100, 2052, 3, True, False, 1.0, True, 24),
            (16, 2052, 4100, 2, False, True, 0.05, False, 12), (3, 12800, 40, 2, False, True, 1.0, False, 12),
            (50, 2052, 4100, 2, False, True, 1.0, True, 112), (64, 516, 2100, 2, True, True, 0.5, True, 112),
            (33, 1028, 520, 1, False, False, 1.0, True, 112), (100, 260, 2100, 2, False, True, 1.0, True, 122),
            (128, 516, 1100, 1, True, True, 1.0, True, 122), (70, 2052, 300, 2, True, False, 0.6, True, 122)]


@pytest.mark.parametrize("rows,k,o,s,xs,bias,fraction,used,shape", ONE_PASS)
def test_backward_in_one_pass_matches_oracle(oracle, hot, rows, k, o, s, xs, bias, fraction, used, shape):
    """Up to 128 rows with dx wanted: hot_linear_backward_rng_ws takes weight, bias and input gradients in one pass
    over the weights (every eps drawn once); same bounds against the oracle as the separate kernels."""
    assert hot.hot_linear_launch_shape(rows, k, o, s, 2, per_sample_x=xs) == shape
    _backward_with_a_workspace(oracle, hot, rows, k, o, s, xs, bias, True, fraction, used, wants_none=((rows, k) == (3, 12800)))


def _backward_with_a_workspace(oracle, hot, rows, k, o, s, xs, bias, want_dx, fraction, used, wants_none=None):
    print("case linear backward with workspace", rows, k, o, s, xs, bias, want_dx, fraction, flush=True)
    c = _layer(rows + k + o, rows, k, o)
    g = np.random.default_rng(rows + s)
    if xs:
        c["x"] = g.normal(size=(s, rows, k)).astype(np.float32)
    dy = (g.normal(size=(s, rows, o)) * 10 ** g.uniform(-2, 1, size=(s, 1, o))).astype(np.float32)
    rng = hot.hot_rng(seed=31, step=2, first_sample=0)
    w_off, b_off = 16, 16 + o * k
    s_total, dsize = 2 * s, 800.0
    want_bytes = hot.hot_linear_backward_workspace_bytes(rows, k, o, s)
    assert (want_bytes > 0) == ((used or fraction <= 0.1) if wants_none is None else not wants_none), want_bytes
    n_ws = max(int(want_bytes * fraction) // 16 * 4, 4)
    ws = torch.full((n_ws + 8,), float("nan"), device=DEV)
    t = {n: torch.from_numpy(c[n]).to(DEV) for n in ("x", "mu_w", "sigma_w", "mu_b", "sigma_b")}
    out = {"gmw": torch.full((o, k), float("nan"), device=DEV), "gsw": torch.full((o, k), float("nan"), device=DEV),
           "gmb": torch.full((o,), float("nan"), device=DEV), "gsb": torch.full((o,), float("nan"), device=DEV),
           "dx": torch.full((s, rows, k), float("nan"), device=DEV)}
    hot.hot_linear_backward_rng(rng, t["x"], torch.from_numpy(dy).to(DEV), t["mu_w"], t["sigma_w"],
                                t["mu_b"] if bias else None, t["sigma_b"] if bias else None, out["gmw"], out["gsw"],
                                out["gmb"] if bias else None, out["gsb"] if bias else None, out["dx"] if want_dx else None,
                                s_total, dsize, hot.HOT_REDUCE_SUM, w_off, b_off, workspace=ws[:n_ws])
    torch.cuda.synchronize()
    assert bool(torch.isnan(ws[n_ws:]).all()), "written beyond the workspace"
    assert bool(torch.isnan(ws[:n_ws]).all()) != used, "workspace use is not what the shape and its size call for"
    got = {n: v.cpu().numpy().astype(np.float64) for n, v in out.items()}
    ew, rw = oracle.eps_normal(o * k, s, rng.seed, rng.step, rng.first_sample, with_radius=True, col0=w_off)
    ew, rw = ew.reshape(s, o, k), rw.reshape(s, o, k)
    eb, rb = oracle.eps_normal(o, s, rng.seed, rng.step, rng.first_sample, with_radius=True, col0=b_off)
    gg, kk = 1.0 / s_total, s / (s_total * dsize)
    want = oracle.linear_backward(c["x"], dy, c["mu_w"], c["sigma_w"], ew, c["mu_b"] if bias else None,
                                  c["sigma_b"] if bias else None, eb if bias else None, g=gg, k=kk, want_dx=want_dx)
    ax, ady = np.abs(c["x"].astype(np.float64)), np.abs(dy.astype(np.float64))
    Gabs = np.matmul(ady.transpose(0, 2, 1), ax)
    m64, s64 = np.abs(c["mu_w"].astype(np.float64)), c["sigma_w"].astype(np.float64)
    checks = [("gmw", want[0], gg * Gabs.sum(0) + kk * m64), ("gsw", want[1], gg * (Gabs * rw).sum(0) + kk * (s64 + 1 / s64))]
    if bias:
        Gb = ady.sum(1)
        mb, sb = np.abs(c["mu_b"].astype(np.float64)), c["sigma_b"].astype(np.float64)
        checks += [("gmb", want[2], gg * Gb.sum(0) + kk * mb), ("gsb", want[3], gg * (Gb * rb).sum(0) + kk * (sb + 1 / sb))]
    if want_dx:
        checks.append(("dx", want[4], np.matmul(ady, m64[None] + s64[None] * rw)))
    for name, w64, A in checks:
        err = np.abs(got[name] - w64)
        assert np.all(np.isfinite(got[name])), name
        assert np.all(err <= 1e-5 * A), f"{name}: worst {np.max(err / A):.3e} of the magnitude sum"


def test_workspace_arguments_are_checked(hot):
    x, w, dy = torch.zeros(4, 8, device=DEV), torch.ones(3, 8, device=DEV), torch.zeros(2, 4, 3, device=DEV)
    rng = hot.hot_rng(seed=1, step=0, first_sample=0)
    ws = torch.zeros(64, device=DEV)
    with pytest.raises(hot.HotError):       # not 16-byte aligned
        hot.hot_linear_backward_rng(rng, x, dy, w, w.clone(), None, None, w.clone(), w.clone(), None, None, None, 2, 1.0, workspace=ws[1:])
    with pytest.raises(TypeError):
        hot.hot_linear_backward_rng(rng, x, dy, w, w.clone(), None, None, w.clone(), w.clone(), None, None, None, 2, 1.0, workspace=ws.cpu())
    hot.hot_linear_backward_rng(rng, x, dy, w, w.clone(), None, None, w.clone(), w.clone(), None, None, None, 2, 1.0, workspace=ws)
    torch.cuda.synchronize()
    with pytest.raises(hot.HotError):
        hot.hot_linear_backward_workspace_bytes(0, 8, 3, 2)


def test_fused_backward_equals_flat_backward_on_materialised_gradients(hot):
    """The layer's weight gradients against hot_backward_rng fed with G_s = dy_s^T x (fp64 einsum,
    rounded to fp32) on the flat parameter vector that holds the layer at its offsets: the same
    draws, the same scaling, the same KL part."""
    rows, k, o, s = 24, 64, 40, 3
    c = _layer(5, rows, k, o)
    g = np.random.default_rng(6)
    dy = g.normal(size=(s, rows, o)).astype(np.float32)
    w_off = 128
    n = w_off + o * k
    rng = hot.hot_rng(seed=4242, step=9, first_sample=0)
    mu = torch.zeros(n, device=DEV)
    sigma = torch.ones(n, device=DEV)
    mu[w_off:] = torch.from_numpy(c["mu_w"]).flatten().to(DEV)
    sigma[w_off:] = torch.from_numpy(c["sigma_w"]).flatten().to(DEV)
    G = np.zeros((s, n), np.float32)
    G[:, w_off:] = np.einsum("sro,rk->sok", dy.astype(np.float64), c["x"].astype(np.float64)).reshape(s, -1)
    plan = hot.hot_create(n, n, s, 2 * s, 300.0, 0)
    gmu, gsig = torch.empty(n, device=DEV), torch.empty(n, device=DEV)
    hot.hot_backward_rng(plan, rng, mu, sigma, torch.from_numpy(G).to(DEV), gmu, gsig)
    hot.hot_destroy(plan)
    gmw, gsw = torch.empty(o, k, device=DEV), torch.empty(o, k, device=DEV)
    hot.hot_linear_backward_rng(rng, torch.from_numpy(c["x"]).to(DEV), torch.from_numpy(dy).to(DEV),
                                torch.from_numpy(c["mu_w"]).to(DEV), torch.from_numpy(c["sigma_w"]).to(DEV), None, None,
                                gmw, gsw, None, None, None, 2 * s, 300.0, hot.HOT_REDUCE_SUM, w_off, 0)
    torch.cuda.synchronize()
    A = np.abs(G[:, w_off:]).sum(0).reshape(o, k) / (2 * s) + 1e-3
    assert np.all(np.abs(gmw.cpu().numpy() - gmu[w_off:].cpu().numpy().reshape(o, k)) <= 1e-5 * A)
    assert np.all(np.abs(gsw.cpu().numpy() - gsig[w_off:].cpu().numpy().reshape(o, k)) <= 6e-5 * A)


def test_backward_rejects_what_it_cannot_run(hot):
    x = torch.zeros(4, 8, device=DEV)
    w = torch.ones(3, 8, device=DEV)
    dy = torch.zeros(2, 4, 3, device=DEV)
    b = torch.ones(3, device=DEV)
    rng = hot.hot_rng(seed=1, step=0, first_sample=0)
    with pytest.raises(ValueError):
        hot.hot_linear_backward_rng(rng, x, dy, w, w.clone(), b, b.clone(), w.clone(), w.clone(), None, None, None, 2, 1.0)
    with pytest.raises(hot.HotError):
        hot.hot_linear_backward_rng(rng, x, dy, w, w.clone(), None, None, w.clone(), w.clone(), None, None, None, 1, 1.0)   # S < S_loc
    with pytest.raises(hot.HotError):
        hot.hot_linear_backward_rng(rng, x, dy, w, w.clone(), None, None, w.clone(), w.clone(), None, None, None, 2, 0.0)   # |D| = 0
    with pytest.raises(TypeError):
        hot.hot_linear_backward_rng(rng, x, dy[:, :3], w, w.clone(), None, None, w.clone(), w.clone(), None, None, None, 2, 1.0)


def test_autograd_two_layer_mlp_on_the_fused_layers(hot):
    """BayesianLinear under torch.autograd: gradients of a two-layer tanh MLP (layer 1 on the shared
    minibatch, layer 2 on per-sample activations) against fp64 autograd on the CPU with the very
    same eps (taken from hot_sample_eps over the flat parameter range), KL/|D| included; then a few
    Adam steps lower the loss."""
    from paper_2604_04736_amd.autograd import BayesianLinear
    torch.manual_seed(3)
    d_in, d_h, d_out, batch, s, dsize = 8, 32, 4, 64, 4, 2000.0
    l1 = BayesianLinear(d_in, d_h, s, dsize, seed=11)
    l2 = BayesianLinear(d_h, d_out, s, dsize, seed=11, weight_offset=l1.next_offset)
    n = l2.next_offset
    xb = torch.randn(batch, d_in, device=DEV)
    yb = torch.sin(xb[:, :d_out] * 2.0)
    p = {"w1": (torch.randn(d_h, d_in, device=DEV) * 0.3), "b1": torch.zeros(d_h, device=DEV),
         "w2": (torch.randn(d_out, d_h, device=DEV) * 0.2), "b2": torch.zeros(d_out, device=DEV)}
    mu = {k: v.clone().requires_grad_(True) for k, v in p.items()}
    sg = {k: torch.full_like(v, 0.05).requires_grad_(True) for k, v in p.items()}

    def loss_of(step):
        h = torch.tanh(l1.forward(xb, mu["w1"], sg["w1"], mu["b1"], sg["b1"], step))
        y = l2.forward(h, mu["w2"], sg["w2"], mu["b2"], sg["b2"], step)
        return ((y - yb[None]) ** 2).mean(dim=(1, 2)).sum() / s

    loss = loss_of(0)
    loss.backward()

    plan = hot.hot_create(n, n, s, s, dsize, 0)
    eps = torch.empty(s, n, device=DEV)
    hot.hot_sample_eps(plan, hot.hot_rng(seed=11, step=0, first_sample=0), eps)
    hot.hot_destroy(plan)
    e = eps.double().cpu()
    off = {"w1": (l1.weight_offset, (d_h, d_in)), "b1": (l1.bias_offset, (d_h,)),
           "w2": (l2.weight_offset, (d_out, d_h)), "b2": (l2.bias_offset, (d_out,))}
    m64 = {k: v.detach().double().cpu().requires_grad_(True) for k, v in mu.items()}
    s64 = {k: v.detach().double().cpu().requires_grad_(True) for k, v in sg.items()}
    x64, y64 = xb.double().cpu(), yb.double().cpu()
    ref = 0.0
    for i in range(s):
        w = {k: m64[k] + s64[k] * e[i, o:o + int(np.prod(shape))].view(shape) for k, (o, shape) in off.items()}
        out = torch.tanh(x64 @ w["w1"].T + w["b1"]) @ w["w2"].T + w["b2"]
        ref = ref + ((out - y64) ** 2).mean() / s
    kl = sum(0.5 * (s64[k] ** 2 + m64[k] ** 2 - 1 - 2 * torch.log(s64[k])).sum() for k in m64)
    (ref + kl / dsize).backward()
    assert abs(loss.item() - ref.item()) <= 1e-5 * abs(ref.item())
    kl_gpu = l1.kl(mu["w1"], sg["w1"], mu["b1"], sg["b1"]) + l2.kl(mu["w2"], sg["w2"], mu["b2"], sg["b2"])
    assert abs(kl_gpu.item() - kl.item()) <= 1e-7 * abs(kl.item())
    for k in mu:
        for got, want in ((mu[k].grad, m64[k].grad), (sg[k].grad, s64[k].grad)):
            scale = want.abs().max().item()
            assert (got.double().cpu() - want).abs().max().item() <= 1e-4 * scale, k

    names = list(mu)
    state = {k: [torch.zeros_like(mu[k]).view(-1) for _ in range(4)] for k in names}
    first = last = None
    for t in range(1, 41):
        for k in names:
            mu[k].grad = sg[k].grad = None
        loss = loss_of(t)
        loss.backward()
        for k in names:
            hot.hot_adam_step(hot.hot_adam(2e-2, 0.9, 0.999, 1e-8, 1.0, 1e-4, t), mu[k].data.view(-1), sg[k].data.view(-1),
                              mu[k].grad.view(-1), sg[k].grad.view(-1), *state[k])
        first = loss.item() if first is None else first
        last = loss.item()
    assert last < 0.5 * first, (first, last)


@pytest.mark.parametrize("flag_name", ["HOT_REDUCE_SUM", "HOT_REDUCE_MEAN", "HOT_REDUCE_NONE"])
def test_backward_scaling_conventions(oracle, hot, flag_name):
    """g and the KL weight under the three conventions: 1/S and S_loc/(S |D|); 1/S_loc and 1/|D|; 1 and 1/|D|."""
    rows, k, o, s, s_total, dsize = 12, 32, 20, 3, 12, 50.0
    c = _layer(77, rows, k, o)
    g = np.random.default_rng(78)
    dy = g.normal(size=(s, rows, o)).astype(np.float32)
    rng = hot.hot_rng(seed=8, step=1, first_sample=0)
    gg, kk = {"HOT_REDUCE_SUM": (1 / s_total, s / (s_total * dsize)), "HOT_REDUCE_MEAN": (1 / s, 1 / dsize),
              "HOT_REDUCE_NONE": (1.0, 1 / dsize)}[flag_name]
    t = {n: torch.from_numpy(c[n]).to(DEV) for n in ("x", "mu_w", "sigma_w", "mu_b", "sigma_b")}
    out = [torch.empty(o, k, device=DEV), torch.empty(o, k, device=DEV), torch.empty(o, device=DEV), torch.empty(o, device=DEV)]
    hot.hot_linear_backward_rng(rng, t["x"], torch.from_numpy(dy).to(DEV), t["mu_w"], t["sigma_w"], t["mu_b"], t["sigma_b"],
                                *out, None, s_total, dsize, getattr(hot, flag_name), 0, o * k)
    torch.cuda.synchronize()
    ew = oracle.eps_normal(o * k, s, 8, 1, 0).reshape(s, o, k)
    eb = oracle.eps_normal(o, s, 8, 1, 0, col0=o * k)
    want = oracle.linear_backward(c["x"], dy, c["mu_w"], c["sigma_w"], ew, c["mu_b"], c["sigma_b"], eb, g=gg, k=kk, want_dx=False)
    for got, w64 in zip(out, want[:4]):
        scale = np.abs(w64).max()
        assert np.abs(got.cpu().numpy() - w64).max() <= 2e-5 * scale


def test_random_layer_shapes_forward_and_backward(oracle, hot):
    """Seeded random draw of layer shapes (every combination of ragged rows, inputs, outputs, sample
    counts, shared or per-sample input, with and without bias): forward and backward against the oracle."""
    rs = np.random.default_rng(424242)
    for case in range(24):
        rows = int(rs.choice([rs.integers(1, 17), rs.integers(17, 70), rs.integers(70, 200)]))
        k = 4 * int(rs.integers(1, 90))
        o = int(rs.choice([rs.integers(1, 17), rs.integers(17, 150)]))
        s = int(rs.integers(1, 7))
        xs, bias = bool(rs.integers(0, 2)), bool(rs.integers(0, 2))
        print("case random layer", case, rows, k, o, s, xs, bias, flush=True)
        c = _layer(1000 + case, rows, k, o)
        if xs:
            c["x"] = rs.normal(size=(s, rows, k)).astype(np.float32)
        dy = rs.normal(size=(s, rows, o)).astype(np.float32)
        rng = hot.hot_rng(seed=int(rs.integers(0, 2 ** 62)), step=int(rs.integers(0, 1000)), first_sample=int(rs.integers(0, 50)))
        w_off = 4 * int(rs.integers(0, 1000))
        b_off = w_off + o * k + 4 * int(rs.integers(0, 10))
        y = _run(hot, c, s, rng, w_off, b_off, bias=bias)
        _check(oracle, c, y, s, rng, w_off, b_off, bias=bias)

        t = {n: torch.from_numpy(c[n]).to(DEV) for n in ("x", "mu_w", "sigma_w", "mu_b", "sigma_b")}
        gmw, gsw = torch.empty(o, k, device=DEV), torch.empty(o, k, device=DEV)
        gmb, gsb = torch.empty(o, device=DEV), torch.empty(o, device=DEV)
        dx = torch.empty(s, rows, k, device=DEV)
        hot.hot_linear_backward_rng(rng, t["x"], torch.from_numpy(dy).to(DEV), t["mu_w"], t["sigma_w"],
                                    t["mu_b"] if bias else None, t["sigma_b"] if bias else None, gmw, gsw,
                                    gmb if bias else None, gsb if bias else None, dx, 3 * s, 77.0, hot.HOT_REDUCE_SUM, w_off, b_off)
        torch.cuda.synchronize()
        ew, rw = oracle.eps_normal(o * k, s, rng.seed, rng.step, rng.first_sample, with_radius=True, col0=w_off)
        ew, rw = ew.reshape(s, o, k), rw.reshape(s, o, k)
        eb, rb = oracle.eps_normal(o, s, rng.seed, rng.step, rng.first_sample, with_radius=True, col0=b_off)
        gg, kk = 1.0 / (3 * s), s / (3 * s * 77.0)
        want = oracle.linear_backward(c["x"], dy, c["mu_w"], c["sigma_w"], ew, c["mu_b"] if bias else None,
                                      c["sigma_b"] if bias else None, eb if bias else None, g=gg, k=kk)
        ax, ady = np.abs(c["x"].astype(np.float64)), np.abs(dy.astype(np.float64))
        Gabs = np.einsum("sro,srk->sok" if xs else "sro,rk->sok", ady, ax)
        m64, s64 = np.abs(c["mu_w"].astype(np.float64)), c["sigma_w"].astype(np.float64)
        checks = [(gmw, want[0], gg * Gabs.sum(0) + kk * m64), (gsw, want[1], gg * (Gabs * rw).sum(0) + kk * (s64 + 1 / s64)),
                  (dx, want[4], np.einsum("sro,sok->srk", ady, m64[None] + s64[None] * rw))]
        if bias:
            Gb = ady.sum(1)
            mb, sb = np.abs(c["mu_b"].astype(np.float64)), c["sigma_b"].astype(np.float64)
            checks += [(gmb, want[2], gg * Gb.sum(0) + kk * mb), (gsb, want[3], gg * (Gb * rb).sum(0) + kk * (sb + 1 / sb))]
        for got, w64, A in checks:
            assert np.all(np.abs(got.cpu().numpy().astype(np.float64) - w64) <= 1e-5 * A), case


def test_swin_layer_at_its_full_size_on_sampled_blocks(oracle, hot):
    """The layer shape the benchmark times for many rows (7260 tokens, 540 -> 2160, two samples), in the
    kernels the default dispatch picks there, against the oracle on blocks it can afford: y for 24 rows x 24
    outputs, the weight gradients of 24 outputs (all rows, all inputs), the bias gradients of those outputs,
    and dx for 24 rows (all outputs, all inputs).  Rows of y and dx and outputs of the weight gradients do
    not depend on one another, so each block is the oracle's result for the sub-layer it spans."""
    rows, k, o, s = 7260, 540, 2160, 2
    print("case linear layer at full size", rows, k, o, s, flush=True)
    c = _layer(99, rows, k, o)
    g = np.random.default_rng(5)
    dy = (g.normal(size=(s, rows, o)) * 0.1).astype(np.float32)
    rng = hot.hot_rng(seed=2025, step=11, first_sample=1)
    w_off, b_off = 64, 64 + o * k
    s_total, dsize = 8, 45000.0
    t = {n: torch.from_numpy(c[n]).to(DEV) for n in ("x", "mu_w", "sigma_w", "mu_b", "sigma_b")}
    y = torch.full((s, rows, o), float("nan"), device=DEV)
    hot.hot_linear_forward_rng(rng, t["x"], t["mu_w"], t["sigma_w"], t["mu_b"], t["sigma_b"], y, w_off, b_off)
    out = {"gmw": torch.full((o, k), float("nan"), device=DEV), "gsw": torch.full((o, k), float("nan"), device=DEV),
           "gmb": torch.full((o,), float("nan"), device=DEV), "gsb": torch.full((o,), float("nan"), device=DEV),
           "dx": torch.full((s, rows, k), float("nan"), device=DEV)}
    hot.hot_linear_backward_rng(rng, t["x"], torch.from_numpy(dy).to(DEV), t["mu_w"], t["sigma_w"], t["mu_b"], t["sigma_b"],
                                out["gmw"], out["gsw"], out["gmb"], out["gsb"], out["dx"], s_total, dsize,
                                hot.HOT_REDUCE_SUM, w_off, b_off)
    torch.cuda.synchronize()
    for v in list(out.values()) + [y]:
        assert bool(torch.isfinite(v).all())
    ew, rw = oracle.eps_normal(o * k, s, rng.seed, rng.step, rng.first_sample, with_radius=True, col0=w_off)
    ew, rw = ew.reshape(s, o, k), rw.reshape(s, o, k)
    eb, rb = oracle.eps_normal(o, s, rng.seed, rng.step, rng.first_sample, with_radius=True, col0=b_off)
    r_sub = np.sort(np.concatenate([[0, 255, 256, rows - 1], g.choice(rows, 20, replace=False)]))
    o_sub = np.sort(np.concatenate([[0, 15, 16, o - 1], g.choice(o, 20, replace=False)]))
    m64, s64 = np.abs(c["mu_w"].astype(np.float64)), c["sigma_w"].astype(np.float64)
    ax, ady = np.abs(c["x"].astype(np.float64)), np.abs(dy.astype(np.float64))
    gg, kk = 1.0 / s_total, s / (s_total * dsize)

    # forward block
    sub = dict(x=c["x"][r_sub], mu_w=c["mu_w"][o_sub], sigma_w=c["sigma_w"][o_sub], mu_b=c["mu_b"][o_sub], sigma_b=c["sigma_b"][o_sub])
    want = oracle.linear_forward(sub["x"], sub["mu_w"], sub["sigma_w"], np.ascontiguousarray(ew[:, o_sub]), sub["mu_b"],
                                 sub["sigma_b"], np.ascontiguousarray(eb[:, o_sub]))
    A = np.einsum("rk,sok->sro", ax[r_sub], m64[o_sub][None] + s64[o_sub][None] * rw[:, o_sub]) + \
        (np.abs(c["mu_b"][o_sub].astype(np.float64)) + c["sigma_b"][o_sub].astype(np.float64) * rb[:, o_sub])[:, None, :]
    got = y.cpu().numpy()[:, r_sub][:, :, o_sub].astype(np.float64)
    assert np.all(np.abs(got - want) <= 1e-5 * A), f"y: worst {np.max(np.abs(got - want) / A):.2e}"

    # weight and bias gradients of the chosen outputs
    wb = oracle.linear_backward(c["x"], np.ascontiguousarray(dy[:, :, o_sub]), sub["mu_w"], sub["sigma_w"],
                                np.ascontiguousarray(ew[:, o_sub]), sub["mu_b"], sub["sigma_b"], np.ascontiguousarray(eb[:, o_sub]),
                                g=gg, k=kk, want_dx=False)
    Gabs = np.matmul(ady[:, :, o_sub].transpose(0, 2, 1), ax)                                  # [S, |o_sub|, K]
    Gb = ady[:, :, o_sub].sum(1)
    mb, sb = np.abs(c["mu_b"][o_sub].astype(np.float64)), c["sigma_b"][o_sub].astype(np.float64)
    for name, w64, mag in (("gmw", wb[0], gg * Gabs.sum(0) + kk * m64[o_sub]),
                           ("gsw", wb[1], gg * (Gabs * rw[:, o_sub]).sum(0) + kk * (s64[o_sub] + 1 / s64[o_sub])),
                           ("gmb", wb[2], gg * Gb.sum(0) + kk * mb), ("gsb", wb[3], gg * (Gb * rb[:, o_sub]).sum(0) + kk * (sb + 1 / sb))):
        err = np.abs(out[name].cpu().numpy()[o_sub].astype(np.float64) - w64)
        assert np.all(err <= 1e-5 * mag), f"{name}: worst {np.max(err / mag):.2e}"

    # input gradients of the chosen rows
    xb = oracle.linear_backward(c["x"][r_sub], np.ascontiguousarray(dy[:, r_sub]), c["mu_w"], c["sigma_w"], ew, None, None, None,
                                g=gg, k=kk, want_dx=True)
    mag = np.einsum("sro,sok->srk", ady[:, r_sub], m64[None] + s64[None] * rw)
    err = np.abs(out["dx"].cpu().numpy()[:, r_sub].astype(np.float64) - xb[4])
    assert np.all(err <= 1e-5 * mag), f"dx: worst {np.max(err / mag):.2e}"


def test_random_layer_shapes_agree_with_and_without_a_workspace(hot):
    """Two launch shapes of the same computation on seeded random layer sizes (hundreds to twenty thousand rows,
    few to many tiles, with and without biases and per-sample inputs, whole and partial workspaces): the call
    with a workspace against the call without one, every output, to the rounding of a different order of
    summation.  Each shape is checked against the oracle elsewhere; this comparison is cheap enough to reach
    sizes and tile counts that the oracle cannot, and it is the one that exposed the stale accumulator read
    which mfma_results_settle now rules out."""
    rs = np.random.default_rng(7)
    done = 0
    while done < 24:
        rows = int(rs.choice([rs.integers(256, 1200), rs.integers(1200, 6000), rs.integers(6000, 20000)]))
        k = 4 * int(rs.choice([rs.integers(1, 20), rs.integers(20, 160)]))
        o = int(rs.choice([rs.integers(1, 40), rs.integers(40, 900), rs.integers(900, 2600)]))
        s = int(rs.integers(1, 4))
        bias, xs = bool(rs.integers(0, 2)), bool(rs.integers(0, 2))
        frac = float(rs.choice([1.0, 1.0, 0.5, 0.2]))
        if rows * k * o * s > 3e9:
            continue
        done += 1
        print("case", done, rows, k, o, s, bias, xs, frac, flush=True)
        g = torch.Generator(device=DEV).manual_seed(done)
        x = torch.randn((s, rows, k) if xs else (rows, k), device=DEV, generator=g)
        mu = torch.randn(o, k, device=DEV, generator=g) * 0.05
        sg = torch.rand(o, k, device=DEV, generator=g) * 0.01 + 0.001
        mb = torch.randn(o, device=DEV, generator=g) if bias else None
        sb = (torch.rand(o, device=DEV, generator=g) * 0.01 + 0.001) if bias else None
        dy = torch.randn(s, rows, o, device=DEV, generator=g)
        n_ws = max(int(hot.hot_linear_backward_workspace_bytes(rows, k, o, s) * frac) // 16 * 4, 4)
        outs = []
        for ws in (None, torch.full((n_ws + 16,), float("nan"), device=DEV)):
            t = [torch.full((o, k), float("nan"), device=DEV), torch.full((o, k), float("nan"), device=DEV),
                 torch.full((o,), float("nan"), device=DEV) if bias else None,
                 torch.full((o,), float("nan"), device=DEV) if bias else None, torch.full((s, rows, k), float("nan"), device=DEV)]
            hot.hot_linear_backward_rng(hot.hot_rng(seed=5, step=done, first_sample=0), x, dy, mu, sg, mb, sb, *t, 2 * s, 4500.0,
                                        hot.HOT_REDUCE_SUM, 0, o * k, workspace=None if ws is None else ws[:n_ws])
            torch.cuda.synchronize()
            if ws is not None:
                assert bool(torch.isnan(ws[n_ws:]).all()), "written beyond the workspace"
            outs.append([v for v in t if v is not None])
        for a, b in zip(*outs):
            assert bool(torch.isfinite(a).all()) and bool(torch.isfinite(b).all())
            # a sum of R (or O) products of unit-scale factors: its fp32 rounding is far below 1e-4 of the largest sum
            assert (a - b).abs().max().item() <= 1e-4 * max(a.abs().max().item(), 1e-6)


def test_random_few_row_layers_in_one_pass_agree_with_the_separate_kernels(hot):
    """The kernels that take both gradients in one pass (a workspace given) against the two separate kernels (none
    given) on seeded random layers of 1 to 128 rows: every output, to the rounding of another order of summation
    and of the single-precision finish.  Reaches tile and strip counts beyond the oracle-checked cases."""
    rs = np.random.default_rng(23)
    done, in_one_pass, codes = 0, 0, set()
    while done < 48:
        rows = int(rs.choice([rs.integers(1, 33), rs.integers(33, 129)]))
        k = 4 * int(rs.choice([rs.integers(1, 40), rs.integers(40, 700), rs.integers(3200, 3400)]))
        o = int(rs.choice([rs.integers(1, 130), rs.integers(130, 3000), rs.integers(1000, 3000)]))
        s = int(rs.choice([1, 2, 2, 3, 4, 6, 8] if rows <= 32 else [1, 2, 2, 3]))
        bias, xs = bool(rs.integers(0, 2)), bool(rs.integers(0, 2))
        frac = float(rs.choice([1.0, 1.0, 0.6, 0.3]))
        if k * o > 6e6:
            continue
        code = hot.hot_linear_launch_shape(rows, k, o, s, 2, per_sample_x=xs)
        if code == 0 and rs.random() < 0.8:      # (mostly shapes that the kernels under test take)
            continue
        done += 1
        print("case", done, rows, k, o, s, bias, xs, frac, code, flush=True)
        g = torch.Generator(device=DEV).manual_seed(100 + done)
        x = torch.randn((s, rows, k) if xs else (rows, k), device=DEV, generator=g)
        mu = torch.randn(o, k, device=DEV, generator=g) * 0.05
        sg = torch.rand(o, k, device=DEV, generator=g) * 0.01 + 0.001
        mb = torch.randn(o, device=DEV, generator=g) if bias else None
        sb = (torch.rand(o, device=DEV, generator=g) * 0.01 + 0.001) if bias else None
        dy = torch.randn(s, rows, o, device=DEV, generator=g)
        want = hot.hot_linear_backward_workspace_bytes(rows, k, o, s)
        n_ws = max(int(want * frac) // 16 * 4, 4)
        outs = []
        for ws in (None, torch.full((n_ws + 16,), float("nan"), device=DEV)):
            t = [torch.full((o, k), float("nan"), device=DEV), torch.full((o, k), float("nan"), device=DEV),
                 torch.full((o,), float("nan"), device=DEV) if bias else None,
                 torch.full((o,), float("nan"), device=DEV) if bias else None, torch.full((s, rows, k), float("nan"), device=DEV)]
            hot.hot_linear_backward_rng(hot.hot_rng(seed=9, step=done, first_sample=1), x, dy, mu, sg, mb, sb, *t, 2 * s, 4500.0,
                                        hot.HOT_REDUCE_MEAN, 8, 8 + o * k, workspace=None if ws is None else ws[:n_ws])
            torch.cuda.synchronize()
            if ws is not None:
                assert bool(torch.isnan(ws[n_ws:]).all()), "written beyond the workspace"
                if want > 0 and not bool(torch.isnan(ws[:n_ws]).all()):
                    in_one_pass += 1
                    codes.add(code)
            outs.append([v for v in t if v is not None])
        for a, b in zip(*outs):
            assert bool(torch.isfinite(a).all()) and bool(torch.isfinite(b).all())
            assert (a - b).abs().max().item() <= 1e-4 * max(a.abs().max().item(), 1e-6)
    assert in_one_pass >= 20 and len(codes) >= 6, (in_one_pass, codes)      # (counted where the workspace was written)


def test_random_layer_shapes_forward_and_dx_against_materialised_weights(hot):
    """Seeded random layer sizes beyond the oracle's reach (one to twenty thousand rows, every kernel of the
    forward and input-gradient dispatch): y and dx of the fused calls against fp64 products on the GPU with
    the weights that hot_forward_rng materialises for the same hot_rng (that call is compared with the
    oracle in test_parity_rng_gpu.py), within 1e-5 of the sum of the magnitudes of the addends."""
    rs = np.random.default_rng(11)
    done = 0
    while done < 24:
        rows = int(rs.choice([rs.integers(1, 70), rs.integers(70, 1200), rs.integers(1200, 20000)]))
        k = 4 * int(rs.choice([rs.integers(1, 20), rs.integers(20, 160)]))
        o = int(rs.choice([rs.integers(1, 40), rs.integers(40, 900), rs.integers(900, 2600)]))
        s = int(rs.integers(1, 4))
        bias, xs = bool(rs.integers(0, 2)), bool(rs.integers(0, 2))
        if rows * k * o * s > 3e9:
            continue
        done += 1
        print("case", done, rows, k, o, s, bias, xs, flush=True)
        g = torch.Generator(device=DEV).manual_seed(100 + done)
        x = torch.randn((s, rows, k) if xs else (rows, k), device=DEV, generator=g)
        n_w = o * k
        b_off = n_w + 8
        n = b_off + ((o + 3) // 4) * 4
        mu = torch.randn(n, device=DEV, generator=g) * 0.1
        sigma = torch.rand(n, device=DEV, generator=g) * 0.05 + 0.01
        rng = hot.hot_rng(seed=17, step=done, first_sample=0)
        plan = hot.hot_create(n, n, s, s, 1.0, 0)
        w = torch.empty(s, n, device=DEV)
        hot.hot_forward_rng(plan, rng, mu, sigma, w)
        hot.hot_destroy(plan)
        mu_w, sg_w = mu[:n_w].view(o, k), sigma[:n_w].view(o, k)
        mu_b, sg_b = (mu[b_off:b_off + o], sigma[b_off:b_off + o]) if bias else (None, None)
        y = torch.full((s, rows, o), float("nan"), device=DEV)
        hot.hot_linear_forward_rng(rng, x, mu_w, sg_w, mu_b, sg_b, y, 0, b_off)
        dy = torch.randn(s, rows, o, device=DEV, generator=g)
        dx = torch.full((s, rows, k), float("nan"), device=DEV)
        gw = [torch.empty(o, k, device=DEV), torch.empty(o, k, device=DEV)]
        gb = [torch.empty(o, device=DEV), torch.empty(o, device=DEV)] if bias else [None, None]
        hot.hot_linear_backward_rng(rng, x, dy, mu_w, sg_w, mu_b, sg_b, gw[0], gw[1], gb[0], gb[1], dx, s, 100.0,
                                    hot.HOT_REDUCE_SUM, 0, b_off)
        torch.cuda.synchronize()
        w3 = w[:, :n_w].view(s, o, k).double()
        x3 = (x if xs else x.unsqueeze(0).expand(s, rows, k)).double()
        want_y = torch.matmul(x3, w3.transpose(1, 2))
        A_y = torch.matmul(x3.abs(), w3.abs().transpose(1, 2))
        if bias:
            want_y = want_y + w[:, b_off:b_off + o].double().unsqueeze(1)
            A_y = A_y + w[:, b_off:b_off + o].double().abs().unsqueeze(1)
        assert bool(torch.isfinite(y).all()) and bool(((y.double() - want_y).abs() <= 1e-5 * A_y + 1e-30).all()), "y"
        want_dx = torch.matmul(dy.double(), w3)
        A_dx = torch.matmul(dy.double().abs(), w3.abs())
        assert bool(torch.isfinite(dx).all()) and bool(((dx.double() - want_dx).abs() <= 1e-5 * A_dx + 1e-30).all()), "dx"
        # weight gradients, mu part: g * sum_s dy_s^T x_s + k_kl mu  (g = 1/S, k_kl = 1/|D| here)
        G = torch.matmul(dy.double().transpose(1, 2), x3)
        A_g = torch.matmul(dy.double().abs().transpose(1, 2), x3.abs()).sum(0) / s + mu_w.double().abs() / 100.0
        want_g = G.sum(0) / s + mu_w.double() / 100.0
        assert bool(((gw[0].double() - want_g).abs() <= 1e-5 * A_g + 1e-30).all()), "grad_mu_w"


def test_random_layers_on_the_256_to_1024_row_kernel_against_materialised_weights(hot):
    """Seeded random layer sizes that the forward call or the input gradients give to the 256/512/1024-row kernel
    (hot_linear_launch_shape says so; sizes that neither does are skipped): y and dx against fp64 products on the GPU with the
    weights that hot_forward_rng materialises, as in the test above.  Every launch shape has to come up."""
    rs = np.random.default_rng(23)
    done, seen = 0, set()
    for _ in range(50000):
        if done == 32:
            break
        rows = int(rs.choice([rs.integers(256, 1200), rs.integers(1200, 9000)]))
        k = 4 * int(rs.choice([rs.integers(1, 24), rs.integers(24, 400)]))
        o = int(rs.choice([rs.integers(100, 1200), rs.integers(1200, 9000)]))
        if rs.integers(0, 3) == 0:
            o = 4 * (o // 4 + 1)                      # rows of dy readable in quads: the input gradients may take the kernel too
        s = int(rs.integers(1, 5))
        bias, xs = bool(rs.integers(0, 2)), bool(rs.integers(0, 2))
        if rows * o * s > 1.2e8 or rows * k * o * s > 2e10:
            continue
        f = hot.hot_linear_launch_shape(rows, k, o, s, 0, per_sample_x=xs)
        d = hot.hot_linear_launch_shape(rows, k, o, s, 1, per_sample_x=xs)
        # what the case would add: ("two", pair shape), ("last", outputs / 32 of an odd last sample's launch), ("one", single
        # shape of the forward call), ("dx", shape of the input gradients)
        pair = f % 1000 in (412, 812, 822)
        new = {("two", f % 1000), ("last", f // 1000)} if pair else {("one", f)}
        new = {c for c in new | {("dx", d)} if c[1] != 0} - seen
        if (f == 0 and d == 0) or (done >= 12 and not new):       # (after a dozen cases only shapes not yet seen)
            continue
        seen |= new
        done += 1
        print("case", done, rows, k, o, s, bias, xs, "shapes", f, d, flush=True)
        g = torch.Generator(device=DEV).manual_seed(500 + done)
        x = torch.randn((s, rows, k) if xs else (rows, k), device=DEV, generator=g)
        n_w = o * k
        b_off = n_w + 8
        n = b_off + ((o + 3) // 4) * 4
        mu = torch.randn(n, device=DEV, generator=g) * 0.1
        sigma = torch.rand(n, device=DEV, generator=g) * 0.05 + 0.01
        rng = hot.hot_rng(seed=29, step=done, first_sample=5)
        plan = hot.hot_create(n, n, s, s, 1.0, 0)
        w = torch.empty(s, n, device=DEV)
        hot.hot_forward_rng(plan, rng, mu, sigma, w)
        hot.hot_destroy(plan)
        mu_w, sg_w = mu[:n_w].view(o, k), sigma[:n_w].view(o, k)
        mu_b, sg_b = (mu[b_off:b_off + o], sigma[b_off:b_off + o]) if bias else (None, None)
        y = torch.full((s, rows, o), float("nan"), device=DEV)
        hot.hot_linear_forward_rng(rng, x, mu_w, sg_w, mu_b, sg_b, y, 0, b_off)
        dy = torch.randn(s, rows, o, device=DEV, generator=g)
        dx = torch.full((s, rows, k), float("nan"), device=DEV)
        gw = [torch.empty(o, k, device=DEV), torch.empty(o, k, device=DEV)]
        gb = [torch.empty(o, device=DEV), torch.empty(o, device=DEV)] if bias else [None, None]
        hot.hot_linear_backward_rng(rng, x, dy, mu_w, sg_w, mu_b, sg_b, gw[0], gw[1], gb[0], gb[1], dx, s, 100.0,
                                    hot.HOT_REDUCE_SUM, 0, b_off)
        torch.cuda.synchronize()
        for si in range(s):                              # one sample at a time: the fp64 products are large
            w2 = w[si, :n_w].view(o, k).double()
            x2 = (x[si] if xs else x).double()
            want_y, A_y = x2 @ w2.T, x2.abs() @ w2.abs().T
            if bias:
                want_y = want_y + w[si, b_off:b_off + o].double()
                A_y = A_y + w[si, b_off:b_off + o].double().abs()
            assert bool(torch.isfinite(y[si]).all()) and bool(((y[si].double() - want_y).abs() <= 1e-5 * A_y + 1e-30).all()), "y"
            del want_y, A_y
            d2 = dy[si].double()
            want_dx, A_dx = d2 @ w2, d2.abs() @ w2.abs()
            assert bool(torch.isfinite(dx[si]).all()) and bool(((dx[si].double() - want_dx).abs() <= 1e-5 * A_dx + 1e-30).all()), "dx"
            del want_dx, A_dx, d2, w2, x2
        del x, w, y, dy, dx, gw
        torch.cuda.empty_cache()
    # forward: pairs on 32 and 64 outputs, single samples on 32 to 128 and in the 1024-row shape, an odd last sample; input gradients
    assert {("two", 412), ("two", 812), ("two", 822), ("one", 411), ("one", 421), ("one", 811), ("one", 821), ("one", 841),
            ("one", 1621)} <= seen, sorted(seen)
    assert {("dx", 411), ("dx", 421), ("dx", 811), ("dx", 821), ("dx", 841), ("dx", 1621)} <= seen, sorted(seen)
    assert any(c[0] == "last" for c in seen), sorted(seen)


# (rows, in, out, samples, per-sample x, bias)
TILED = [(300, 2900, 4228, 2, False, True),      # 23 x 34 tiles of 128 x 128, ragged in rows, inputs and outputs
         (272, 2048, 4096, 3, True, False),      # 16 x 32 whole tiles, three samples with inputs of their own
         (257, 3000, 4092, 1, False, True),      # 24 x 32 tiles, both edges ragged, a single sample, an odd number of steps
         (1030, 2048, 2000, 2, False, True),     # one tile per compute unit, from a thousand rows on
         (150, 2048, 4096, 2, False, True),      # fewer rows than one 256-row block (the kernel runs from 129 rows on)
         (260, 1500, 2048, 2, False, True),      # 12 x 16 = 192 tiles: fewer than a round of 512 (the kernel takes these from 256 rows on)
         (300, 2160, 8640, 2, False, False)]     # 17 x 68 = 1156 tiles: a last round of 512 that is a quarter full


@pytest.mark.parametrize("rows,k,o,s,xs,bias", TILED)
def test_large_layer_weight_gradients_on_sampled_outputs(oracle, hot, rows, k, o, s, xs, bias):
    """Layers large enough for the weight-gradient kernel with tiles of 128 x 128 (at least two tiles per compute
    unit), against the oracle on the outputs it can afford: the weight gradients of 40 outputs (all rows, all
    inputs; the first and last output of the first, second and last tile among them) and their bias gradients.
    Outputs do not depend on one another, so the block is the oracle's result for the sub-layer it spans."""
    print("case linear backward, large layer", rows, k, o, s, xs, bias, flush=True)
    c = _layer(7 * rows + k + o, rows, k, o)
    g = np.random.default_rng(rows + o)
    if xs:
        c["x"] = g.normal(size=(s, rows, k)).astype(np.float32)
    dy = (g.normal(size=(s, rows, o)) * 10 ** g.uniform(-2, 1, size=(s, 1, o))).astype(np.float32)
    rng = hot.hot_rng(seed=31, step=2, first_sample=3)
    w_off, b_off = 128, 128 + o * k
    s_total, dsize = 2 * s, 45000.0
    t = {n: torch.from_numpy(c[n]).to(DEV) for n in ("x", "mu_w", "sigma_w", "mu_b", "sigma_b")}
    out = {"gmw": torch.full((o, k), float("nan"), device=DEV), "gsw": torch.full((o, k), float("nan"), device=DEV),
           "gmb": torch.full((o,), float("nan"), device=DEV), "gsb": torch.full((o,), float("nan"), device=DEV)}
    hot.hot_linear_backward_rng(rng, t["x"], torch.from_numpy(dy).to(DEV), t["mu_w"], t["sigma_w"],
                                t["mu_b"] if bias else None, t["sigma_b"] if bias else None, out["gmw"], out["gsw"],
                                out["gmb"] if bias else None, out["gsb"] if bias else None, None,
                                s_total, dsize, hot.HOT_REDUCE_SUM, w_off, b_off)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out["gmw"]).all()) and bool(torch.isfinite(out["gsw"]).all())
    ew, rw = oracle.eps_normal(o * k, s, rng.seed, rng.step, rng.first_sample, with_radius=True, col0=w_off)
    ew, rw = ew.reshape(s, o, k), rw.reshape(s, o, k)
    eb, rb = oracle.eps_normal(o, s, rng.seed, rng.step, rng.first_sample, with_radius=True, col0=b_off)
    last = (o - 1) // 128 * 128
    o_sub = np.unique(np.concatenate([[0, 31, 32, 63, 64, 127, 128, 255, last, o - 1], g.choice(o, 30, replace=False)]))
    gg, kk = 1.0 / s_total, s / (s_total * dsize)
    sub_b = (c["mu_b"][o_sub], c["sigma_b"][o_sub], np.ascontiguousarray(eb[:, o_sub])) if bias else (None, None, None)
    want = oracle.linear_backward(c["x"], np.ascontiguousarray(dy[:, :, o_sub]), c["mu_w"][o_sub], c["sigma_w"][o_sub],
                                  np.ascontiguousarray(ew[:, o_sub]), *sub_b, g=gg, k=kk, want_dx=False)
    ax, ady = np.abs(c["x"].astype(np.float64)), np.abs(dy[:, :, o_sub].astype(np.float64))
    Gabs = np.matmul(ady.transpose(0, 2, 1), ax)                                                 # [S, |o_sub|, K]
    m64, s64 = np.abs(c["mu_w"][o_sub].astype(np.float64)), c["sigma_w"][o_sub].astype(np.float64)
    checks = [("gmw", want[0], gg * Gabs.sum(0) + kk * m64), ("gsw", want[1], gg * (Gabs * rw[:, o_sub]).sum(0) + kk * (s64 + 1 / s64))]
    if bias:
        Gb = ady.sum(1)
        mb, sb = np.abs(c["mu_b"][o_sub].astype(np.float64)), c["sigma_b"][o_sub].astype(np.float64)
        checks += [("gmb", want[2], gg * Gb.sum(0) + kk * mb), ("gsb", want[3], gg * (Gb * rb[:, o_sub]).sum(0) + kk * (sb + 1 / sb))]
    else:
        assert np.isnan(out["gmb"].cpu().numpy()).all() and np.isnan(out["gsb"].cpu().numpy()).all()
    for name, w64, mag in checks:
        err = np.abs(out[name].cpu().numpy()[o_sub].astype(np.float64) - w64)
        assert np.all(err <= 1e-5 * mag), f"{name}: worst {np.max(err / mag):.2e}"
        print("  %s worst error / magnitude sum: %.2e" % (name, np.max(err / mag)), flush=True)
