"""GPU parity of the Adam step and of the weight-space MC-dropout layer against the fp64 oracle.

Adam (fp32 arithmetic on fp32 state, a handful of roundings per quantity), relative to the sum of
addend magnitudes:  m: 1e-6 (beta1 |m| + (1-beta1) |g|),  v: 1e-6 (beta2 v + (1-beta2) g^2),
theta: 1e-6 (|theta| + |step taken|).  Dropout: the mask is an integer comparison and must agree
bit for bit; kept weights are mu * fp32(1/keep): 1e-6 |mu| / keep; gradients 1e-6 g sum|G| / keep."""
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


def _dev(a, offset=0):
    buf = torch.empty(a.size + offset, device=DEV)
    v = buf[offset:].view(a.shape)
    v.copy_(torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)))
    return v


@pytest.mark.parametrize("n,offset", [(1, 0), (5, 0), (1023, 0), (4096, 0), (100_003, 0), (100_003, 1), (1_048_579, 3)])
def test_adam_steps_match_oracle(oracle, hot, n, offset):
    print("case adam", n, offset, flush=True)
    r = np.random.default_rng(n)
    state = {"mu": r.normal(size=n), "sigma": r.uniform(0.01, 1.0, size=n), "m_mu": np.zeros(n), "v_mu": np.zeros(n),
             "m_sigma": np.zeros(n), "v_sigma": np.zeros(n)}
    d = {k: _dev(v, offset) for k, v in state.items()}
    lr, b1, b2, eps, gs, smin = 3e-3, 0.9, 0.999, 1e-8, 0.25, 0.02
    for t in range(1, 6):
        g_mu = (r.normal(size=n) * 10 ** r.uniform(-4, 3, size=n)).astype(np.float32)
        g_sg = (r.normal(size=n) * 10 ** r.uniform(-4, 3, size=n)).astype(np.float32)
        if t == 3:
            g_mu[: n // 2] = 0.0
        before = {k: v.cpu().numpy().astype(np.float64) for k, v in d.items()}
        hot.hot_adam_step(hot.hot_adam(lr, b1, b2, eps, gs, smin, t), d["mu"], d["sigma"], _dev(g_mu, offset),
                          _dev(g_sg, offset), d["m_mu"], d["v_mu"], d["m_sigma"], d["v_sigma"])
        torch.cuda.synchronize()
        want = oracle.adam_step(before["mu"], before["sigma"], g_mu, g_sg, before["m_mu"], before["v_mu"],
                                before["m_sigma"], before["v_sigma"], step=t, lr=lr, beta1=b1, beta2=b2, eps=eps,
                                grad_scale=gs, sigma_min=smin)
        got = {k: v.cpu().numpy().astype(np.float64) for k, v in d.items()}
        for name, grad, m_key, v_key, th_key, w_th, w_m, w_v in (("mu", g_mu, "m_mu", "v_mu", "mu", want[0], want[2], want[3]),
                                                                 ("sigma", g_sg, "m_sigma", "v_sigma", "sigma", want[1], want[4], want[5])):
            g = gs * grad.astype(np.float64)
            assert np.all(np.abs(got[m_key] - w_m) <= 1e-6 * (b1 * np.abs(before[m_key]) + (1 - b1) * np.abs(g)) + 1e-45)
            assert np.all(np.abs(got[v_key] - w_v) <= 1e-6 * (b2 * before[v_key] + (1 - b2) * g * g) + 1e-45)
            step = np.abs(w_th - before[th_key])
            assert np.all(np.abs(got[th_key] - w_th) <= 1e-6 * (np.abs(before[th_key]) + step + lr))
        assert got["sigma"].min() >= smin * (1 - 1e-7)


def test_adam_trajectory_matches_torch_adam(hot):
    n, steps, lr = 10_000, 20, 1e-2
    r = np.random.default_rng(0)
    mu0, sg0 = r.normal(size=n).astype(np.float32), r.uniform(0.1, 1, size=n).astype(np.float32)
    d = [_dev(mu0), _dev(sg0)] + [_dev(np.zeros(n)) for _ in range(4)]
    p_mu = torch.tensor(mu0, dtype=torch.float64, requires_grad=True)
    p_sg = torch.tensor(sg0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p_mu, p_sg], lr=lr)
    for t in range(1, steps + 1):
        g_mu, g_sg = r.normal(size=n).astype(np.float32), r.normal(size=n).astype(np.float32)
        p_mu.grad, p_sg.grad = torch.tensor(g_mu, dtype=torch.float64), torch.tensor(g_sg, dtype=torch.float64)
        opt.step()
        hot.hot_adam_step(hot.hot_adam(lr, 0.9, 0.999, 1e-8, 1.0, 0.0, t), d[0], d[1], _dev(g_mu), _dev(g_sg), *d[2:])
    torch.cuda.synchronize()
    assert np.abs(d[0].cpu().numpy() - p_mu.detach().numpy()).max() <= 1e-5 * steps * lr + 1e-6
    assert np.abs(d[1].cpu().numpy() - p_sg.detach().numpy()).max() <= 1e-5 * steps * lr + 1e-6


@pytest.mark.parametrize("n,ld,s,offset,keep", [(300_001, 300_001, 5, 0, 0.5), (70_003, 70_016, 4, 0, 0.9), (4099, 4099, 3, 1, 0.2),
                                                  (2, 2, 2, 0, 1.0), (500_003, 500_003, 3, 0, 1.0), (1_000_000, 1_000_000, 16, 0, 0.75),
                                                  # larger than the 256 MiB memory-side cache (non-temporal accesses), aligned and not
                                                  (16_800_000, 16_800_000, 4, 0, 0.6), (11_200_003, 11_200_003, 6, 3, 0.35)])
def test_dropout_layer_matches_oracle(oracle, hot, n, ld, s, offset, keep):
    print("case dropout", n, ld, s, offset, keep, flush=True)
    r = np.random.default_rng(n + s)
    mu = r.normal(size=n).astype(np.float32)
    G = np.full((s, ld), np.nan, np.float32)
    G[:, :n] = r.normal(size=(s, n)) * 3
    rng = hot.hot_rng(seed=31337, step=2, first_sample=s)
    plan = hot.hot_create(n, ld, s, 2 * s, 1.0, 0)
    mu_d, G_d = _dev(mu, offset), _dev(G, offset)
    w = _dev(np.full((s, ld), 7.0, np.float32), offset)
    gmu = _dev(np.zeros(n), offset)
    hot.hot_forward_dropout_rng(plan, rng, keep, mu_d, w)
    hot.hot_backward_dropout_rng(plan, rng, keep, G_d, gmu)
    torch.cuda.synchronize()
    hot.hot_destroy(plan)
    words = oracle.eps_bits(n, s, rng.seed, rng.step, rng.first_sample)
    w64 = oracle.dropout_forward(mu, words, keep)
    got = w.cpu().numpy()
    if ld > n:
        assert np.all(got[:, n:] == 7.0), "w padding written"
    assert np.array_equal(got[:, :n] == 0, w64 == 0), "mask differs"
    assert np.all(np.abs(got[:, :n] - w64) <= 1e-6 * np.abs(mu)[None, :] / keep)
    gm64 = oracle.dropout_backward(G, words, keep, s_total=2 * s, n=n)
    scale = np.abs(G[:, :n].astype(np.float64)).sum(0) / (2 * s) / keep
    assert np.all(np.abs(gmu.cpu().numpy() - gm64) <= 1e-6 * scale)
    if keep == 1.0:
        assert np.array_equal(got[:, :n], np.broadcast_to(mu, (s, n)))


@pytest.mark.parametrize("o,k,ld_pad,s,offset,keep,unit_off", [(7, 12, 0, 3, 0, 0.5, 0), (128, 96, 4, 4, 0, 0.8, 64), (33, 100, 0, 5, 1, 0.3, 8),
                                                             (2160, 540, 0, 2, 0, 0.9, 4096), (1, 4, 0, 1, 0, 1.0, 0)])
def test_unit_dropout_layer_matches_oracle(oracle, hot, o, k, ld_pad, s, offset, keep, unit_off):
    """One Bernoulli variable per input unit and sample: the oracle's per-weight functions fed with
    the unit words spread over the weight matrix (word of weight (o, k) = word of unit k)."""
    print("case unit dropout", o, k, ld_pad, s, offset, keep, unit_off, flush=True)
    n, ld = o * k, o * k + ld_pad
    r = np.random.default_rng(o + k)
    mu = r.normal(size=n).astype(np.float32)
    G = np.full((s, ld), np.nan, np.float32)
    G[:, :n] = r.normal(size=(s, n)) * 2
    rng = hot.hot_rng(seed=2718, step=3, first_sample=1)
    plan = hot.hot_create(n, ld, s, 3 * s, 1.0, 0)
    mu_d, G_d = _dev(mu, offset), _dev(G, offset)
    w = _dev(np.full((s, ld), 7.0, np.float32), offset)
    gmu = _dev(np.zeros(n), offset)
    hot.hot_forward_dropout_units_rng(plan, rng, keep, k, unit_off, mu_d, w)
    hot.hot_backward_dropout_units_rng(plan, rng, keep, k, unit_off, G_d, gmu)
    torch.cuda.synchronize()
    hot.hot_destroy(plan)
    unit_words = oracle.eps_bits(unit_off + k, s, rng.seed, rng.step, rng.first_sample)[:, unit_off:unit_off + k]   # [S, K]
    words = np.ascontiguousarray(np.tile(unit_words, (1, o)))                                                      # [S, O*K]
    w64 = oracle.dropout_forward(mu, words, keep)
    got = w.cpu().numpy()
    if ld > n:
        assert np.all(got[:, n:] == 7.0), "w padding written"
    assert np.array_equal(got[:, :n] == 0, w64 == 0), "mask differs"
    assert np.all(np.abs(got[:, :n] - w64) <= 1e-6 * np.abs(mu)[None, :] / keep)
    # a dropped unit zeroes its whole column, a kept one none of it
    cols = (got[:, :n].reshape(s, o, k) != 0)
    assert np.all(cols.all(axis=1) | ~cols.any(axis=1))
    gm64 = oracle.dropout_backward(G, words, keep, s_total=3 * s, n=n)
    scale = np.abs(G[:, :n].astype(np.float64)).sum(0) / (3 * s) / keep
    assert np.all(np.abs(gmu.cpu().numpy() - gm64) <= 1e-6 * scale + 1e-30)


def test_update_errors(hot):
    t = torch.zeros(16, device=DEV)
    with pytest.raises(hot.HotError):
        hot.hot_adam_step(hot.hot_adam(1e-3, 0.9, 0.999, 1e-8, 1.0, 0.0, 0), *[t.clone() for _ in range(8)])     # step 0
    with pytest.raises(hot.HotError):
        hot.hot_adam_step(hot.hot_adam(1e-3, 1.0, 0.999, 1e-8, 1.0, 0.0, 1), *[t.clone() for _ in range(8)])     # beta1 = 1
    plan = hot.hot_create(16, 16, 1, 1, 1.0, 0)
    rng = hot.hot_rng(seed=1, step=0, first_sample=0)
    for keep in (0.0, 1.5, float("nan")):
        with pytest.raises(hot.HotError):
            hot.hot_forward_dropout_rng(plan, rng, keep, t, t.clone().view(1, 16))
    hot.hot_destroy(plan)


# (n, ld, samples, pointer offset in floats, eps drawn in the kernel)
FUSED = [(1, 1, 1, 0, False), (5, 8, 2, 0, True), (100_003, 100_003, 3, 0, False), (100_003, 100_004, 4, 1, True),
         (3 * 4096 + 5, 3 * 4096 + 8, 16, 0, True), (1_048_579, 1_048_579, 2, 3, False), (262_144, 262_144, 5, 0, False)]


@pytest.mark.parametrize("n,ld,s,offset,gen", FUSED)
def test_fused_backward_adam(oracle, hot, n, ld, s, offset, gen):
    """hot_backward_adam against (a) hot_backward followed by hot_adam_step, bit for bit, and (b) the
    oracle's gradient (fp64, never rounded) fed to the oracle's Adam step.  For (b) the rounding of
    the gradient to fp32 on the GPU moves an Adam step by about twice the gradient's relative error
    r = 1e-6 A / |grad| (A the sum of the gradient's addend magnitudes): elements with r > 0.05,
    where cancellation leaves the sign of the gradient itself in doubt, are checked to be rare and
    excluded from the theta bound."""
    print("case fused backward+adam", n, ld, s, offset, gen, flush=True)
    r = np.random.default_rng(n * 31 + s)
    D, t, lr, b1, b2, eps_a, gsc, smin = 1000.0, 3, 2e-3, 0.9, 0.999, 1e-8, 0.5, 0.02
    mu = r.normal(size=n).astype(np.float32)
    sigma = r.uniform(0.01, 1.0, size=n).astype(np.float32)
    G = np.full((s, ld), np.nan, np.float32)
    G[:, :n] = r.normal(size=(s, n)) * 10 ** r.uniform(-3, 2, size=(1, n))
    rng = hot.hot_rng(seed=99, step=t, first_sample=0)
    eps64 = oracle.eps_normal(n, s, rng.seed, rng.step, rng.first_sample) if gen else r.normal(size=(s, n))
    eps = np.full((s, ld), np.nan, np.float32)
    eps[:, :n] = eps64
    state = {"m_mu": r.normal(size=n) * 0.1, "v_mu": r.uniform(0, 1, size=n) * 0.01,
             "m_sigma": r.normal(size=n) * 0.1, "v_sigma": r.uniform(0, 1, size=n) * 0.01}
    state = {k: v.astype(np.float32) for k, v in state.items()}
    plan = hot.hot_create(n, ld, s, s, D, 0)
    G_d, eps_d = _dev(G, offset), (None if gen else _dev(eps, offset))
    params = hot.hot_adam(lr, b1, b2, eps_a, gsc, smin, t)

    two = {"mu": _dev(mu, offset), "sigma": _dev(sigma, offset), **{k: _dev(v, offset) for k, v in state.items()}}
    gmu, gsig = _dev(np.zeros(n), offset), _dev(np.zeros(n), offset)
    if gen:
        hot.hot_backward_rng(plan, rng, two["mu"], two["sigma"], G_d, gmu, gsig)
    else:
        hot.hot_backward(plan, two["mu"], two["sigma"], eps_d, G_d, gmu, gsig)
    hot.hot_adam_step(params, two["mu"], two["sigma"], gmu, gsig, two["m_mu"], two["v_mu"], two["m_sigma"], two["v_sigma"])

    one = {"mu": _dev(mu, offset), "sigma": _dev(sigma, offset), **{k: _dev(v, offset) for k, v in state.items()}}
    hot.hot_backward_adam(plan, rng if gen else None, params, one["mu"], one["sigma"], eps_d, G_d,
                          one["m_mu"], one["v_mu"], one["m_sigma"], one["v_sigma"])
    torch.cuda.synchronize()
    hot.hot_destroy(plan)
    for k in one:
        assert torch.equal(one[k], two[k]), f"{k}: fused and two-call results differ"

    eps_in = eps if not gen else eps     # fp32 values either way (the generator's output is fp32)
    gm64, gs64 = oracle.grad(mu, sigma, eps_in, G, s, D)
    want = oracle.adam_step(mu, sigma, gm64, gs64, state["m_mu"], state["v_mu"], state["m_sigma"], state["v_sigma"],
                            step=t, lr=lr, beta1=b1, beta2=b2, eps=eps_a, grad_scale=gsc, sigma_min=smin)
    got = {k: v.cpu().numpy().astype(np.float64) for k, v in one.items()}
    g_abs = np.abs(G[:, :n].astype(np.float64))
    k_kl = 1.0 / D
    A = {"mu": g_abs.sum(0) / s + k_kl * np.abs(mu), "sigma": (g_abs * np.abs(eps[:, :n])).sum(0) / s + k_kl * (sigma + 1.0 / sigma)}
    for name, g64, w_th, w_m, w_v, m_key, v_key, th0 in (("mu", gm64, want[0], want[2], want[3], "m_mu", "v_mu", mu),
                                                        ("sigma", gs64, want[1], want[4], want[5], "m_sigma", "v_sigma", sigma)):
        a = gsc * A[name]
        assert np.all(np.abs(got[m_key] - w_m) <= 1e-6 * (b1 * np.abs(state[m_key]) + (1 - b1) * a) + 1e-45), name
        assert np.all(np.abs(got[v_key] - w_v) <= 3e-6 * (b2 * state[v_key] + (1 - b2) * a * a) + 1e-45), name
        rel = 1e-6 * A[name] / np.maximum(np.abs(g64), 1e-300)
        sure = rel <= 0.05
        assert sure.mean() >= 0.999 or n < 1000
        step = np.abs(w_th - th0)
        bound = 1e-6 * (np.abs(th0) + step + lr) + 2.0 * rel * (step + lr)
        assert np.all((np.abs(got[name] - w_th) <= bound)[sure]), name
    assert got["sigma"].min() >= smin * (1 - 1e-7)


@pytest.mark.parametrize("n,ld,s,offset,gen,want_kl", [(1, 1, 1, 0, False, True), (5, 8, 2, 0, True, True), (100_003, 100_003, 3, 0, False, True),
                                                       (100_003, 100_004, 4, 1, True, False), (3 * 4096 + 5, 3 * 4096 + 8, 16, 0, True, True),
                                                       (1_048_579, 1_048_579, 2, 3, False, True), (300_000, 300_000, 2, 0, True, True)])
def test_fused_adam_forward(oracle, hot, n, ld, s, offset, gen, want_kl):
    """hot_adam_forward against hot_adam_step followed by hot_forward / hot_forward_rng, bit for bit
    (parameters, moments, w, KL), and against the oracle: Adam step in fp64, then w and KL from the
    GPU's updated fp32 parameters."""
    print("case fused adam+forward", n, ld, s, offset, gen, want_kl, flush=True)
    r = np.random.default_rng(n * 7 + s)
    t_step, lr, b1, b2, eps_a, gsc, smin = 4, 3e-3, 0.9, 0.999, 1e-8, 0.5, 0.02
    st = {"mu": r.normal(size=n), "sigma": r.uniform(0.01, 1.0, size=n), "m_mu": r.normal(size=n) * 0.1,
          "v_mu": r.uniform(0, 1, size=n) * 0.01, "m_sigma": r.normal(size=n) * 0.1, "v_sigma": r.uniform(0, 1, size=n) * 0.01}
    st = {k: v.astype(np.float32) for k, v in st.items()}
    g_mu = (r.normal(size=n) * 10 ** r.uniform(-3, 2, size=n)).astype(np.float32)
    g_sg = (r.normal(size=n) * 10 ** r.uniform(-3, 2, size=n)).astype(np.float32)
    eps = np.full((s, ld), np.nan, np.float32)
    eps[:, :n] = r.normal(size=(s, n))
    rng = hot.hot_rng(seed=5, step=t_step + 1, first_sample=0)
    params = hot.hot_adam(lr, b1, b2, eps_a, gsc, smin, t_step)
    plan = hot.hot_create(n, ld, s, 4 * s, 100.0, 0)
    gmu_d, gsg_d = _dev(g_mu, offset), _dev(g_sg, offset)
    eps_d = None if gen else _dev(eps, offset)
    names = ("mu", "sigma", "m_mu", "v_mu", "m_sigma", "v_sigma")

    two = {k: _dev(st[k], offset) for k in names}
    w2 = _dev(np.full((s, ld), 7.0, np.float32), offset)
    kl2 = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    hot.hot_adam_step(params, two["mu"], two["sigma"], gmu_d, gsg_d, two["m_mu"], two["v_mu"], two["m_sigma"], two["v_sigma"])
    if gen:
        hot.hot_forward_rng(plan, rng, two["mu"], two["sigma"], w2, kl2 if want_kl else None)
    else:
        hot.hot_forward(plan, two["mu"], two["sigma"], eps_d, w2, kl2 if want_kl else None)

    one = {k: _dev(st[k], offset) for k in names}
    w1 = _dev(np.full((s, ld), 7.0, np.float32), offset)
    kl1 = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    hot.hot_adam_forward(plan, rng if gen else None, params, one["mu"], one["sigma"], gmu_d, gsg_d, one["m_mu"], one["v_mu"],
                         one["m_sigma"], one["v_sigma"], eps_d, w1, kl1 if want_kl else None)
    torch.cuda.synchronize()
    hot.hot_destroy(plan)
    for k in names:
        assert torch.equal(one[k], two[k]), f"{k}: fused and two-call results differ"
    assert torch.equal(w1, w2) and kl1.item() == kl2.item()
    if ld > n:
        assert torch.all(w1[:, n:] == 7.0), "w padding written"

    want = oracle.adam_step(st["mu"], st["sigma"], g_mu, g_sg, st["m_mu"], st["v_mu"], st["m_sigma"], st["v_sigma"],
                            step=t_step, lr=lr, beta1=b1, beta2=b2, eps=eps_a, grad_scale=gsc, sigma_min=smin)
    got_mu, got_sg = one["mu"].cpu().numpy(), one["sigma"].cpu().numpy()
    for got, w_th, th0 in ((got_mu, want[0], st["mu"]), (got_sg, want[1], st["sigma"])):
        assert np.all(np.abs(got - w_th) <= 1e-6 * (np.abs(th0) + np.abs(w_th - th0) + lr))
    e_used = oracle.eps_normal(n, s, rng.seed, rng.step, rng.first_sample).astype(np.float32) if gen else eps[:, :n]
    w64 = oracle.reparam(got_mu, got_sg, np.ascontiguousarray(e_used))
    tol = 1e-5 * np.abs(w64) + (4e-6 * got_sg[None, :].astype(np.float64) * 6.0 if gen else 0.0)
    assert np.all(np.abs(w1.cpu().numpy()[:, :n] - w64) <= tol)
    if want_kl:
        m64, s64 = got_mu.astype(np.float64), got_sg.astype(np.float64)
        scale = 0.5 * float(np.sum(s64 * s64 + m64 * m64 + 1.0 + np.abs(2.0 * np.log(s64))))
        assert abs(kl1.item() - oracle.kl(got_mu, got_sg)) <= 1e-5 * scale


@pytest.mark.parametrize("n,ld,s,offset,want_kl,launch", [
    (1, 1, 1, 0, True, {}), (5, 8, 2, 0, True, {}), (100_003, 100_004, 3, 1, True, {}), (3 * 4096 + 5, 3 * 4096 + 8, 16, 0, False, {}),
    (1_048_579, 1_048_579, 2, 3, True, {}), (300_000, 300_000, 2, 0, True, dict(chunks=1, unroll=1, grid_blocks=7)),
    (2_000_000, 2_000_000, 5, 0, True, dict(chunks=2, unroll=4, nontemporal=1))])
def test_fused_backward_adam_forward(oracle, hot, n, ld, s, offset, want_kl, launch):
    """The whole step of Algorithm 1 behind the network's backward pass, hot_backward_adam_forward, against
    hot_backward_adam followed by hot_forward_rng with the next step's draw: parameters, moments and w bit
    for bit; KL bit for bit when both kernels run with one launch shape on more than 64 workgroups (the
    forward kernel then leaves the sum of the partials to the same finish kernel), else to the rounding of the
    fp64 sum.  (Each of the two calls is checked against the oracle in its own test; here w and KL are checked
    against the oracle once more, from the updated parameters.)"""
    print("case fused backward+adam+forward", n, ld, s, offset, want_kl, launch, flush=True)
    r = np.random.default_rng(n * 13 + s)
    D, t, lr, b1, b2, eps_a, gsc, smin = 500.0, 6, 2e-3, 0.9, 0.999, 1e-8, 1.0, 0.02
    st = {"mu": r.normal(size=n), "sigma": r.uniform(0.01, 1.0, size=n), "m_mu": r.normal(size=n) * 0.1,
          "v_mu": r.uniform(0, 1, size=n) * 0.01, "m_sigma": r.normal(size=n) * 0.1, "v_sigma": r.uniform(0, 1, size=n) * 0.01}
    st = {k: v.astype(np.float32) for k, v in st.items()}
    G = np.full((s, ld), np.nan, np.float32)
    G[:, :n] = r.normal(size=(s, n)) * 10 ** r.uniform(-3, 2, size=(1, n))
    rng, rng_next = hot.hot_rng(seed=77, step=t, first_sample=0), hot.hot_rng(seed=77, step=t + 1, first_sample=0)
    params = hot.hot_adam(lr, b1, b2, eps_a, gsc, smin, t)
    plan = hot.hot_create(n, ld, s, s, D, 0)
    same_shape = bool(launch)
    if launch:
        for kern in (hot.HOT_KERNEL_BACKWARD_RNG, hot.HOT_KERNEL_FORWARD_RNG):
            hot.hot_set_launch(plan, kern, **launch)
    else:
        fr, br = hot.hot_get_launch(plan, hot.HOT_KERNEL_FORWARD_RNG), hot.hot_get_launch(plan, hot.HOT_KERNEL_BACKWARD_RNG)
        same_shape = fr["chunks"] == br["chunks"] and fr["grid_blocks"] == br["grid_blocks"]
    G_d = _dev(G, offset)
    names = ("mu", "sigma", "m_mu", "v_mu", "m_sigma", "v_sigma")

    two = {k: _dev(st[k], offset) for k in names}
    w2 = _dev(np.full((s, ld), 7.0, np.float32), offset)
    kl2 = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    hot.hot_backward_adam(plan, rng, params, two["mu"], two["sigma"], None, G_d, two["m_mu"], two["v_mu"], two["m_sigma"], two["v_sigma"])
    hot.hot_forward_rng(plan, rng_next, two["mu"], two["sigma"], w2, kl2 if want_kl else None)

    one = {k: _dev(st[k], offset) for k in names}
    w1 = _dev(np.full((s, ld), 7.0, np.float32), offset)
    kl1 = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    hot.hot_backward_adam_forward(plan, rng, rng_next, params, one["mu"], one["sigma"], G_d, one["m_mu"], one["v_mu"],
                                  one["m_sigma"], one["v_sigma"], w1, kl1 if want_kl else None)
    torch.cuda.synchronize()
    hot.hot_destroy(plan)
    for k in names:
        assert torch.equal(one[k], two[k]), f"{k}: fused and two-call results differ"
    assert torch.equal(w1, w2)
    if ld > n:
        assert torch.all(w1[:, n:] == 7.0), "w padding written"
    got_mu, got_sg = one["mu"].cpu().numpy(), one["sigma"].cpu().numpy()
    if want_kl:
        m64, s64 = got_mu.astype(np.float64), got_sg.astype(np.float64)
        scale = 0.5 * float(np.sum(s64 * s64 + m64 * m64 + 1.0 + np.abs(2.0 * np.log(s64))))
        grid = min(-(-n // (1024 * (launch.get("chunks", 4) if launch else 4))), launch.get("grid_blocks", 65536) if launch else 65536)
        if same_shape and grid > 64:        # up to 64 workgroups the forward kernel adds the partials itself, in another order
            assert kl1.item() == kl2.item()
        assert abs(kl1.item() - kl2.item()) <= 1e-13 * scale
        assert abs(kl1.item() - oracle.kl(got_mu, got_sg)) <= 1e-5 * scale
    else:
        assert kl1.item() == -1.0
    e_next = oracle.eps_normal(n, s, rng_next.seed, rng_next.step, rng_next.first_sample).astype(np.float32)
    w64 = oracle.reparam(got_mu, got_sg, np.ascontiguousarray(e_next))
    assert np.all(np.abs(w1.cpu().numpy()[:, :n] - w64) <= 1e-5 * np.abs(w64) + 4e-6 * got_sg[None, :].astype(np.float64) * 6.0)


@pytest.mark.parametrize("n,ld,s,offset", [(700_001, 700_004, 3, 0), (700_001, 700_001, 2, 1)])
def test_fused_calls_with_non_temporal_accesses(hot, n, ld, s, offset):
    """The three fused calls with the non-temporal variants of their kernels (the default only above
    256 MiB) against the unfused calls with the same launch shape, bit for bit.  The unfused kernels'
    non-temporal variants are compared with the oracle in test_parity_gpu.py."""
    print("case fused calls, non-temporal", n, ld, s, offset, flush=True)
    r = np.random.default_rng(n + s)
    st = {"mu": r.normal(size=n), "sigma": r.uniform(0.01, 1.0, size=n), "m_mu": r.normal(size=n) * 0.1,
          "v_mu": r.uniform(0, 1, size=n) * 0.01, "m_sigma": r.normal(size=n) * 0.1, "v_sigma": r.uniform(0, 1, size=n) * 0.01}
    st = {k: v.astype(np.float32) for k, v in st.items()}
    names = ("mu", "sigma", "m_mu", "v_mu", "m_sigma", "v_sigma")
    G = np.full((s, ld), np.nan, np.float32)
    G[:, :n] = r.normal(size=(s, n))
    eps = np.full((s, ld), np.nan, np.float32)
    eps[:, :n] = r.normal(size=(s, n))
    G_d, eps_d = _dev(G, offset), _dev(eps, offset)
    gmu_in, gsg_in = _dev(r.normal(size=n).astype(np.float32), offset), _dev(r.normal(size=n).astype(np.float32), offset)
    rng, nxt = hot.hot_rng(seed=3, step=8, first_sample=0), hot.hot_rng(seed=3, step=9, first_sample=0)
    params = hot.hot_adam(1e-3, 0.9, 0.999, 1e-8, 1.0, 0.02, 8)
    plan = hot.hot_create(n, ld, s, s, 100.0, 0)
    for kern in range(4):
        hot.hot_set_launch(plan, kern, chunks=4, unroll=2, nontemporal=1)

    def fresh():
        return {k: _dev(st[k], offset) for k in names}, _dev(np.full((s, ld), 7.0, np.float32), offset), \
            torch.full((1,), -1.0, dtype=torch.float64, device=DEV)

    def same(a, b):
        for k in names:
            assert torch.equal(a[0][k], b[0][k]), k
        assert torch.equal(a[1], b[1]) and a[2].item() == b[2].item()

    for gen in (False, True):
        # backward + Adam
        a, b = fresh(), fresh()
        gm, gs = _dev(np.zeros(n), offset), _dev(np.zeros(n), offset)
        if gen:
            hot.hot_backward_rng(plan, rng, a[0]["mu"], a[0]["sigma"], G_d, gm, gs)
        else:
            hot.hot_backward(plan, a[0]["mu"], a[0]["sigma"], eps_d, G_d, gm, gs)
        hot.hot_adam_step(params, a[0]["mu"], a[0]["sigma"], gm, gs, *[a[0][k] for k in names[2:]])
        hot.hot_backward_adam(plan, rng if gen else None, params, b[0]["mu"], b[0]["sigma"], None if gen else eps_d, G_d,
                              *[b[0][k] for k in names[2:]])
        torch.cuda.synchronize()
        same(a, b)
        # Adam + forward
        a, b = fresh(), fresh()
        hot.hot_adam_step(params, a[0]["mu"], a[0]["sigma"], gmu_in, gsg_in, *[a[0][k] for k in names[2:]])
        if gen:
            hot.hot_forward_rng(plan, nxt, a[0]["mu"], a[0]["sigma"], a[1], a[2])
        else:
            hot.hot_forward(plan, a[0]["mu"], a[0]["sigma"], eps_d, a[1], a[2])
        hot.hot_adam_forward(plan, nxt if gen else None, params, b[0]["mu"], b[0]["sigma"], gmu_in, gsg_in,
                             *[b[0][k] for k in names[2:]], None if gen else eps_d, b[1], b[2])
        torch.cuda.synchronize()
        same(a, b)
    # backward + Adam + forward
    a, b = fresh(), fresh()
    hot.hot_backward_adam(plan, rng, params, a[0]["mu"], a[0]["sigma"], None, G_d, *[a[0][k] for k in names[2:]])
    hot.hot_forward_rng(plan, nxt, a[0]["mu"], a[0]["sigma"], a[1], a[2])
    hot.hot_backward_adam_forward(plan, rng, nxt, params, b[0]["mu"], b[0]["sigma"], G_d, *[b[0][k] for k in names[2:]], b[1], b[2])
    torch.cuda.synchronize()
    same(a, b)
    if ld > n:
        assert torch.all(b[1][:, n:] == 7.0), "w padding written"
    hot.hot_destroy(plan)


@pytest.mark.parametrize("n,s", [(30_011, 4), (400_003, 2)])
def test_fused_step_replayed_from_a_hip_graph(hot, n, s):
    """hot_backward_adam_forward neither allocates nor synchronises, so a stream capture takes it.  The call
    updates its state in place: three replays of the captured step, with eager work and synchronisations
    between them, must walk through the same three states as three eager calls, bit for bit (parameters,
    moments, w and KL; the smaller case lets the kernel add the KL partials itself, the larger one uses the
    finish kernel)."""
    print("case fused step under a HIP graph", n, s, flush=True)
    r = np.random.default_rng(n + s)
    names = ("mu", "sigma", "m_mu", "v_mu", "m_sigma", "v_sigma")
    st = {"mu": r.normal(size=n), "sigma": r.uniform(0.05, 1.0, size=n), "m_mu": r.normal(size=n) * 0.1,
          "v_mu": r.uniform(0, 1, size=n) * 0.01, "m_sigma": r.normal(size=n) * 0.1, "v_sigma": r.uniform(0, 1, size=n) * 0.01}
    G = torch.from_numpy(r.normal(size=(s, n)).astype(np.float32)).to(DEV)
    rng, rng_next = hot.hot_rng(seed=9, step=3, first_sample=0), hot.hot_rng(seed=9, step=4, first_sample=0)
    params = hot.hot_adam(1e-2, 0.9, 0.999, 1e-8, 1.0, 0.01, 4)
    plan = hot.hot_create(n, n, s, s, 300.0, 0)

    def fresh():
        d = {k: torch.from_numpy(st[k].astype(np.float32)).to(DEV) for k in names}
        d["w"] = torch.zeros(s, n, device=DEV)
        d["kl"] = torch.zeros(1, dtype=torch.float64, device=DEV)
        return d

    def step(d):
        hot.hot_backward_adam_forward(plan, rng, rng_next, params, d["mu"], d["sigma"], G, d["m_mu"], d["v_mu"],
                                      d["m_sigma"], d["v_sigma"], d["w"], d["kl"])

    eager, trail = fresh(), []
    for _ in range(3):
        step(eager)
        torch.cuda.synchronize()
        trail.append({k: v.clone() for k, v in eager.items()})
    assert not torch.equal(trail[0]["mu"], trail[1]["mu"])          # the state does move

    warm = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(warm)                              # warm-up on the capture stream, on buffers of its own
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    held = fresh()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(held)
    for k, v in fresh().items():                # capture does not run the kernels; start from the initial state anyway
        held[k].copy_(v)
    for rep in range(3):
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in held:
            assert torch.equal(held[k], trail[rep][k]), (rep, k)
        scratch = torch.randn(1000, device=DEV).sum().item()       # eager work between replays
        assert scratch == scratch
    hot.hot_destroy(plan)


def test_fused_backward_adam_forward_errors(hot):
    n = 64
    t = [torch.zeros(n, device=DEV) for _ in range(6)]
    G, w = torch.zeros(2, n, device=DEV), torch.zeros(2, n, device=DEV)
    params = hot.hot_adam(1e-3, 0.9, 0.999, 1e-8, 1.0, 0.0, 1)
    rng, nxt = hot.hot_rng(seed=1, step=0, first_sample=0), hot.hot_rng(seed=1, step=1, first_sample=0)
    shared = hot.hot_create(n, n, 2, 4, 1.0, 0)            # only half of the samples are local
    with pytest.raises(hot.HotError):
        hot.hot_backward_adam_forward(shared, rng, nxt, params, t[0], t[1], G, *t[2:], w)
    hot.hot_destroy(shared)
    plan = hot.hot_create(n, n, 2, 2, 1.0, 0)
    with pytest.raises(hot.HotError):
        hot.hot_backward_adam_forward(plan, rng, nxt, params, t[0], t[1], G, *t[2:], G)      # w must not be grad_w
    with pytest.raises(hot.HotError):
        hot.hot_backward_adam_forward(plan, rng, hot.hot_rng(seed=1, step=1, first_sample=2 ** 32 - 1), params, t[0], t[1], G, *t[2:], w)
    hot.hot_backward_adam_forward(plan, rng, nxt, params, t[0], t[1], G, *t[2:], w)
    torch.cuda.synchronize()
    hot.hot_destroy(plan)


def test_fused_backward_adam_errors(hot):
    n = 64
    t = [torch.zeros(n, device=DEV) for _ in range(6)]
    G = torch.zeros(2, n, device=DEV)
    params = hot.hot_adam(1e-3, 0.9, 0.999, 1e-8, 1.0, 0.0, 1)
    rng = hot.hot_rng(seed=1, step=0, first_sample=0)
    shared = hot.hot_create(n, n, 2, 4, 1.0, 0)            # only half of the samples are local
    with pytest.raises(hot.HotError):
        hot.hot_backward_adam(shared, rng, params, t[0], t[1], None, G, *t[2:])
    hot.hot_destroy(shared)
    plan = hot.hot_create(n, n, 2, 2, 1.0, 0)
    with pytest.raises(ValueError):
        hot.hot_backward_adam(plan, rng, params, t[0], t[1], G.clone(), G, *t[2:])       # both sources of eps
    with pytest.raises(hot.HotError):
        hot.hot_backward_adam(plan, rng, hot.hot_adam(1e-3, 0.9, 0.999, 1e-8, 1.0, 0.0, 0), t[0], t[1], None, G, *t[2:])
    hot.hot_destroy(plan)
